// Grouped bf16 GEMM on MFMA for expert blocks with many rows per expert (prefill-sized batches).
// FaaSMoE Sec. 3: an expert block holds several experts and computes on the tokens handed to it;
// Sec. 4.1: the tokens of one block arrive as one batch.  Here a block is an expert range
// [lo,hi) and its batch is a contiguous row range, cut per expert by expert_offsets.
//
// Two instantiations of one kernel:
//   gate/up : h[r, n]  = silu(<A[r,:], Wg[e][n,:]>) * <A[r,:], Wu[e][n,:]>      (A = Xp, Kdim = H)
//   down    : Yp[r, n] = <A[r,:], Wd[e][n,:]>                                   (A = h,  Kdim = I)
// Both operands are K-contiguous, so token rows and weight rows are staged the same way.
//
// Work decomposition.  A tile is BM token rows of ONE expert by BN weight rows (gate/up: BN/2 gate
// rows and the matching BN/2 up rows, so the SwiGLU product is formed in registers).  The number
// of tiles depends on expert_offsets, which only the device knows: the kernel is persistent, every
// workgroup first builds the per-expert tile prefix in LDS and then walks tile indices with a
// fixed stride, so there is no host synchronisation and no atomic.  Workgroup b runs on XCD
// b mod 8; the index walk hands each XCD runs of consecutive tiles that share weight and token
// panels, so they meet in that XCD's L2.
//
// Inside a tile: 4 waves, K steps of 64 through a double-buffered LDS stage (16-byte chunks,
// chunk index xor row&7 so the MFMA operand reads are bank-conflict free), global loads of step
// k+1 are in flight while step k is multiplied.  MFMA 32x32x16 bf16 with the WEIGHT rows as the
// first operand and the TOKEN rows as the second: a lane then owns 4 consecutive output columns
// of one token row per accumulator quad, which makes the bf16 stores 8 bytes wide.
// Rows past the end of an expert are clamped on load and masked on store; 32-row token blocks
// that are entirely past the end are skipped.
#include "common.h"

namespace moe {

template <int BM, int BN, int WAVES_M, int WAVES_N, bool GATEUP>
struct TileShape {
  static constexpr int BK = 64;
  static constexpr int ROWB = BK * 2;             // bytes per staged row
  static constexpr int WTM = BM / WAVES_M;        // token rows per wave
  static constexpr int WTN = BN / WAVES_N;        // weight rows per wave
  static constexpr int TB = WTM / 32;             // 32-row token blocks per wave
  static constexpr int NB = WTN / 32;             // 32-row weight blocks per wave
  static constexpr int NBH = GATEUP ? NB / 2 : NB;
  static constexpr int LA = BM / 32;              // 16-byte global loads per thread and K step (tokens)
  static constexpr int LB = BN / 32;              // (weights)
  static constexpr int STAGE = (BM + BN) * ROWB;  // bytes per LDS stage
  static constexpr int NOUT = GATEUP ? BN / 2 : BN;  // output columns per tile
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of 32x32 blocks");
  static_assert(!GATEUP || NB % 2 == 0, "gate and up blocks come in pairs");
};

constexpr int TILE_EMAX = 256;
constexpr int TILE_GM = 4;   // token tiles per locality group

template <int BM, int BN, int WAVES_M, int WAVES_N, bool GATEUP>
__global__ __launch_bounds__(256, 1) void expert_tile_kernel(GemmArgs a) {
  using S = TileShape<BM, BN, WAVES_M, WAVES_N, GATEUP>;
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_pref[TILE_EMAX + 1];
  __shared__ int s_rb[TILE_EMAX + 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int nexp = a.offsets ? a.hi - a.lo : 1;

  // per-expert row begin and number of token tiles -> exclusive prefix in LDS
  for (int i = tid; i <= nexp; i += 256) s_rb[i] = a.offsets ? a.offsets[a.lo + i] : (i == 0 ? 0 : a.rows_fixed);
  __syncthreads();
  if (wave == 0) {
    int v[4], sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane * 4 + i;
      v[i] = e < nexp ? (s_rb[e + 1] - s_rb[e] + BM - 1) / BM : 0;
      sum += v[i];
    }
    int incl = sum;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const int o = __shfl_up(incl, s, WAVE);
      if (lane >= s) incl += o;
    }
    int base = incl - sum;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane * 4 + i;
      if (e < nexp) s_pref[e] = base;
      base += v[i];
    }
    if (lane == 63) s_pref[nexp] = incl;
  }
  __syncthreads();
  const int totalM = s_pref[nexp];
  const int NT = (a.N + S::NOUT - 1) / S::NOUT;
  const int Kdim = a.Kdim;
  const int nk = Kdim / S::BK;
  const int groupTiles = TILE_GM * NT;
  const int Lend = ((totalM + TILE_GM - 1) / TILE_GM) * groupTiles;

  // staging assignment of this thread: chunk lchk of rows lrow + 32*i
  const int lrow = tid >> 3, lchk = tid & 7;
  const int lds_w = lrow * S::ROWB + ((lchk ^ (lrow & 7)) << 4);
  const int frag_row = lane & 31;
  const int frag_half = lane >> 5;

  const int G = gridDim.x;
  const bool xcd_walk = (G % 8) == 0;
  for (int it = 0;; ++it) {
    const int L = xcd_walk ? ((it * 8 + (int)(blockIdx.x & 7)) * (G >> 3) + (int)(blockIdx.x >> 3))
                           : (it * G + (int)blockIdx.x);
    if (L >= Lend) break;
    const int grp = L / groupTiles, rem = L - grp * groupTiles;
    const int mrow = grp * TILE_GM + rem % TILE_GM;
    const int nt = rem / TILE_GM;
    if (mrow >= totalM) continue;

    // expert of this token tile: last e with s_pref[e] <= mrow
    int elo = 0, ehi = nexp;
    while (ehi - elo > 1) {
      const int mid = (elo + ehi) >> 1;
      if (s_pref[mid] <= mrow) elo = mid; else ehi = mid;
    }
    const int e = elo;
    const int row0 = s_rb[e] + (mrow - s_pref[e]) * BM;
    const int rowEnd = s_rb[e + 1];
    const int rowsValid = min(BM, rowEnd - row0);
    const int n0 = nt * S::NOUT;
    const int eg = a.offsets ? a.lo + e : 0;

    const bf16_t* Ag = a.A + (size_t)row0 * Kdim;
    const bf16_t* Bg0 = a.B0 + (size_t)eg * a.N * Kdim;
    const bf16_t* Bg1 = GATEUP ? a.B1 + (size_t)eg * a.N * Kdim : nullptr;
    int offA[S::LA], offB[S::LB];
#pragma unroll
    for (int i = 0; i < S::LA; ++i) offA[i] = min(lrow + 32 * i, rowsValid - 1) * Kdim + lchk * 8;
#pragma unroll
    for (int i = 0; i < S::LB; ++i) {
      int r = lrow + 32 * i;
      if (GATEUP && i >= S::LB / 2) r -= BN / 2;   // second half of the staged rows: the up branch
      offB[i] = min(n0 + r, a.N - 1) * Kdim + lchk * 8;
    }
    // 32-row token blocks of this wave that hold at least one valid row
    const int tbValid = min(S::TB, (rowsValid - wm * S::WTM + 31) / 32);

    f32x16 acc[S::NB][S::TB];
#pragma unroll
    for (int nb = 0; nb < S::NB; ++nb)
#pragma unroll
      for (int tb = 0; tb < S::TB; ++tb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nb][tb][i] = 0.0f;

    u32x4 ra[S::LA], rb[S::LB];
    // global -> registers for K step k0 (both panels), and registers -> LDS stage
#define MOE_TILE_GLOAD(k0)                                                                      \
    {                                                                                           \
      _Pragma("unroll") for (int i = 0; i < S::LA; ++i)                                         \
        ra[i] = *reinterpret_cast<const u32x4*>(Ag + offA[i] + (k0));                           \
      _Pragma("unroll") for (int i = 0; i < S::LB; ++i)                                         \
        rb[i] = *reinterpret_cast<const u32x4*>(((GATEUP && i >= S::LB / 2) ? Bg1 : Bg0) + offB[i] + (k0)); \
    }
#define MOE_TILE_LSTORE(stage)                                                                  \
    {                                                                                           \
      unsigned char* As_ = smem + (stage) * S::STAGE;                                           \
      unsigned char* Bs_ = As_ + BM * S::ROWB;                                                  \
      _Pragma("unroll") for (int i = 0; i < S::LA; ++i)                                         \
        *reinterpret_cast<u32x4*>(As_ + lds_w + i * 32 * S::ROWB) = ra[i];                      \
      _Pragma("unroll") for (int i = 0; i < S::LB; ++i)                                         \
        *reinterpret_cast<u32x4*>(Bs_ + lds_w + i * 32 * S::ROWB) = rb[i];                      \
    }

    MOE_TILE_GLOAD(0);
    MOE_TILE_LSTORE(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt & 1;
      const bool more = kt + 1 < nk;
      if (more) MOE_TILE_GLOAD((kt + 1) * S::BK);
      const unsigned char* As = smem + cur * S::STAGE;
      const unsigned char* Bs = As + BM * S::ROWB;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int coff = ((kk * 2 + frag_half) ^ (lane & 7)) << 4;
        bf16x8 fa[S::TB], fb[S::NB];
#pragma unroll
        for (int tb = 0; tb < S::TB; ++tb)
          fa[tb] = as_bf16x8(*reinterpret_cast<const u32x4*>(As + (wm * S::WTM + tb * 32 + frag_row) * S::ROWB + coff));
#pragma unroll
        for (int nb = 0; nb < S::NB; ++nb) {
          const int brow = GATEUP ? ((nb < S::NBH ? 0 : BN / 2) + wn * (S::WTN / 2) + (nb % S::NBH) * 32)
                                  : (wn * S::WTN + nb * 32);
          fb[nb] = as_bf16x8(*reinterpret_cast<const u32x4*>(Bs + (brow + frag_row) * S::ROWB + coff));
        }
#pragma unroll
        for (int tb = 0; tb < S::TB; ++tb) {
          if (tb < tbValid) {
#pragma unroll
            for (int nb = 0; nb < S::NB; ++nb)
              acc[nb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[nb], fa[tb], acc[nb][tb], 0, 0, 0);
          }
        }
      }
      if (more) MOE_TILE_LSTORE(cur ^ 1);
      __syncthreads();
    }
#undef MOE_TILE_GLOAD
#undef MOE_TILE_LSTORE

    // epilogue: accumulator element i of block (nb, tb) is output column
    // 8*(i/4) + 4*(lane/32) + i%4 of the block, token row lane%32.
#pragma unroll
    for (int tb = 0; tb < S::TB; ++tb) {
      const int m = row0 + wm * S::WTM + tb * 32 + frag_row;
      if (tb < tbValid && m < rowEnd) {
        bf16_t* crow = a.C + (size_t)m * a.N;
#pragma unroll
        for (int nb = 0; nb < S::NBH; ++nb) {
          const int nbase = n0 + (GATEUP ? wn * (S::WTN / 2) : wn * S::WTN) + nb * 32 + 4 * frag_half;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = nbase + 8 * q;
            if (n < a.N) {
              float v[4];
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                if (GATEUP) {
                  const float g = acc[nb][tb][4 * q + j];
                  const float u = acc[nb + S::NBH][tb][4 * q + j];
                  v[j] = g / (1.0f + __expf(-g)) * u;
                } else {
                  v[j] = acc[nb][tb][4 * q + j];
                }
              }
              uint2 o;
              o.x = pack_bf16x2(v[0], v[1]);
              o.y = pack_bf16x2(v[2], v[3]);
              *reinterpret_cast<uint2*>(crow + n) = o;
            }
          }
        }
      }
    }
  }
}

static int num_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    cus = n;
  }
  return cus;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool GATEUP>
static int launch_tile_t(const GemmArgs& a, hipStream_t st) {
  using S = TileShape<BM, BN, WAVES_M, WAVES_N, GATEUP>;
  auto kern = expert_tile_kernel<BM, BN, WAVES_M, WAVES_N, GATEUP>;
  static bool attr_set = false;
  const int lds = 2 * S::STAGE;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return -4;
    attr_set = true;
  }
  const int nexp = a.offsets ? a.hi - a.lo : 1;
  const int NT = (a.N + S::NOUT - 1) / S::NOUT;
  const long mt_bound = (long)a.rows_total / BM + nexp;
  const long bound = ((mt_bound + TILE_GM - 1) / TILE_GM) * TILE_GM * NT;
  int grid = (int)(bound < (long)num_cus() ? bound : (long)num_cus());
  if (grid <= 0) return 0;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int launch_tile_gateup(const GemmArgs& a, int tile_rows, hipStream_t st) {
  if (tile_rows >= 256) return launch_tile_t<256, 256, 2, 2, true>(a, st);
  return launch_tile_t<128, 256, 1, 4, true>(a, st);
}
int launch_tile_down(const GemmArgs& a, int tile_rows, hipStream_t st) {
  if (tile_rows >= 256) return launch_tile_t<256, 256, 2, 2, false>(a, st);
  return launch_tile_t<128, 256, 1, 4, false>(a, st);
}

}  // namespace moe
