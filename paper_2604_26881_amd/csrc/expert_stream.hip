// Weight-streaming grouped GEMM for expert blocks with FEW rows per expert (decode-sized batches).
// FaaSMoE Sec. 3: an expert block computes statelessly on the tokens it is handed; with one
// token per request an expert sees a handful of rows, so the work is reading the expert's weights
// once from HBM.  Experts without rows return at once: their weights are never touched, which is
// the device-side form of the paper's "only activated experts cost anything".
//
//   gate/up : h[r, n]  = silu(<A[r,:], Wg[e][n,:]>) * <A[r,:], Wu[e][n,:]>
//   down    : Yp[r, n] = <A[r,:], Wd[e][n,:]>
//
// No LDS staging: a wave owns 16 weight rows (and the 16 matching rows of the up branch) and
// keeps up to MT token tiles of 16 rows in MFMA accumulators, so every weight byte is loaded
// exactly once per pass and used for all the expert's rows.  MFMA 16x16x32 bf16, weights as the
// first operand and tokens as the second: lane (l%16, l/16) supplies row l%16 and the k-group
// l/16.  The k index inside an MFMA is only a label shared by both operands, so per 64-wide K step
// a lane loads 32 contiguous bytes (k = 16*(l/16) .. +15) and feeds the two halves to two MFMAs:
// the four lanes of a row then cover one full 128-byte line per load pair.
// Loads for the next K step are issued before the MFMAs of the current one (two register sets).
//
// The 4 waves of a workgroup are arranged NBW x MS x KSP (product 4):
//   NBW  neighbouring 16-row weight blocks, one per wave (plenty of blocks: routed experts);
//   MS   waves that share one weight block and split the expert's token tiles (many rows, one
//        expert: the shared expert at decode sizes; the block's weights come from HBM once and
//        from the L1/L2 for the other waves);
//   KSP  waves that split the K steps of one block (step s goes to wave s mod KSP); their partial
//        sums are added in wave order through LDS (too few blocks to fill the chip otherwise).
#include "common.h"

namespace moe {

template <int MT, bool GATEUP>
struct StreamFrag {
  u32x4 wg[2][2];          // [k-step within the pair][first/second 16 bytes]
  u32x4 wu[2][2];
  u32x4 x[MT][2][2];
};

template <int MT, int NBW, int MS, int KSP, bool GATEUP>
__global__ __launch_bounds__(256) void expert_stream_kernel(GemmArgs a) {
  static_assert(NBW * MS * KSP == 4, "four waves per workgroup");
  constexpr int NBR = GATEUP ? 2 : 1;
  __shared__ float s_red[KSP > 1 ? 4 : 1][KSP > 1 ? MT * NBR * 4 : 1][64];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nb_w = wave % NBW, ms_w = (wave / NBW) % MS, ks_w = wave / (NBW * MS);
  const int y = blockIdx.y;
  const int eg = a.offsets ? (a.ids ? a.ids[a.lo + y] : a.lo + y) : 0;
  const int rb = a.offsets ? a.offsets[eg] : 0;
  const int re = a.offsets ? a.offsets[eg + 1] : a.rows_fixed;
  const int Me = re - rb;
  if (Me <= 0) return;                         // whole workgroup: no barrier is skipped by part of it

  const int N = a.N, Kdim = a.Kdim;
  const int nb = (int)blockIdx.x * NBW + nb_w;
  const int n0 = nb * 16;
  if (KSP == 1 && n0 >= N) return;             // without a K split there is no barrier
  const int kg = lane >> 4, r16 = lane & 15;
  const size_t wrow = (size_t)eg * N + min(n0 + r16, N - 1);
  const bf16_t* wg = a.B0 + wrow * Kdim + 16 * kg;
  const bf16_t* wu = GATEUP ? a.B1 + wrow * Kdim + 16 * kg : nullptr;

  const int npairs = (Kdim + 127) / 128;       // K steps of 64 come in pairs
  const int p_begin = ks_w;
  const int p_stride = KSP;

  for (int m0 = 0; m0 < Me; m0 += 16 * MT * MS) {
    const int mw = m0 + ms_w * 16 * MT;        // first row of this wave's token tiles
    const int mtv = max(0, min(MT, (Me - mw + 15) / 16));
    const bf16_t* xr[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int r = rb + min(mw + mt * 16 + r16, Me - 1);
      xr[mt] = a.A + (size_t)(a.gather ? a.gather[r] / a.gather_div : r) * Kdim + 16 * kg;
    }

    f32x4 accg[MT], accu[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      accg[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      accu[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    auto load = [&](StreamFrag<MT, GATEUP>& f, int p) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = p * 128 + h * 64;
        if (k < Kdim) {
          f.wg[h][0] = *reinterpret_cast<const u32x4*>(wg + k);
          f.wg[h][1] = *reinterpret_cast<const u32x4*>(wg + k + 8);
          if (GATEUP) {
            f.wu[h][0] = *reinterpret_cast<const u32x4*>(wu + k);
            f.wu[h][1] = *reinterpret_cast<const u32x4*>(wu + k + 8);
          }
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            if (mt < mtv) {
              f.x[mt][h][0] = *reinterpret_cast<const u32x4*>(xr[mt] + k);
              f.x[mt][h][1] = *reinterpret_cast<const u32x4*>(xr[mt] + k + 8);
            }
          }
        }
      }
    };
    auto mma = [&](const StreamFrag<MT, GATEUP>& f, int p) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = p * 128 + h * 64;
        if (k < Kdim) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            if (mt < mtv) {
#pragma unroll
              for (int j = 0; j < 2; ++j) {
                accg[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(f.wg[h][j]), as_bf16x8(f.x[mt][h][j]),
                                                                    accg[mt], 0, 0, 0);
                if (GATEUP)
                  accu[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(f.wu[h][j]), as_bf16x8(f.x[mt][h][j]),
                                                                      accu[mt], 0, 0, 0);
              }
            }
          }
        }
      }
    };

    if (mtv > 0) {
      StreamFrag<MT, GATEUP> f0, f1;
      int p = p_begin;
      if (p < npairs) load(f0, p);
      while (p < npairs) {
        const int p1 = p + p_stride, p2 = p + 2 * p_stride;
        if (p1 < npairs) load(f1, p1);
        mma(f0, p);
        if (p1 < npairs) {
          if (p2 < npairs) load(f0, p2);
          mma(f1, p1);
        }
        p = p2;
      }
    }

    // accumulator element j of tile mt: output column n0 + 4*(lane/16) + j, token row lane%16
    auto store_tile = [&](int mt, const f32x4& g, const f32x4& u) {
      const int m = mw + mt * 16 + r16;
      const int n = n0 + 4 * kg;
      if (m < Me && n < N) {
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = GATEUP ? __fdividef(g[j], 1.0f + __expf(-g[j])) * u[j] : g[j];
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]);
        o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>(a.C + (size_t)(rb + m) * N + n) = o;
      }
    };

    if (KSP == 1) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        if (mt < mtv) store_tile(mt, accg[mt], accu[mt]);
    } else {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          s_red[wave][(mt * NBR + 0) * 4 + j][lane] = accg[mt][j];
          if (GATEUP) s_red[wave][(mt * NBR + NBR - 1) * 4 + j][lane] = accu[mt][j];
        }
      }
      __syncthreads();
      // the KSP waves of one (weight block, token split) add up in wave order; tile mt is finished
      // by the wave of that group whose K-split index is mt % KSP
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        if (mt < mtv && (mt % KSP) == ks_w) {
          f32x4 g, u;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float sg_ = 0.f, su_ = 0.f;
#pragma unroll
            for (int w = 0; w < KSP; ++w) {             // fixed order of the K slices
              const int src = nb_w + NBW * (ms_w + MS * w);
              sg_ += s_red[src][(mt * NBR + 0) * 4 + j][lane];
              if (GATEUP) su_ += s_red[src][(mt * NBR + NBR - 1) * 4 + j][lane];
            }
            g[j] = sg_;
            u[j] = su_;
          }
          store_tile(mt, g, u);
        }
      }
      __syncthreads();                                 // s_red is reused by the next pass over rows
    }
  }
}

template <int MT, int NBW, int MS, int KSP, bool GATEUP>
static int launch_stream_t(const GemmArgs& a, hipStream_t st) {
  const int nexp = a.offsets ? a.hi - a.lo : 1;
  const int nblocks = (a.N + 15) / 16;
  const int gx = (nblocks + NBW - 1) / NBW;
  if (gx <= 0 || nexp <= 0) return 0;
  hipLaunchKernelGGL((expert_stream_kernel<MT, NBW, MS, KSP, GATEUP>), dim3(gx, nexp), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// mode: 1 = one weight block per wave; 4 = the waves split K; 5 = the waves split the token tiles;
//       6 = two-way token split times two-way K split.
template <bool GATEUP>
static int launch_stream_any(const GemmArgs& a, int mode, hipStream_t st) {
  // token tiles held in registers by a wave.  With expert_offsets the rows per expert vary around
  // the mean: leave room for twice the mean.
  const int ms = mode == 5 ? 4 : (mode == 6 ? 2 : 1);
  const int rows = a.offsets ? 2 * a.mean_rows : a.rows_fixed;
  const int want = (rows + 16 * ms - 1) / (16 * ms);
  const int mt = want <= 1 ? 1 : (want <= 2 ? 2 : 4);
  switch (mode) {
    case 4:
      if (mt == 1) return launch_stream_t<1, 1, 1, 4, GATEUP>(a, st);
      if (mt == 2) return launch_stream_t<2, 1, 1, 4, GATEUP>(a, st);
      return launch_stream_t<4, 1, 1, 4, GATEUP>(a, st);
    case 5:
      if (mt == 1) return launch_stream_t<1, 1, 4, 1, GATEUP>(a, st);
      if (mt == 2) return launch_stream_t<2, 1, 4, 1, GATEUP>(a, st);
      return launch_stream_t<4, 1, 4, 1, GATEUP>(a, st);
    case 6:
      if (mt == 1) return launch_stream_t<1, 1, 2, 2, GATEUP>(a, st);
      if (mt == 2) return launch_stream_t<2, 1, 2, 2, GATEUP>(a, st);
      return launch_stream_t<4, 1, 2, 2, GATEUP>(a, st);
    default:
      if (mt == 1) return launch_stream_t<1, 4, 1, 1, GATEUP>(a, st);
      if (mt == 2) return launch_stream_t<2, 4, 1, 1, GATEUP>(a, st);
      return launch_stream_t<4, 4, 1, 1, GATEUP>(a, st);
  }
}

int launch_stream_gateup(const GemmArgs& a, int mode, hipStream_t st) { return launch_stream_any<true>(a, mode, st); }
int launch_stream_down(const GemmArgs& a, int mode, hipStream_t st) { return launch_stream_any<false>(a, mode, st); }

}  // namespace moe
