// Weight-streaming grouped GEMM for expert blocks with FEW rows per expert, weights staged through
// LDS.  FaaSMoE Sec. 3: an expert block computes statelessly on the tokens it is handed; at decode
// sizes an expert sees a handful of rows, so the work is reading its weights once from HBM, and
// experts without rows return at once (only activated experts cost anything).
//
//   gate/up : h[r, n]  = silu(<A[r,:], Wg[e][n,:]>) * <A[r,:], Wu[e][n,:]>
//   down    : Yp[r, n] = <A[r,:], Wd[e][n,:]>
//
// Why LDS: the MFMA 16x16x32 operand layout gives a weight row to only four lanes, so loading the
// operand straight into registers asks memory for 16 rows x 64 bytes (or interleaved 16-byte
// pieces) per instruction.  Measured on a 1 GiB read of 4 KB rows, that request shape reaches
// 5.7-5.9 TB/s, whole 128-byte lines per row (8 lanes per row) reach 6.8 TB/s.  So the weights are
// copied global -> LDS with 8 lanes per row (one full line each, no registers in between) and the
// MFMA operands are read back from LDS in the layout the matrix core wants.
//
// One wave per workgroup, no barrier anywhere: a wave owns two 16-row weight blocks (gate/up: a
// gate block and the matching up block, so SwiGLU is formed in registers; down: two neighbouring
// blocks) and MT tiles of 16 token rows.  Per 64-wide K step it copies 2 x 16 x 128 bytes of
// weights and MT x 16 x 128 bytes of token rows into its own ring of NST LDS stages; NST-1 stages
// are in flight while one is multiplied.  Copies complete in issue order, so "all but the newest
// (NST-2) stages have landed" is a plain s_waitcnt vmcnt(n).  Token rows go through the same ring
// (they come from L2): a register load of them would sit in the same in-order queue behind the
// deep weight prefetch and drain it.  A row's eight 16-byte chunks are stored at slot = chunk xor
// row%8, which keeps the operand reads (16 rows, same chunk) off each other's banks.
// Several such workgroups share a CU (LDS decides how many), so the start-up of one overlaps the
// steady state of the others, and the hardware dispatcher balances the 16-row blocks dynamically.
// An expert with more rows than one pass covers (16 x MT) re-reads its weights once per pass; its
// passes are spread over up to eight workgroups, so that the hot expert of a skewed batch does not
// become one long chain.
#include "common.h"

namespace moe {

template <int MT, int NST>
struct StreamLdsShape {
  static constexpr int WBYTES = 2 * 16 * 128;   // two weight blocks, one K step
  static constexpr int XBYTES = MT * 16 * 128;  // token tiles, one K step
  static constexpr int STAGE = WBYTES + XBYTES;
  static constexpr int NI = 4 + 2 * MT;         // 1 KB copies per stage
  static constexpr int D = NST - 1;             // stages in flight
  static_assert(D >= 1 && D * NI < 64, "the wait counter holds 6 bits");
};

template <int J, int D, int NI, class F>
__device__ __forceinline__ void stream_tail(F&& step) {
  if constexpr (J < D) {
    wait_copies_but<(D - 1 - J) * NI>();
    step(J);
    stream_tail<J + 1, D, NI>(step);
  }
}

template <int MT, bool GATEUP, int NST>
__global__ __launch_bounds__(64) void expert_stream_lds_kernel(GemmArgs a) {
  using S = StreamLdsShape<MT, NST>;
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NPER = GATEUP ? 16 : 32;   // output columns of one item (two 16-row weight blocks)

  const int lane = threadIdx.x;
  const int y = blockIdx.y;
  const int eg = a.offsets ? (a.ids ? a.ids[a.lo + y] : a.lo + y) : 0;
  const int rb = a.offsets ? a.offsets[eg] : 0;
  const int re = a.offsets ? a.offsets[eg + 1] : a.rows_fixed;
  const int Me = re - rb;
  // An expert with more rows than one pass covers takes further passes over its weights.  They are dealt
  // round-robin to the gridDim.z workgroups of this (expert, column block): workgroups without a pass leave
  // at once (they cost nothing measurable), and a hot expert of a skewed batch no longer runs all its passes
  // one after another in one wave while the rest of the chip has finished.
  const int pass_rows = 16 * MT;
  if (Me <= (int)blockIdx.z * pass_rows) return;

  const int N = a.N, Kdim = a.Kdim;
  const int nk = Kdim / 64;
  // The walk over K starts at step `rot` and wraps around.  Thousands of these waves start within a
  // few microseconds of each other; if all began at K step 0 their requests of one moment would sit
  // at the same offset inside the weight rows, which for rows of a power-of-two length (4 KB at
  // K = 2048) lands them in the same memory channels (measured on the decode batch: gate/up 134 us
  // with a common start, 121 us with staggered starts; the 2816-byte rows of the down projection
  // show no difference).  rot depends on the expert and the column block only, so results do not
  // depend on the block cut.
  const int rot = (int)(((unsigned)blockIdx.x * 3u + (unsigned)eg * 5u) % (unsigned)nk);
  // this wave's output columns: rows [n0, n0+16) of both branches (gate/up) or rows [n0, n0+32) (down)
  const int n0 = (int)blockIdx.x * NPER;
  if (n0 >= N) return;
  const unsigned char* W0 = reinterpret_cast<const unsigned char*>(a.B0 + ((size_t)eg * N + n0) * Kdim);
  const unsigned char* W1 = GATEUP ? reinterpret_cast<const unsigned char*>(a.B1 + ((size_t)eg * N + n0) * Kdim)
                                   : W0 + (size_t)16 * Kdim * 2;
  const unsigned char* Ab = reinterpret_cast<const unsigned char*>(a.A);

  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  // copies: lane -> row lane/8 of an 8-row group, slot lane%8 holding chunk slot xor row%8
  const int crow = lane >> 3;
  const int cchunk = (lane & 7) ^ crow;
  uint32_t coffW[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) coffW[i] = (uint32_t)(i * 8 + crow) * (uint32_t)Kdim * 2u + (uint32_t)cchunk * 16u;
  // operand reads: lane -> row lane%16, chunk 4*j + lane/16 for the j-th MFMA of the K step
  const int r16 = lane & 15, q = lane >> 4;
  const int frag_off = r16 * 128;
  const int swz = r16 & 7;

  for (int m0 = (int)blockIdx.z * pass_rows; m0 < Me; m0 += pass_rows * (int)gridDim.z) {
    uint32_t coffX[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int m = min(m0 + mt * 16 + i * 8 + crow, Me - 1);   // rows past the end repeat the last row
        const int arow = a.gather ? a.gather[rb + m] / a.gather_div : rb + m;
        coffX[mt][i] = (uint32_t)arow * (uint32_t)Kdim * 2u + (uint32_t)cchunk * 16u;
      }

    f32x4 acc0[MT], acc1[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      acc0[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      acc1[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // K step s into ring slot `slot`: the weights with the read-once hint, the token rows without
    auto issue = [&](int s, int slot) {
      const uint32_t l = lds0 + (uint32_t)slot * S::STAGE;
      const size_t kb = (size_t)(s + rot >= nk ? s + rot - nk : s + rot) * 128;
      copy_to_lds_16_stream(W0 + kb, coffW[0], l);
      copy_to_lds_16_stream(W0 + kb, coffW[1], l + 1024u);
      copy_to_lds_16_stream(W1 + kb, coffW[0], l + 2048u);
      copy_to_lds_16_stream(W1 + kb, coffW[1], l + 3072u);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        copy_to_lds_16(Ab + kb, coffX[mt][0], l + (uint32_t)S::WBYTES + (uint32_t)mt * 2048u);
        copy_to_lds_16(Ab + kb, coffX[mt][1], l + (uint32_t)S::WBYTES + (uint32_t)mt * 2048u + 1024u);
      }
    };
    // accumulator element j of tile mt: weight row (output column) 4*(lane/16) + j of the block,
    // token row lane%16
    auto store = [&]() {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = m0 + r16 + mt * 16;
        if (m < Me) {
          bf16_t* crow_out = a.C + (size_t)(rb + m) * N + n0 + 4 * q;
          uint2 o;
          if (GATEUP) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = __fdividef(acc0[mt][j], 1.0f + __expf(-acc0[mt][j])) * acc1[mt][j];
            o.x = pack_bf16x2(v[0], v[1]);
            o.y = pack_bf16x2(v[2], v[3]);
            *reinterpret_cast<uint2*>(crow_out) = o;
          } else {
            o.x = pack_bf16x2(acc0[mt][0], acc0[mt][1]);
            o.y = pack_bf16x2(acc0[mt][2], acc0[mt][3]);
            *reinterpret_cast<uint2*>(crow_out) = o;
            o.x = pack_bf16x2(acc1[mt][0], acc1[mt][1]);
            o.y = pack_bf16x2(acc1[mt][2], acc1[mt][3]);
            *reinterpret_cast<uint2*>(crow_out + 16) = o;
          }
        }
      }
    };
    // multiply the stage in `slot`; `then` runs after the operands are in registers and before the
    // MFMAs (the place to reuse the ring slot that was read one step earlier)
    auto consume = [&](int slot, auto&& then) {
      const unsigned char* st = smem + slot * S::STAGE + frag_off;
      u32x4 w0[2], w1[2], xf[MT][2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int c = ((4 * j + q) ^ swz) << 4;
        w0[j] = *reinterpret_cast<const u32x4*>(st + c);
        w1[j] = *reinterpret_cast<const u32x4*>(st + 2048 + c);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) xf[mt][j] = *reinterpret_cast<const u32x4*>(st + S::WBYTES + mt * 2048 + c);
      }
      // the empty asm makes the compiler wait for the LDS reads here: after it the slot may be overwritten
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        asm volatile("" : "+v"(w0[j]));
        asm volatile("" : "+v"(w1[j]));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) asm volatile("" : "+v"(xf[mt][j]));
      }
      then();
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc0[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w0[j]), as_bf16x8(xf[mt][j]), acc0[mt], 0, 0, 0);
          acc1[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w1[j]), as_bf16x8(xf[mt][j]), acc1[mt], 0, 0, 0);
        }
    };

    if (nk > S::D) {
#pragma unroll
      for (int s = 0; s < S::D; ++s) issue(s, s);
      int slot = 0;
      for (int s = 0; s + S::D < nk; ++s) {
        wait_copies_but<(S::D - 1) * S::NI>();          // step s has landed
        const int free_slot = slot == 0 ? NST - 1 : slot - 1;   // read one step ago (or never used yet)
        consume(slot, [&] { issue(s + S::D, free_slot); });
        slot = slot + 1 == NST ? 0 : slot + 1;
      }
      stream_tail<0, S::D, S::NI>([&](int) {
        consume(slot, [] {});
        slot = slot + 1 == NST ? 0 : slot + 1;
      });
    } else {   // fewer K steps than ring stages: one stage at a time
      for (int s = 0; s < nk; ++s) {
        issue(s, 0);
        wait_copies_but<0>();
        consume(0, [] {});
      }
    }
    store();
  }
}

constexpr int STREAM_PASS_GROUPS = 8;

template <int MT, bool GATEUP, int NST>
static int launch_stream_lds_t(const GemmArgs& a, hipStream_t st) {
  using S = StreamLdsShape<MT, NST>;
  static_assert(NST * S::STAGE <= 64 * 1024, "dynamic LDS without an opt-in attribute");
  auto kern = expert_stream_lds_kernel<MT, GATEUP, NST>;
  const int nexp = a.offsets ? a.hi - a.lo : 1;
  const int per = GATEUP ? 16 : 32;
  const int gx = (a.N + per - 1) / per;
  if (gx <= 0 || nexp <= 0) return 0;
  // workgroups per (expert, column block): enough that an expert holding every row of the batch runs at most
  // about two passes per workgroup, at most STREAM_PASS_GROUPS (from layer-wide sizes only; a row's result does
  // not depend on it).  Measured at the Qwen shape: 8 cost nothing on unbiased batches (T = 16 ... 384) and
  // take a batch whose hot expert holds nearly every token from 172 + 96 us to 141 + 73 us at T = 128 and
  // from 250 + 159 to 180 + 98 us at T = 384; 16 and 32 begin to cost the unbiased batches 5 - 20 %.
  const int passes_max = (a.rows_total + 16 * MT - 1) / (16 * MT);
  const int gz = std::max(1, std::min(STREAM_PASS_GROUPS, passes_max / 2));
  hipLaunchKernelGGL(kern, dim3(gx, nexp, gz), dim3(64), NST * S::STAGE, st, a);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Token tiles per pass from layer-wide sizes: with expert_offsets the rows per expert scatter
// around the mean (binomial), one tile of 16 covers nearly all experts up to a mean of 10; an
// expert with more rows takes further passes over its weights.  Ring depths from 2 to 8 stages
// measured the same within noise; 4 leaves room for five to six workgroups per CU.
template <bool GATEUP>
static int launch_stream_lds_any(const GemmArgs& a, hipStream_t st) {
  if (a.N % 32 != 0 || a.Kdim % 64 != 0) return -2;
  const int rows = a.offsets ? a.mean_rows : a.rows_fixed;
  if (rows <= 10) return launch_stream_lds_t<1, GATEUP, 4>(a, st);
  return launch_stream_lds_t<2, GATEUP, 4>(a, st);
}
int launch_stream_lds_gateup(const GemmArgs& a, hipStream_t st) { return launch_stream_lds_any<true>(a, st); }
int launch_stream_lds_down(const GemmArgs& a, hipStream_t st) { return launch_stream_lds_any<false>(a, st); }

}  // namespace moe
