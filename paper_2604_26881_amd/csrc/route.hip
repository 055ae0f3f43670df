// Gating kernel: router logits, softmax and top-k per token (FaaSMoE Sec. 2.1: the gating
// network selects the top-k experts for each token; Sec. 3: it runs in the orchestrator).
//
// A wave keeps TOK token rows in registers as fp32, streams EB router rows per step and forms
// TOK*EB dot products at once; the waves of a workgroup either share the tokens and split the
// experts, or each take their own tokens and all the experts.  The dot products are formed
// (independent accumulator chains) in the fixed order of the interface: lane j owns elements 512*c + 8*j .. +7 of every 512-element chunk c (one 16-byte
// load per chunk) and accumulates them in ascending index by fused multiply-add; the 64 lane sums
// are folded pairwise over lane strides 1, 2, 4, 8, 16, 32.  The fold runs on the VALU with DPP
// lane selects: after the stride-1 and stride-2 steps the four lanes of a quad hold the same
// value, so "the lane at xor 4" may be any lane of the neighbouring quad (row_half_mirror), and
// likewise row_mirror for stride 8 and the row broadcasts for strides 16 and 32; fp32 addition is
// commutative, so every pairing adds the same two numbers as the xor butterfly.  bf16 products
// are exact in fp32, so a CPU evaluation in the same order reproduces the logits bit for bit.
// The logits meet in LDS; then one wave per token runs softmax and K rounds of wave-wide argmax
// (a max fold, then ballots over the lanes that hold the maximum: the lowest expert id wins).
#include "common.h"

namespace moe {

constexpr int ROUTE_EMAX = 256;

template <int CTRL, int RMASK>
__device__ __forceinline__ float dpp_or(float keep, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(keep), __float_as_int(v), CTRL, RMASK, 0xF, false));
}
// Sum of the 64 lane values, pairing lanes at strides 1,2,4,8,16,32; every lane returns the total.
__device__ __forceinline__ float fold_sum(float a) {
  a = a + dpp_or<0xB1, 0xF>(0.0f, a);    // quad_perm [1,0,3,2]  : stride 1
  a = a + dpp_or<0x4E, 0xF>(0.0f, a);    // quad_perm [2,3,0,1]  : stride 2
  a = a + dpp_or<0x141, 0xF>(0.0f, a);   // row_half_mirror      : stride 4
  a = a + dpp_or<0x140, 0xF>(0.0f, a);   // row_mirror           : stride 8
  a = a + dpp_or<0x142, 0xA>(0.0f, a);   // row_bcast15 into rows 1 and 3 : stride 16
  a = a + dpp_or<0x143, 0xC>(0.0f, a);   // row_bcast31 into rows 2 and 3 : stride 32
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), 63));
}
__device__ __forceinline__ float fold_max(float a) {
  a = fmaxf(a, dpp_or<0xB1, 0xF>(a, a));
  a = fmaxf(a, dpp_or<0x4E, 0xF>(a, a));
  a = fmaxf(a, dpp_or<0x141, 0xF>(a, a));
  a = fmaxf(a, dpp_or<0x140, 0xF>(a, a));
  a = fmaxf(a, dpp_or<0x142, 0xA>(a, a));
  a = fmaxf(a, dpp_or<0x143, 0xC>(a, a));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), 63));
}

__device__ __forceinline__ void widen8(u32x4 v, float* f) {
  f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
  f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

template <int C, int TOK, int EB, int NW, bool TSPLIT>
__global__ __launch_bounds__(NW * 64) void route_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wr,
                                                        const float* __restrict__ bias, int T, int H, int E, int K,
                                                        int renorm, int32_t* __restrict__ ids, float* __restrict__ w) {
  constexpr int WTOK = TSPLIT ? NW * TOK : TOK;   // tokens of the workgroup
  __shared__ float s_logit[WTOK][ROUTE_EMAX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // TSPLIT: every wave has its own TOK tokens and walks all experts (the waves read the same router
  // rows at about the same time, so they reach L2 once per workgroup); otherwise the waves share
  // TOK tokens and split the experts.
  const int t0 = blockIdx.x * WTOK + (TSPLIT ? wave * TOK : 0);
  const int lrow = TSPLIT ? wave * TOK : 0;        // first row of this wave in s_logit

  // token rows -> fp32 registers (zero beyond H or T; a zero product leaves a partial sum unchanged)
  float xf[TOK][C][8];
#pragma unroll
  for (int tk = 0; tk < TOK; ++tk) {
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const int h = 512 * c + 8 * lane;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (h < H && t0 + tk < T) v = *reinterpret_cast<const u32x4*>(x + (size_t)(t0 + tk) * H + h);
      widen8(v, xf[tk][c]);
    }
  }

  // router rows EB at a time; the next batch is requested before the current one is multiplied
  auto load_batch = [&](u32x4 (&wr)[EB][C], int e0) {
#pragma unroll
    for (int i = 0; i < EB; ++i) {
      const int e = min(e0 + i, E - 1);
#pragma unroll
      for (int c = 0; c < C; ++c) {
        const int h = 512 * c + 8 * lane;
        wr[i][c] = u32x4{0u, 0u, 0u, 0u};
        if (h < H) wr[i][c] = *reinterpret_cast<const u32x4*>(Wr + (size_t)e * H + h);
      }
    }
  };
  auto dot_batch = [&](const u32x4 (&wr)[EB][C], int e0) {
    float a[EB][TOK];
#pragma unroll
    for (int i = 0; i < EB; ++i)
#pragma unroll
      for (int tk = 0; tk < TOK; ++tk) a[i][tk] = 0.0f;
#pragma unroll
    for (int c = 0; c < C; ++c) {
      float wf[EB][8];
#pragma unroll
      for (int i = 0; i < EB; ++i) widen8(wr[i][c], wf[i]);
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int i = 0; i < EB; ++i)
#pragma unroll
          for (int tk = 0; tk < TOK; ++tk) a[i][tk] = __builtin_fmaf(xf[tk][c][k], wf[i][k], a[i][tk]);
    }
#pragma unroll
    for (int i = 0; i < EB; ++i) {
      const int e = e0 + i;
      if (e < E) {
        const float b = bias ? bias[e] : 0.0f;
#pragma unroll
        for (int tk = 0; tk < TOK; ++tk) {
          float r = fold_sum(a[i][tk]);
          if (bias) r = r + b;
          if (lane == 0) s_logit[lrow + tk][e] = r;
        }
      }
    }
  };
  {
    constexpr int STEP = TSPLIT ? EB : NW * EB;
    u32x4 wrA[EB][C], wrB[EB][C];
    int e0 = TSPLIT ? 0 : wave * EB;
    if (e0 < E) load_batch(wrA, e0);
    while (e0 < E) {
      const int e1 = e0 + STEP, e2 = e0 + 2 * STEP;
      if (e1 < E) load_batch(wrB, e1);
      dot_batch(wrA, e0);
      if (e1 < E) {
        if (e2 < E) load_batch(wrA, e2);
        dot_batch(wrB, e1);
      }
      e0 = e2;
    }
  }
  __syncthreads();

  const int tbase = blockIdx.x * WTOK;
  for (int tk = wave; tk < WTOK; tk += NW) {
    const int t = tbase + tk;
    if (t >= T) break;
    float l[4];
    bool taken[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      l[i] = e < E ? s_logit[tk][e] : -INFINITY;
      taken[i] = e >= E;
    }
    const float m = fold_max(fmaxf(fmaxf(l[0], l[1]), fmaxf(l[2], l[3])));
    float z = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (lane + 64 * i < E) z += expf(l[i] - m);
    const float denom = fold_sum(z);

    int my_id = 0;
    float my_w = 0.0f, run = 0.0f;
    for (int j = 0; j < K; ++j) {
      float bv = -INFINITY;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (!taken[i]) bv = fmaxf(bv, l[i]);
      bv = fold_max(bv);
      // lowest expert id among the untaken experts whose logit equals the maximum (-0 == +0)
      int be = -1;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const unsigned long long hit = __ballot(!taken[i] && l[i] == bv);
        if (be < 0 && hit != 0ull) be = __builtin_ctzll(hit) + 64 * i;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (be == lane + 64 * i) taken[i] = true;
      const float wj = expf(bv - m) / denom;
      run += wj;
      if (lane == j) { my_id = be; my_w = wj; }
    }
    if (renorm) my_w = my_w / run;
    if (lane < K) {
      ids[(size_t)t * K + lane] = my_id;
      w[(size_t)t * K + lane] = my_w;
    }
  }
}

template <int C, int TOK, int EB, int NW, bool TSPLIT = false>
static int launch_route_t(const void* x, const void* Wr, const float* bias, int T, int H, int E, int K, int renorm,
                          int32_t* ids, float* w, hipStream_t st) {
  constexpr int WTOK = TSPLIT ? NW * TOK : TOK;
  const int blocks = (T + WTOK - 1) / WTOK;
  hipLaunchKernelGGL((route_kernel<C, TOK, EB, NW, TSPLIT>), dim3(blocks), dim3(NW * 64), 0, st, (const bf16_t*)x,
                     (const bf16_t*)Wr, bias, T, H, E, K, renorm, ids, w);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Few tokens: one token per workgroup of 8 waves that split the experts, each wave takes its
// experts in one batch (latency).  From 384 tokens: the same with 4 waves (19 against 22 us at
// T = 512, and with one wave per SIMD the workgroup fits beside a 128-row GEMM tile of another
// stream instead of waiting behind it).  From 1024 tokens: 4 waves with two tokens each, every
// wave walks all experts in batches of 4 (throughput; 53 against 61 us at T = 4096 for the same
// waves splitting the experts of two shared tokens).
#define MOE_ROUTE_ARGS x, Wr, bias, T, H, E, K, renorm, ids, w, st
int launch_route(const void* x, const void* Wr, const float* bias, int T, int H, int E, int K, int renorm,
                 int32_t* ids, float* w, hipStream_t st) {
  const int chunks = (H + 511) / 512;
  const bool many = T >= 1024, mid = T >= 384;
  if (chunks <= 1)
    return many ? launch_route_t<1, 4, 4, 4, true>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<1, 1, 8, 4>(MOE_ROUTE_ARGS) : launch_route_t<1, 1, 8, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 2)
    return many ? launch_route_t<2, 2, 4, 4, true>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<2, 1, 8, 4>(MOE_ROUTE_ARGS) : launch_route_t<2, 1, 8, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 4)
    return many ? launch_route_t<4, 2, 4, 4, true>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<4, 1, 4, 4>(MOE_ROUTE_ARGS) : launch_route_t<4, 1, 4, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 8)
    return many ? launch_route_t<8, 2, 2, 4, true>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<8, 1, 2, 4>(MOE_ROUTE_ARGS) : launch_route_t<8, 1, 2, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 16) return launch_route_t<16, 1, 1, 4>(MOE_ROUTE_ARGS);
  return -2;
}
#undef MOE_ROUTE_ARGS

}  // namespace moe
