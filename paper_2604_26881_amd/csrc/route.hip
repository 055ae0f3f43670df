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

template <int CTRL, int BMASK>
__device__ __forceinline__ float dpp_banks(float keep, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(keep), __float_as_int(v), CTRL, 0xF, BMASK, false));
}
// The same fold for NV values at once, transposed: at strides 1 and 2 a lane keeps only the value
// its low lane bits select and hands the other one to its partner, so the number of values halves
// per step while every addition still pairs the two numbers the butterfly pairs (lane l and lane
// l xor stride of one value).  Afterwards c[j] in lane l belongs to value 4j + (l & 3); strides 4
// and 8 need the true xor partner now (row shifts by 4 split over the lane banks, row rotate by
// 8).  On return c[j] holds the sum over the lane's row of 16; the strides 16 and 32, which pair
// rows (0,1), (2,3) and then the two results, are left to the reader of the four row sums.
template <int NV>
__device__ __forceinline__ void fold_rows(const float (&a)[NV], float (&c)[NV / 4], int lane) {
  static_assert(NV >= 4 && (NV & (NV - 1)) == 0, "power of two");
  const bool o1 = lane & 1, o2 = lane & 2;
  float b[NV / 2];
#pragma unroll
  for (int j = 0; j < NV / 2; ++j) {
    const float keep = o1 ? a[2 * j + 1] : a[2 * j], send = o1 ? a[2 * j] : a[2 * j + 1];
    b[j] = keep + dpp_or<0xB1, 0xF>(0.0f, send);                       // stride 1
  }
#pragma unroll
  for (int j = 0; j < NV / 4; ++j) {
    const float keep = o2 ? b[2 * j + 1] : b[2 * j], send = o2 ? b[2 * j] : b[2 * j + 1];
    c[j] = keep + dpp_or<0x4E, 0xF>(0.0f, send);                       // stride 2
  }
#pragma unroll
  for (int j = 0; j < NV / 4; ++j) {
    float t = dpp_banks<0x104, 0x5>(0.0f, c[j]);                       // row_shl:4 -> lanes with bit 2 clear read lane + 4
    t = dpp_banks<0x114, 0xA>(t, c[j]);                                // row_shr:4 -> lanes with bit 2 set read lane - 4
    c[j] = c[j] + t;                                                   // stride 4
    c[j] = c[j] + dpp_or<0x128, 0xF>(0.0f, c[j]);                      // row_ror:8 : stride 8
  }
}

__device__ __forceinline__ void widen8(u32x4 v, float* f) {
  f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
  f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

// Softmax and top-k of one token by one wave: lane j holds the logits of experts j, j+64, j+128,
// j+192 (-inf beyond E).  K rounds of wave-wide argmax (a max fold, then ballots over the lanes
// that hold the maximum: the lowest expert id wins); lane j < K writes the j-th choice.
__device__ __forceinline__ void softmax_topk(const float (&l)[4], int lane, int E, int K, int renorm,
                                             int32_t* __restrict__ ids_t, float* __restrict__ w_t) {
  bool taken[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) taken[i] = lane + 64 * i >= E;
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
    ids_t[lane] = my_id;
    w_t[lane] = my_w;
  }
}

// Few tokens: the NW waves of a workgroup share TOK tokens and split the experts.
// FULL: H == 512 * C, so no lane is beyond the row and the loads carry no predicate.
// Bias row of token t.  With segment bounds (seg[0] = 0 < ... , n_seg + 1 ascending entries) token
// t of segment s (seg[s] <= t < seg[s+1]; tokens at or past seg[n_seg] count to the last one) takes
// row s of bias [n_seg, E]; without them every token takes the one row.  t is uniform in the wave.
__device__ __forceinline__ const float* bias_row(const float* bias, const int32_t* seg, int n_seg, int t, int E) {
  if (bias == nullptr || seg == nullptr) return bias;
  int s = 0, hi = n_seg - 1;       // last s with seg[s] <= t (s = 0 when there is none), by bisection
  while (s < hi) {
    const int mid = (s + hi + 1) >> 1;
    if (t >= seg[mid]) s = mid; else hi = mid - 1;
  }
  return bias + (size_t)s * E;
}

template <int C, int TOK, int EB, int NW, bool FULL>
__global__ __launch_bounds__(NW * 64) void route_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wr,
                                                        const float* __restrict__ bias_rows,
                                                        const int32_t* __restrict__ seg, int n_seg, int T, int H,
                                                        int E, int K, int renorm, int32_t* __restrict__ ids,
                                                        float* __restrict__ w) {
  static_assert(TOK == 1, "one bias row per workgroup");
  __shared__ float s_logit[TOK][ROUTE_EMAX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * TOK;
  const float* bias = bias_row(bias_rows, seg, n_seg, t0, E);

  // token rows -> fp32 registers (zero beyond H or T; a zero product leaves a partial sum unchanged)
  float xf[TOK][C][8];
#pragma unroll
  for (int tk = 0; tk < TOK; ++tk) {
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const int h = 512 * c + 8 * lane;
      u32x4 v = {0u, 0u, 0u, 0u};
      if ((FULL || h < H) && t0 + tk < T) v = *reinterpret_cast<const u32x4*>(x + (size_t)(t0 + tk) * H + h);
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
        if (FULL) {
          wr[i][c] = *reinterpret_cast<const u32x4*>(Wr + (size_t)e * H + h);
        } else {
          wr[i][c] = u32x4{0u, 0u, 0u, 0u};
          if (h < H) wr[i][c] = *reinterpret_cast<const u32x4*>(Wr + (size_t)e * H + h);
        }
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
          if (lane == 0) s_logit[tk][e] = r;
        }
      }
    }
  };
  {
    constexpr int STEP = NW * EB;
    u32x4 wrA[EB][C], wrB[EB][C];
    int e0 = wave * EB;
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

  for (int tk = wave; tk < TOK; tk += NW) {
    const int t = t0 + tk;
    if (t >= T) break;
    float l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      l[i] = e < E ? s_logit[tk][e] : -INFINITY;
    }
    softmax_topk(l, lane, E, K, renorm, ids + (size_t)t * K, w + (size_t)t * K);
  }
}

// Many tokens: each of the four waves keeps its own TOK tokens and walks all experts EB at a time
// (the waves read the same router rows at about the same time, so they reach L2 once per
// workgroup).  The EB * TOK lane sums of a batch are folded together (fold_rows); the four row sums
// of every logit go to LDS as one float4, and the lane that later owns the expert finishes the fold:
// strides 16 and 32 pair rows (0,1), (2,3) and then the two results.  Dynamic LDS:
// 4 * TOK * EP float4, EP = E rounded up to a multiple of EB (the rows of a ragged last batch are
// clamped copies of row E-1; their sums land in the padding and are never read).
template <int C, int TOK, int EB, bool FULL>
__global__ __launch_bounds__(256) void route_many_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wr,
                                                         const float* __restrict__ bias_rows,
                                                         const int32_t* __restrict__ seg, int n_seg, int T, int H,
                                                         int E, int EP, int K, int renorm,
                                                         int32_t* __restrict__ ids, float* __restrict__ w) {
  constexpr int NW = 4, WTOK = NW * TOK, NV = EB * TOK, NJ = NV / 4;
  extern __shared__ float4 s_rows[];   // [WTOK][EP] : row sums 0..3 of a logit
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * WTOK + wave * TOK;

  float xf[TOK][C][8];
#pragma unroll
  for (int tk = 0; tk < TOK; ++tk) {
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const int h = 512 * c + 8 * lane;
      u32x4 v = {0u, 0u, 0u, 0u};
      if ((FULL || h < H) && t0 + tk < T) v = *reinterpret_cast<const u32x4*>(x + (size_t)(t0 + tk) * H + h);
      widen8(v, xf[tk][c]);
    }
  }

  // After fold_rows, value 4j + (lane & 3) = i * TOK + tk of the batch sits in c[j]; the lanes
  // 0..3 of every row of 16 store it as component (lane >> 4) of the float4 of (token tk, expert e0 + i).
  int slot[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int v = 4 * j + (lane & 3);
    slot[j] = ((wave * TOK + v % TOK) * EP + v / TOK) * 4 + (lane >> 4);
  }
  const bool writer = (lane & 12) == 0;
  float* s_flat = reinterpret_cast<float*>(s_rows);

  auto load_batch = [&](u32x4 (&wr)[EB][C], int e0) {
#pragma unroll
    for (int i = 0; i < EB; ++i) {
      const int e = min(e0 + i, E - 1);
#pragma unroll
      for (int c = 0; c < C; ++c) {
        const int h = 512 * c + 8 * lane;
        if (FULL) {
          wr[i][c] = *reinterpret_cast<const u32x4*>(Wr + (size_t)e * H + h);
        } else {
          wr[i][c] = u32x4{0u, 0u, 0u, 0u};
          if (h < H) wr[i][c] = *reinterpret_cast<const u32x4*>(Wr + (size_t)e * H + h);
        }
      }
    }
  };
  auto dot_batch = [&](const u32x4 (&wr)[EB][C], int e0) {
    float a[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) a[v] = 0.0f;
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
          for (int tk = 0; tk < TOK; ++tk) a[i * TOK + tk] = __builtin_fmaf(xf[tk][c][k], wf[i][k], a[i * TOK + tk]);
    }
    float cs[NJ];
    fold_rows<NV>(a, cs, lane);
    if (writer) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) s_flat[slot[j] + e0 * 4] = cs[j];
    }
  };
  {
    u32x4 wrA[EB][C], wrB[EB][C];
    int e0 = 0;
    load_batch(wrA, e0);
    while (e0 < E) {
      const int e1 = e0 + EB, e2 = e0 + 2 * EB;
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
    const float* bias = bias_row(bias_rows, seg, n_seg, t, E);
    float l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      l[i] = -INFINITY;
      if (e < E) {
        const float4 p = s_rows[tk * EP + e];
        float r = (p.x + p.y) + (p.z + p.w);
        if (bias) r = r + bias[e];
        l[i] = r;
      }
    }
    softmax_topk(l, lane, E, K, renorm, ids + (size_t)t * K, w + (size_t)t * K);
  }
}

#define MOE_ROUTE_PARAMS const void* x, const void* Wr, const float* bias, const int32_t* seg, int n_seg, int T, int H, \
                         int E, int K, int renorm, int32_t* ids, float* w, hipStream_t st
#define MOE_ROUTE_ARGS x, Wr, bias, seg, n_seg, T, H, E, K, renorm, ids, w, st

template <int C, int TOK, int EB, int NW>
static int launch_route_t(MOE_ROUTE_PARAMS) {
  const int blocks = (T + TOK - 1) / TOK;
  if (H == 512 * C)
    hipLaunchKernelGGL((route_kernel<C, TOK, EB, NW, true>), dim3(blocks), dim3(NW * 64), 0, st, (const bf16_t*)x,
                       (const bf16_t*)Wr, bias, seg, n_seg, T, H, E, K, renorm, ids, w);
  else
    hipLaunchKernelGGL((route_kernel<C, TOK, EB, NW, false>), dim3(blocks), dim3(NW * 64), 0, st, (const bf16_t*)x,
                       (const bf16_t*)Wr, bias, seg, n_seg, T, H, E, K, renorm, ids, w);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

template <int C, int TOK, int EB>
static int launch_route_many(MOE_ROUTE_PARAMS) {
  constexpr int WTOK = 4 * TOK;
  const int blocks = (T + WTOK - 1) / WTOK;
  const int EP = (E + EB - 1) / EB * EB;
  const size_t lds = (size_t)WTOK * EP * sizeof(float4);   // at most 16 tokens * 256 experts * 16 B = 64 KiB
  if (H == 512 * C)
    hipLaunchKernelGGL((route_many_kernel<C, TOK, EB, true>), dim3(blocks), dim3(256), lds, st, (const bf16_t*)x,
                       (const bf16_t*)Wr, bias, seg, n_seg, T, H, E, EP, K, renorm, ids, w);
  else
    hipLaunchKernelGGL((route_many_kernel<C, TOK, EB, false>), dim3(blocks), dim3(256), lds, st, (const bf16_t*)x,
                       (const bf16_t*)Wr, bias, seg, n_seg, T, H, E, EP, K, renorm, ids, w);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Few tokens: one token per workgroup of 8 waves that split the experts, each wave takes its
// experts in one batch (latency).  From 384 tokens: the same with 4 waves (19 against 22 us at
// T = 512, and with one wave per SIMD the workgroup fits beside a 128-row GEMM tile of another
// stream instead of waiting behind it).  From 1024 tokens: the many-token kernel (throughput).
int launch_route(MOE_ROUTE_PARAMS) {
  const int chunks = (H + 511) / 512;
  const bool many = T >= 1024, mid = T >= 384;
  if (chunks <= 1)
    return many ? launch_route_many<1, 4, 4>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<1, 1, 8, 4>(MOE_ROUTE_ARGS) : launch_route_t<1, 1, 8, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 2)
    return many ? launch_route_many<2, 2, 4>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<2, 1, 8, 4>(MOE_ROUTE_ARGS) : launch_route_t<2, 1, 8, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 4)
    return many ? launch_route_many<4, 2, 2>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<4, 1, 4, 4>(MOE_ROUTE_ARGS) : launch_route_t<4, 1, 4, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 8)
    return many ? launch_route_many<8, 2, 2>(MOE_ROUTE_ARGS)
                : (mid ? launch_route_t<8, 1, 2, 4>(MOE_ROUTE_ARGS) : launch_route_t<8, 1, 2, 8>(MOE_ROUTE_ARGS));
  if (chunks <= 16) return launch_route_t<16, 1, 1, 4>(MOE_ROUTE_ARGS);
  return -2;
}
#undef MOE_ROUTE_ARGS
#undef MOE_ROUTE_PARAMS

}  // namespace moe
