// Gating kernel: router logits, softmax and top-k per token (FaaSMoE Sec. 2.1: the gating
// network selects the top-k experts for each token; Sec. 3: it runs in the orchestrator).
//
// One workgroup of four waves serves TOK tokens.  The experts are dealt round-robin to the four
// waves; a wave keeps the TOK token rows in registers as fp32, streams one router row at a time
// and forms the dot product in the fixed order of the interface: lane j owns elements
// 512*c + 8*j .. +7 of every 512-element chunk c (one 16-byte load per chunk), accumulates them
// in ascending index by fused multiply-add, and the 64 lane sums are folded by an xor butterfly
// 32,16,...,1.  bf16 products are exact in fp32, so this reproduces a CPU evaluation in the same
// order bit for bit.  The logits meet in LDS; then one wave per token runs softmax and K rounds
// of wave-wide argmax (ties to the lower expert id).
#include "common.h"

namespace moe {

constexpr int ROUTE_EMAX = 256;
constexpr int ROUTE_KMAX = 16;

template <int C, int TOK>
__global__ __launch_bounds__(256) void route_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wr,
                                                    const float* __restrict__ bias, int T, int H, int E, int K,
                                                    int renorm, int32_t* __restrict__ ids, float* __restrict__ w) {
  __shared__ float s_logit[TOK][ROUTE_EMAX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * TOK;

  // token rows -> fp32 registers (zero beyond H or T; a zero product leaves a partial sum unchanged)
  float xf[TOK][C][8];
#pragma unroll
  for (int tk = 0; tk < TOK; ++tk) {
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const int h = 512 * c + 8 * lane;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (h < H && t0 + tk < T) v = *reinterpret_cast<const uint4*>(x + (size_t)(t0 + tk) * H + h);
      xf[tk][c][0] = bf16_lo(v.x); xf[tk][c][1] = bf16_hi(v.x);
      xf[tk][c][2] = bf16_lo(v.y); xf[tk][c][3] = bf16_hi(v.y);
      xf[tk][c][4] = bf16_lo(v.z); xf[tk][c][5] = bf16_hi(v.z);
      xf[tk][c][6] = bf16_lo(v.w); xf[tk][c][7] = bf16_hi(v.w);
    }
  }

  for (int e = wave; e < E; e += 4) {
    float wf[C][8];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const int h = 512 * c + 8 * lane;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (h < H) v = *reinterpret_cast<const uint4*>(Wr + (size_t)e * H + h);
      wf[c][0] = bf16_lo(v.x); wf[c][1] = bf16_hi(v.x);
      wf[c][2] = bf16_lo(v.y); wf[c][3] = bf16_hi(v.y);
      wf[c][4] = bf16_lo(v.z); wf[c][5] = bf16_hi(v.z);
      wf[c][6] = bf16_lo(v.w); wf[c][7] = bf16_hi(v.w);
    }
    const float b = bias ? bias[e] : 0.0f;
#pragma unroll
    for (int tk = 0; tk < TOK; ++tk) {
      float a = 0.0f;
#pragma unroll
      for (int c = 0; c < C; ++c) {
#pragma unroll
        for (int i = 0; i < 8; ++i) a = __builtin_fmaf(xf[tk][c][i], wf[c][i], a);
      }
#pragma unroll
      for (int s = 32; s >= 1; s >>= 1) a = a + __shfl_xor(a, s, WAVE);
      if (bias) a = a + b;
      if (lane == 0) s_logit[tk][e] = a;
    }
  }
  __syncthreads();

  for (int tk = wave; tk < TOK; tk += 4) {
    const int t = t0 + tk;
    if (t >= T) break;
    float l[4];
    bool taken[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      l[i] = e < E ? s_logit[tk][e] : -INFINITY;
      taken[i] = e >= E;
    }
    const float m = wave_max(fmaxf(fmaxf(l[0], l[1]), fmaxf(l[2], l[3])));
    float z = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (lane + 64 * i < E) z += expf(l[i] - m);
    const float denom = wave_sum(z);

    int my_id = 0;
    float my_w = 0.0f, run = 0.0f;
    for (int j = 0; j < K; ++j) {
      float bv = -INFINITY;
      int be = 0x7fffffff;
#pragma unroll
      for (int i = 0; i < 4; ++i) {  // ascending expert id inside the lane: '>' keeps the lower id
        if (!taken[i] && (be == 0x7fffffff || l[i] > bv)) { bv = l[i]; be = lane + 64 * i; }
      }
#pragma unroll
      for (int s = 32; s >= 1; s >>= 1) {
        const float ov = __shfl_xor(bv, s, WAVE);
        const int oe = __shfl_xor(be, s, WAVE);
        const bool take = (oe != 0x7fffffff) && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be));
        if (take) { bv = ov; be = oe; }
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

template <int C, int TOK>
static int launch_route_t(const void* x, const void* Wr, const float* bias, int T, int H, int E, int K, int renorm,
                          int32_t* ids, float* w, hipStream_t st) {
  const int blocks = (T + TOK - 1) / TOK;
  hipLaunchKernelGGL((route_kernel<C, TOK>), dim3(blocks), dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)Wr,
                     bias, T, H, E, K, renorm, ids, w);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int launch_route(const void* x, const void* Wr, const float* bias, int T, int H, int E, int K, int renorm,
                 int32_t* ids, float* w, hipStream_t st) {
  const int chunks = (H + 511) / 512;
  const bool many = T >= 2048;  // enough tokens to fill the chip with 4 per workgroup
  if (chunks <= 1) return many ? launch_route_t<1, 4>(x, Wr, bias, T, H, E, K, renorm, ids, w, st)
                               : launch_route_t<1, 1>(x, Wr, bias, T, H, E, K, renorm, ids, w, st);
  if (chunks <= 2) return many ? launch_route_t<2, 4>(x, Wr, bias, T, H, E, K, renorm, ids, w, st)
                               : launch_route_t<2, 1>(x, Wr, bias, T, H, E, K, renorm, ids, w, st);
  if (chunks <= 4) return many ? launch_route_t<4, 4>(x, Wr, bias, T, H, E, K, renorm, ids, w, st)
                               : launch_route_t<4, 1>(x, Wr, bias, T, H, E, K, renorm, ids, w, st);
  if (chunks <= 8) return many ? launch_route_t<8, 2>(x, Wr, bias, T, H, E, K, renorm, ids, w, st)
                               : launch_route_t<8, 1>(x, Wr, bias, T, H, E, K, renorm, ids, w, st);
  if (chunks <= 16) return launch_route_t<16, 1>(x, Wr, bias, T, H, E, K, renorm, ids, w, st);
  return -2;
}

}  // namespace moe
