// Aggregation (FaaSMoE Sec. 3 and Sec. 4.2: the orchestrator aggregates what the expert blocks
// return).  out[t,:] = sum_j topk_w[t,j] * Yp[row_of_pair[t*K+j],:] + sigmoid(sg[t]) * S[t,:],
// where S may come as the separate outputs of the shared experts (n_parts tensors [T,H], added in
// fp32 in ascending order before the gate is applied).
//
// A gather, not a scatter: one workgroup per token reads its K expert rows (and the shared
// row) with 16-byte loads, accumulates in fp32 in slot order j = 0..K-1 and rounds once to
// bf16.  No atomics, so the result does not depend on which block produced a row or when.
#include "common.h"

namespace moe {

constexpr int COMBINE_KMAX = 16;

__global__ __launch_bounds__(256) void combine_kernel(const bf16_t* __restrict__ Yp,
                                                      const int32_t* __restrict__ row_of_pair,
                                                      const float* __restrict__ topk_w,
                                                      const bf16_t* __restrict__ S, int n_parts, long part_stride,
                                                      const float* __restrict__ sg, int H, int K,
                                                      bf16_t* __restrict__ out) {
  const int t = blockIdx.x;
  __shared__ int s_row[COMBINE_KMAX];
  __shared__ float s_w[COMBINE_KMAX];
  if (threadIdx.x < K) {
    s_row[threadIdx.x] = row_of_pair[(size_t)t * K + threadIdx.x];
    s_w[threadIdx.x] = topk_w[(size_t)t * K + threadIdx.x];
  }
  __syncthreads();
  float gate = 0.0f;
  if (S != nullptr) gate = 1.0f / (1.0f + expf(-sg[t]));

  for (int c = threadIdx.x; c < H / 8; c += 256) {
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
    // the shared row and four expert rows at a time are requested before any of them is used
    // (the sum still takes the rows in slot order)
    uint4 vs = {0u, 0u, 0u, 0u};
    if (S != nullptr) vs = reinterpret_cast<const uint4*>(S + (size_t)t * H)[c];
    float sh[8];
    if (n_parts > 1) {   // the shared experts' outputs come as separate tensors: summed first, in order
      sh[0] = bf16_lo(vs.x); sh[1] = bf16_hi(vs.x); sh[2] = bf16_lo(vs.y); sh[3] = bf16_hi(vs.y);
      sh[4] = bf16_lo(vs.z); sh[5] = bf16_hi(vs.z); sh[6] = bf16_lo(vs.w); sh[7] = bf16_hi(vs.w);
      for (int p = 1; p < n_parts; ++p) {
        const uint4 v = reinterpret_cast<const uint4*>(S + (size_t)p * part_stride + (size_t)t * H)[c];
        sh[0] += bf16_lo(v.x); sh[1] += bf16_hi(v.x); sh[2] += bf16_lo(v.y); sh[3] += bf16_hi(v.y);
        sh[4] += bf16_lo(v.z); sh[5] += bf16_hi(v.z); sh[6] += bf16_lo(v.w); sh[7] += bf16_hi(v.w);
      }
    }
    for (int j0 = 0; j0 < K; j0 += 4) {
      uint4 vv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (j0 + u < K) vv[u] = reinterpret_cast<const uint4*>(Yp + (size_t)s_row[j0 + u] * H)[c];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (j0 + u < K) {
          const uint4 v = vv[u];
          const float wj = s_w[j0 + u];
          acc[0] = __builtin_fmaf(wj, bf16_lo(v.x), acc[0]); acc[1] = __builtin_fmaf(wj, bf16_hi(v.x), acc[1]);
          acc[2] = __builtin_fmaf(wj, bf16_lo(v.y), acc[2]); acc[3] = __builtin_fmaf(wj, bf16_hi(v.y), acc[3]);
          acc[4] = __builtin_fmaf(wj, bf16_lo(v.z), acc[4]); acc[5] = __builtin_fmaf(wj, bf16_hi(v.z), acc[5]);
          acc[6] = __builtin_fmaf(wj, bf16_lo(v.w), acc[6]); acc[7] = __builtin_fmaf(wj, bf16_hi(v.w), acc[7]);
        }
      }
    }
    if (S != nullptr && n_parts > 1) {
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(gate, sh[i], acc[i]);
    } else if (S != nullptr) {
      const uint4 v = vs;
      acc[0] = __builtin_fmaf(gate, bf16_lo(v.x), acc[0]); acc[1] = __builtin_fmaf(gate, bf16_hi(v.x), acc[1]);
      acc[2] = __builtin_fmaf(gate, bf16_lo(v.y), acc[2]); acc[3] = __builtin_fmaf(gate, bf16_hi(v.y), acc[3]);
      acc[4] = __builtin_fmaf(gate, bf16_lo(v.z), acc[4]); acc[5] = __builtin_fmaf(gate, bf16_hi(v.z), acc[5]);
      acc[6] = __builtin_fmaf(gate, bf16_lo(v.w), acc[6]); acc[7] = __builtin_fmaf(gate, bf16_hi(v.w), acc[7]);
    }
    uint4 o;
    o.x = pack_bf16x2(acc[0], acc[1]);
    o.y = pack_bf16x2(acc[2], acc[3]);
    o.z = pack_bf16x2(acc[4], acc[5]);
    o.w = pack_bf16x2(acc[6], acc[7]);
    reinterpret_cast<uint4*>(out + (size_t)t * H)[c] = o;
  }
}

// sg[t] = <x[t,:], wgate>: one wave per token, fp32.
__global__ __launch_bounds__(256) void gate_dot_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ wgate,
                                                       int T, int H, float* __restrict__ sg) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float a = 0.0f;
  for (int c = lane; c < H / 8; c += 64) {
    const uint4 v = reinterpret_cast<const uint4*>(x + (size_t)t * H)[c];
    const uint4 g = reinterpret_cast<const uint4*>(wgate)[c];
    a = __builtin_fmaf(bf16_lo(v.x), bf16_lo(g.x), a); a = __builtin_fmaf(bf16_hi(v.x), bf16_hi(g.x), a);
    a = __builtin_fmaf(bf16_lo(v.y), bf16_lo(g.y), a); a = __builtin_fmaf(bf16_hi(v.y), bf16_hi(g.y), a);
    a = __builtin_fmaf(bf16_lo(v.z), bf16_lo(g.z), a); a = __builtin_fmaf(bf16_hi(v.z), bf16_hi(g.z), a);
    a = __builtin_fmaf(bf16_lo(v.w), bf16_lo(g.w), a); a = __builtin_fmaf(bf16_hi(v.w), bf16_hi(g.w), a);
  }
  a = wave_sum(a);
  if (lane == 0) sg[t] = a;
}

// out[t,:] = bf16( u / sqrt(mean_h(u^2) + eps) ),  u = x[t,:] + y[t,:] in fp32: the step between two
// MoE layers when layers are chained without attention.  One workgroup per token; the row stays in
// registers between the two passes (H <= 8192).
__global__ __launch_bounds__(256) void residual_norm_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ y,
                                                            int H, float eps, bf16_t* __restrict__ out) {
  __shared__ float s_part[4];
  const int t = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float u[4][8];
  float ss = 0.0f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int c = threadIdx.x + 256 * r;
#pragma unroll
    for (int i = 0; i < 8; ++i) u[r][i] = 0.0f;
    if (c < H / 8) {
      const uint4 a = reinterpret_cast<const uint4*>(x + (size_t)t * H)[c];
      const uint4 b = reinterpret_cast<const uint4*>(y + (size_t)t * H)[c];
      u[r][0] = bf16_lo(a.x) + bf16_lo(b.x); u[r][1] = bf16_hi(a.x) + bf16_hi(b.x);
      u[r][2] = bf16_lo(a.y) + bf16_lo(b.y); u[r][3] = bf16_hi(a.y) + bf16_hi(b.y);
      u[r][4] = bf16_lo(a.z) + bf16_lo(b.z); u[r][5] = bf16_hi(a.z) + bf16_hi(b.z);
      u[r][6] = bf16_lo(a.w) + bf16_lo(b.w); u[r][7] = bf16_hi(a.w) + bf16_hi(b.w);
#pragma unroll
      for (int i = 0; i < 8; ++i) ss = __builtin_fmaf(u[r][i], u[r][i], ss);
    }
  }
  ss = wave_sum(ss);
  if (lane == 0) s_part[wave] = ss;
  __syncthreads();
  const float total = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
  const float scale = 1.0f / sqrtf(total / (float)H + eps);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int c = threadIdx.x + 256 * r;
    if (c < H / 8) {
      uint4 o;
      o.x = pack_bf16x2(u[r][0] * scale, u[r][1] * scale);
      o.y = pack_bf16x2(u[r][2] * scale, u[r][3] * scale);
      o.z = pack_bf16x2(u[r][4] * scale, u[r][5] * scale);
      o.w = pack_bf16x2(u[r][6] * scale, u[r][7] * scale);
      reinterpret_cast<uint4*>(out + (size_t)t * H)[c] = o;
    }
  }
}

int launch_residual_norm(const void* x, const void* y, int T, int H, float eps, void* out, hipStream_t st) {
  if (T == 0) return 0;
  hipLaunchKernelGGL(residual_norm_kernel, dim3(T), dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)y, H, eps,
                     (bf16_t*)out);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int launch_combine(const void* Yp, const int32_t* row_of_pair, const float* w, const void* S, int n_parts,
                   const float* sg, int T, int H, int K, void* out, hipStream_t st) {
  if (T == 0) return 0;
  hipLaunchKernelGGL(combine_kernel, dim3(T), dim3(256), 0, st, (const bf16_t*)Yp, row_of_pair, w,
                     (const bf16_t*)S, n_parts, (long)T * H, sg, H, K, (bf16_t*)out);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int launch_gate_dot(const void* x, const void* wgate, int T, int H, float* sg, hipStream_t st) {
  if (T == 0) return 0;
  hipLaunchKernelGGL(gate_dot_kernel, dim3((T + 3) / 4), dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)wgate,
                     T, H, sg);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // namespace moe
