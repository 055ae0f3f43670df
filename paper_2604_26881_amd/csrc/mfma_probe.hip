// Measurement aid, not part of the MoE path: the rate the matrix pipes sustain on operands the caller
// supplies, with nothing else going on (operands and accumulators stay in registers, no memory traffic
// in the loop), and the shader clock the chip holds meanwhile.  The chip lowers its clock under dense
// MFMA work on operands with realistic bit activity; timing this kernel on zeros and on random bf16
// values separates that effect from the kernels' own losses.
//
// One workgroup of four waves per launch slot; every wave issues iters x 16 independent
// v_mfma_f32_32x32x16_bf16 (4 x 4 fragment pairs, 16 accumulators of 16 registers).
#include "common.h"

namespace moe {

__global__ __launch_bounds__(256, 1) void mfma_probe_kernel(const u32x4* __restrict__ operands, int iters,
                                                            long long* __restrict__ clocks) {
  u32x4 fa[4], fb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    fa[i] = operands[threadIdx.x + 256 * i];
    fb[i] = operands[threadIdx.x + 256 * (4 + i)];
  }
  f32x16 acc[4][4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[j][k][i] = 0.0f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int k = 0; k < 4; ++k)
        acc[j][k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fa[j]), as_bf16x8(fb[k]), acc[j][k], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int i = 0; i < 16; ++i) s += acc[j][k][i];
  const long long c1 = clock64(), w1 = wall_clock64();
  // the sums are consumed (a value no input produces would be stored), so the loop is not dropped
  if (threadIdx.x == 0 || s == -123456.789f) {
    clocks[blockIdx.x * 2] = c1 - c0;        // shader clock ticks
    clocks[blockIdx.x * 2 + 1] = w1 - w0;    // ticks of the constant 100 MHz clock
  }
}

int launch_mfma_probe(const void* operands, int iters, int workgroups, long long* clocks, hipStream_t st) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, st, (const u32x4*)operands, iters, clocks);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // namespace moe
