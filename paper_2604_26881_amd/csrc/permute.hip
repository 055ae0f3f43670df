// Micro-batch construction (FaaSMoE Sec. 3 and Sec. 4.1: all tokens routed to one expert block
// are consolidated into one batched invocation).  A stable counting sort of the P = T*K
// (token, slot) pairs by expert id, followed by a coalesced gather of the token rows.
//
// permute_index_kernel: ONE workgroup of 16 waves, no global atomics, so the ranks are
// deterministic.  Wave w owns a contiguous segment of the pairs.
//   pass 1  per-wave histogram in LDS (LDS atomics: integer counts, order-free); the expert ids
//           are parked in LDS as bytes so pass 2 does not wait on global memory again;
//   scan    per expert: exclusive prefix over the 16 waves; over experts: exclusive prefix of
//           the totals -> expert_offsets;
//   pass 2  each wave walks its segment 64 pairs at a time; lanes with the same expert find
//           each other with bit-sliced ballots (log2 E ballots), rank = number of lower lanes in
//           the match set; row = offsets[e] + pairs of e in earlier waves/chunks + rank.
// gather_rows_kernel: one workgroup per output row, 16-byte loads and stores.
#include "common.h"

namespace moe {

constexpr int PERM_WAVES = 16;
constexpr int PERM_EMAX = 256;
constexpr int PERM_STAGE_MAX = 96 * 1024;  // pairs whose ids fit the LDS byte buffer

__global__ __launch_bounds__(1024) void permute_index_kernel(const int32_t* __restrict__ ids, int P, int E,
                                                             int32_t* __restrict__ offsets,
                                                             int32_t* __restrict__ src_of_row,
                                                             int32_t* __restrict__ row_of_pair) {
  extern __shared__ unsigned char s_ids[];              // [min(P, PERM_STAGE_MAX)] when staged
  __shared__ int s_hist[PERM_WAVES][PERM_EMAX];         // counts, then running row bases
  __shared__ int s_tot[PERM_EMAX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool staged = P <= PERM_STAGE_MAX;

  for (int i = tid; i < PERM_WAVES * PERM_EMAX; i += 1024) (&s_hist[0][0])[i] = 0;
  __syncthreads();

  // segment of this wave: whole 64-pair chunks
  const int chunks = (P + 63) / 64;
  const int per = (chunks + PERM_WAVES - 1) / PERM_WAVES;
  const int c_beg = wave * per;
  const int c_end = min(chunks, c_beg + per);

  for (int c = c_beg; c < c_end; ++c) {
    const int p = c * 64 + lane;
    if (p < P) {
      const int e = min(max(ids[p], 0), E - 1);   // an id outside [0,E) must not leave the table
      if (staged) s_ids[p] = (unsigned char)e;
      atomicAdd(&s_hist[wave][e], 1);
    }
  }
  __syncthreads();

  // exclusive prefix over waves, per expert
  if (tid < E) {
    int run = 0;
    for (int wv = 0; wv < PERM_WAVES; ++wv) {
      const int c = s_hist[wv][tid];
      s_hist[wv][tid] = run;
      run += c;
    }
    s_tot[tid] = run;
  }
  __syncthreads();
  // exclusive prefix over experts (E <= 256: done by wave 0, four experts per lane)
  if (wave == 0) {
    int v[4], sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane * 4 + i;
      v[i] = e < E ? s_tot[e] : 0;
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
      if (e < E) {
        s_tot[e] = base;
        offsets[e] = base;
      }
      base += v[i];
    }
    if (lane == 63) offsets[E] = incl;
  }
  __syncthreads();
  if (tid < E) {
    const int off = s_tot[tid];
    for (int wv = 0; wv < PERM_WAVES; ++wv) s_hist[wv][tid] += off;
  }
  __syncthreads();

  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  volatile int* base_row = &s_hist[wave][0];
  for (int c = c_beg; c < c_end; ++c) {
    const int p = c * 64 + lane;
    const bool valid = p < P;
    int e = 0;
    if (valid) e = staged ? (int)s_ids[p] : min(max(ids[p], 0), E - 1);
    unsigned long long match = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
      const unsigned long long bal = __ballot(valid && ((e >> b) & 1));
      match &= ((e >> b) & 1) ? bal : ~bal;
    }
    if (valid) {
      const unsigned long long below = match & ((1ull << lane) - 1ull);
      const int rank = __popcll(below);
      const int row = base_row[e] + rank;
      row_of_pair[p] = row;
      src_of_row[row] = p;
    }
    __builtin_amdgcn_wave_barrier();   // every lane has read its base before a leader moves it
    if (valid) {
      const unsigned long long below = match & ((1ull << lane) - 1ull);
      if (below == 0ull) base_row[e] = base_row[e] + __popcll(match);
    }
    __builtin_amdgcn_wave_barrier();
  }
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const bf16_t* __restrict__ x,
                                                          const int32_t* __restrict__ src_of_row, int K, int H,
                                                          bf16_t* __restrict__ Xp) {
  const int r = blockIdx.x;
  const int t = src_of_row[r] / K;
  const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)t * H);
  uint4* dst = reinterpret_cast<uint4*>(Xp + (size_t)r * H);
  for (int i = threadIdx.x; i < H / 8; i += 256) dst[i] = src[i];
}

int launch_permute(const int32_t* ids, const void* x, int T, int H, int E, int K, int32_t* offsets,
                   int32_t* src_of_row, int32_t* row_of_pair, void* Xp, hipStream_t st) {
  const int P = T * K;
  const size_t dyn = P <= PERM_STAGE_MAX ? (size_t)((P + 255) / 256) * 256 : 0;
  if (dyn > 32 * 1024) {  // more dynamic LDS than the default limit: raise it for this kernel
    if (hipFuncSetAttribute((const void*)permute_index_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            PERM_STAGE_MAX) != hipSuccess)
      return -4;
  }
  hipLaunchKernelGGL(permute_index_kernel, dim3(1), dim3(1024), dyn, st, ids, P, E, offsets, src_of_row,
                     row_of_pair);
  if (hipGetLastError() != hipSuccess) return -4;
  if (P > 0) {
    hipLaunchKernelGGL(gather_rows_kernel, dim3(P), dim3(256), 0, st, (const bf16_t*)x, src_of_row, K, H,
                       (bf16_t*)Xp);
    if (hipGetLastError() != hipSuccess) return -4;
  }
  return 0;
}

}  // namespace moe
