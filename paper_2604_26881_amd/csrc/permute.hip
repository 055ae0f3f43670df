// Micro-batch construction (FaaSMoE Sec. 3; Sec. 4.1 "token-level micro-batching": each expert block
// is invoked once, on the batch of every token gating sent to it).  A stable counting sort of the P = T*K
// (token, slot) pairs by expert id, followed by a coalesced gather of the token rows.
// No atomics anywhere, so the result is deterministic; every step runs on many CUs.
//
// The pairs are cut into chunks of 64 (one wave).
// permute_hist_kernel: one wave per chunk.  Lanes with the same expert find each other with
//   bit-sliced ballots (log2 E ballots); the first lane of each group writes the group size:
//   hist[chunk][e] = number of pairs of expert e in the chunk (E contiguous ints per chunk).
// permute_scatter_kernel: one workgroup per chunk (several for small P).  It sums the table over
//   all chunks (-> totals, hence expert_offsets by a scan over experts) and over the chunks before
//   its own (-> rows taken by earlier pairs), recomputes the rank of each pair inside the chunk
//   with the same ballots, and has row = offsets[e] + earlier[e] + rank.  It writes row_of_pair and
//   src_of_row and copies the 64 token rows with 16-byte loads and stores.  The table is P/64 x E
//   ints (61 KB at 16 384 pairs), read from L2 by every workgroup.
#include "common.h"

namespace moe {

constexpr int PERM_EMAX = 256;

// match set of each lane: the lanes of the wave whose (valid) pair has the same expert id
__device__ __forceinline__ unsigned long long match_expert(int e, bool valid, int nbits) {
  unsigned long long match = __ballot(valid);
  for (int b = 0; b < nbits; ++b) {
    const unsigned long long bal = __ballot(valid && ((e >> b) & 1));
    match &= ((e >> b) & 1) ? bal : ~bal;
  }
  return match;
}
__device__ __forceinline__ int bits_for(int E) {
  int nbits = 0;
  while ((1 << nbits) < E) ++nbits;
  return nbits;
}

__global__ __launch_bounds__(256) void permute_hist_kernel(const int32_t* __restrict__ ids, int P, int E,
                                                           int32_t* __restrict__ hist) {
  const int lane = threadIdx.x & 63;
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c * 64 >= P) return;
  const int p = c * 64 + lane;
  const bool valid = p < P;
  const int e = valid ? min(max(ids[p], 0), E - 1) : 0;   // an id outside [0,E) must not leave the table
  int32_t* row = hist + (size_t)c * E;
  for (int i = lane; i < E; i += 64) row[i] = 0;
  const unsigned long long match = match_expert(e, valid, bits_for(E));
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the zeros are written before the counts
  if (valid && (match & ((1ull << lane) - 1ull)) == 0ull) row[e] = __popcll(match);
}

__global__ __launch_bounds__(256) void permute_scatter_kernel(const int32_t* __restrict__ ids,
                                                              const int32_t* __restrict__ hist,
                                                              const bf16_t* __restrict__ x, int P, int E, int K, int H,
                                                              int split, int32_t* __restrict__ offsets,
                                                              int32_t* __restrict__ src_of_row,
                                                              int32_t* __restrict__ row_of_pair,
                                                              bf16_t* __restrict__ Xp) {
  __shared__ int s_before[4][PERM_EMAX];   // partial sums over earlier chunks, per quarter of the threads
  __shared__ int s_total[4][PERM_EMAX];    // partial sums over all chunks
  __shared__ int s_base[PERM_EMAX];        // first row of expert e for this chunk
  __shared__ int s_row[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.x / split, part = blockIdx.x % split;
  const int chunks = (P + 63) / 64;

  // column sums of the table: thread (q, e) takes chunks q, q+4, ... for experts e, e+64, ...
  for (int e = lane; e < E; e += 64) {
    int before = 0, total = 0;
    for (int cb = wave; cb < chunks; cb += 32) {   // 8 loads in flight per thread
      int v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int cc = cb + 4 * u;
        v[u] = cc < chunks ? hist[(size_t)cc * E + e] : 0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        total += v[u];
        if (cb + 4 * u < c) before += v[u];
      }
    }
    s_before[wave][e] = before;
    s_total[wave][e] = total;
  }
  __syncthreads();
  if (wave == 0) {   // exclusive scan of the totals over experts, four experts per lane
    int v[4], sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane * 4 + i;
      v[i] = e < E ? s_total[0][e] + s_total[1][e] + s_total[2][e] + s_total[3][e] : 0;
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
        s_base[e] = base + s_before[0][e] + s_before[1][e] + s_before[2][e] + s_before[3][e];
        if (blockIdx.x == 0) offsets[e] = base;
      }
      base += v[i];
    }
    if (blockIdx.x == 0 && lane == 63) offsets[E] = incl;
  }
  __syncthreads();
  if (wave == 0) {
    const int p = c * 64 + lane;
    const bool valid = p < P;
    const int e = valid ? min(max(ids[p], 0), E - 1) : 0;
    const unsigned long long match = match_expert(e, valid, bits_for(E));
    int row = -1;
    if (valid) {
      row = s_base[e] + __popcll(match & ((1ull << lane) - 1ull));
      if (part == 0) {
        row_of_pair[p] = row;
        src_of_row[row] = p;
      }
    }
    s_row[lane] = row;
  }
  __syncthreads();
  if (Xp == nullptr) return;   // index arrays only: the expert kernels gather the token rows themselves
  // rows of this chunk are dealt to the (split * 4) waves that serve it
  for (int i = part * 4 + wave; i < 64; i += split * 4) {
    const int row = s_row[i];
    if (row < 0) break;                       // pairs past P sit at the end of the last chunk
    const int t = (c * 64 + i) / K;
    const u32x4* src = reinterpret_cast<const u32x4*>(x + (size_t)t * H);
    u32x4* dst = reinterpret_cast<u32x4*>(Xp + (size_t)row * H);
    for (int j = lane; j < H / 8; j += 64) dst[j] = src[j];
  }
}

// Few pairs and no row copies (index arrays only): the whole sort in one workgroup of up to 16
// waves, one pair per thread.  Same arithmetic as the two kernels above (counts per wave and
// expert, sums over earlier waves, scan over experts, rank inside the wave), without the table in
// global memory and with one launch instead of two: at decode sizes the launches are the cost.
constexpr int PERM_SMALL_MAX = 1024;
__global__ __launch_bounds__(PERM_SMALL_MAX) void permute_small_kernel(const int32_t* __restrict__ ids, int P, int E,
                                                                       int32_t* __restrict__ offsets,
                                                                       int32_t* __restrict__ src_of_row,
                                                                       int32_t* __restrict__ row_of_pair) {
  __shared__ int s_cnt[PERM_SMALL_MAX / 64][PERM_EMAX];   // pairs of expert e in wave w; then: in earlier waves
  __shared__ int s_base[PERM_EMAX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  for (int i = tid; i < nwaves * PERM_EMAX; i += blockDim.x) (&s_cnt[0][0])[i] = 0;
  __syncthreads();
  const int p = tid;
  const bool valid = p < P;
  const int e = valid ? min(max(ids[p], 0), E - 1) : 0;
  const unsigned long long match = match_expert(e, valid, bits_for(E));
  const unsigned long long below = match & ((1ull << lane) - 1ull);
  if (valid && below == 0ull) s_cnt[wave][e] = __popcll(match);
  __syncthreads();
  for (int x = tid; x < E; x += blockDim.x) {   // expert x: exclusive sums over the waves, total
    int run = 0;
    for (int w = 0; w < nwaves; ++w) {
      const int c = s_cnt[w][x];
      s_cnt[w][x] = run;
      run += c;
    }
    s_base[x] = run;
  }
  __syncthreads();
  if (wave == 0) {   // exclusive scan of the totals over experts, four experts per lane
    int v[4], sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int x = lane * 4 + i;
      v[i] = x < E ? s_base[x] : 0;
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
      const int x = lane * 4 + i;
      if (x < E) {
        s_base[x] = base;
        offsets[x] = base;
      }
      base += v[i];
    }
    if (lane == 63) offsets[E] = incl;
  }
  __syncthreads();
  if (valid) {
    const int row = s_base[e] + s_cnt[wave][e] + __popcll(below);
    row_of_pair[p] = row;
    src_of_row[row] = p;
  }
}

// P == 0: every offset is zero.
__global__ void permute_empty_kernel(int E, int32_t* __restrict__ offsets) {
  for (int e = threadIdx.x; e <= E; e += blockDim.x) offsets[e] = 0;
}

int launch_permute(const int32_t* ids, const void* x, int T, int H, int E, int K, int32_t* offsets,
                   int32_t* src_of_row, int32_t* row_of_pair, void* Xp, void* workspace, hipStream_t st) {
  const int P = T * K;
  if (P == 0) {
    hipLaunchKernelGGL(permute_empty_kernel, dim3(1), dim3(256), 0, st, E, offsets);
    return hipGetLastError() == hipSuccess ? 0 : -4;
  }
  if (Xp == nullptr && P <= PERM_SMALL_MAX) {
    const int threads = ((P + 63) / 64) * 64;
    hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(threads), 0, st, ids, P, E, offsets, src_of_row, row_of_pair);
    return hipGetLastError() == hipSuccess ? 0 : -4;
  }
  int32_t* hist = static_cast<int32_t*>(workspace);
  const int chunks = (P + 63) / 64;
  hipLaunchKernelGGL(permute_hist_kernel, dim3((chunks + 3) / 4), dim3(256), 0, st, ids, P, E, hist);
  if (hipGetLastError() != hipSuccess) return -4;
  // several workgroups share the row copies of one chunk, about a thousand workgroups in all
  const int split = Xp == nullptr ? 1 : (chunks >= 1024 ? 1 : (chunks >= 64 ? min(16, 1024 / chunks) : 16));
  hipLaunchKernelGGL(permute_scatter_kernel, dim3(chunks * split), dim3(256), 0, st, ids, hist, (const bf16_t*)x, P,
                     E, K, H, split, offsets, src_of_row, row_of_pair, (bf16_t*)Xp);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // namespace moe
