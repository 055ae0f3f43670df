// Shared device helpers for the gfx950 MoE-layer kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

typedef uint16_t bf16_t;  // raw bf16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // 16 bytes moved as one register quad

constexpr int WAVE = 64;

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
// Two fp32 -> packed bf16 pair, round to nearest even: one v_cvt_pk_bf16_f32 on gfx950 (the same
// result as f32_to_bf16_bits for finite values).
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v = fmaxf(v, __shfl_xor(v, s, WAVE));
  return v;
}

// Lanes l < 32 and l + 32 trade registers: afterwards a holds, in lanes 32-63, what b held in lanes
// 0-31, and b holds, in lanes 0-31, what a held in lanes 32-63 (v_permlane32_swap); the other
// halves keep their values.
__device__ __forceinline__ void trade_halves(uint32_t& a, uint32_t& b) {
  const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  a = r[0];
  b = r[1];
}

// One 16-byte-per-lane copy from global memory straight into LDS (no registers in between):
// lane l of the wave writes LDS bytes [lds + 16*l, +16) from global address base + voff.
// The copy is asynchronous; it is counted by vmcnt like any other vector memory load.
// (One wait state between the write of m0 and the instruction that reads it: the ISA asks for it, and the
// compiler, which pads its own such pairs, does not look inside an asm statement.)
__device__ __forceinline__ void copy_to_lds_16(const void* base, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds)
               : "memory", "m0");
}
// The same copy with the non-temporal hint: for data that is read once (streamed weights), so that
// it does not displace reusable lines from the caches.  Measured on a 1 GiB stream of 4 KB rows:
// 6.0 TB/s without the hint, 6.8 TB/s with it.
__device__ __forceinline__ void copy_to_lds_16_stream(const void* base, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(voff), "s"(base), "s"(lds)
               : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_copies_but() {   // all but the N most recent copies have landed
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void workgroup_barrier() { asm volatile("s_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_lds_reads() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// Launch helpers used by the C entry points.
struct GemmArgs {
  const bf16_t* A;     // token rows [rows, Kdim]
  const bf16_t* B0;    // weights [E, N, Kdim]  (gate branch, or the down projection)
  const bf16_t* B1;    // weights of the up branch (gate/up kernels), else unused
  bf16_t* C;           // output rows [rows, N]
  const int32_t* offsets;  // expert_offsets on the device, or nullptr for one expert on rows [0, rows_fixed)
  int lo, hi;          // experts [lo, hi); with an id list: positions [lo, hi) of the list
  const int32_t* ids;  // nullptr: expert id = position; else the block is the experts ids[lo .. hi) (device memory)
  int rows_fixed;
  int rows_total;      // number of rows of A and C (upper bound used to size the grid)
  int mean_rows;       // expected rows per expert (rows_total / experts of the layer): picks kernel shapes
  int N;               // output columns (per branch for gate/up)
  int Kdim;            // contraction length
  float* Cpart;        // fp32 partial outputs [parts, rows_total, N] of kernels that cut K, else unused
  const int32_t* gather;   // nullptr: row r of A is A[r]; else row r of A is A[gather[r] / gather_div]
  int gather_div;          // (the token rows themselves, addressed through src_of_row: no permuted copy)
  int leave_room;          // 1: no tile shape that takes a whole CU (all registers of every SIMD): kernels of
                           // other streams can then share the CUs with this one
  // Shared experts riding along with a routed block (tile kernels only; n_shared == 0: none).  They are
  // n_shared more weight sets, each applied to all shared_rows tokens.  In the row space of A and C
  // the routed rows are [0, rows_routed) and set s owns rows rows_routed + s*shared_rows onwards.
  int n_shared;
  int shared_rows;         // tokens T
  int rows_routed;         // P
  const bf16_t* Bs0;       // weights of set 0 (gate branch, or the down projection); set s starts s*shared_b_step
  const bf16_t* Bs1;       // elements further on; consecutive weight rows of a set are ldb_shared elements apart
  long shared_b_step;
  int ldb_shared;
  const bf16_t* As;        // not nullptr: set s reads its token rows from As[0 .. shared_rows) instead of A (gate/up: x)
  bf16_t* Cs;              // not nullptr: row r of set s goes to Cs[s*shared_rows + r] instead of C (down: the S parts)
  // Measurement aid (tile kernels; nullptr: off): workgroup b < clock_groups writes four values at clocks[4*b]:
  // shader-clock ticks and ticks of the constant 100 MHz clock between its start and its end, the shader-clock
  // ticks it spent inside the K loops of its tiles, and the number of its tiles.
  long long* clocks;
  int clock_groups;
};
// Where the tile-kernel launches of the calling host thread record their clocks (nullptr: nowhere).
void set_tile_clock_buffer(long long* clocks, int groups);

// bias [E] for all tokens (seg == nullptr), or bias [n_seg, E] with seg [n_seg + 1] segment bounds on the device
int launch_route(const void* x, const void* Wr, const float* bias, const int32_t* seg, int n_seg, int T, int H, int E,
                 int K, int renorm, int32_t* ids, float* w, hipStream_t st);
int launch_permute(const int32_t* ids, const void* x, int T, int H, int E, int K, int32_t* offsets,
                   int32_t* src_of_row, int32_t* row_of_pair, void* Xp, void* workspace, hipStream_t st);
int launch_combine(const void* Yp, const int32_t* row_of_pair, const float* w, const void* S, int n_parts,
                   const float* sg, int T, int H, int K, void* out, hipStream_t st);
int launch_residual_norm(const void* x, const void* y, int T, int H, float eps, void* out, hipStream_t st);
int launch_gate_dot(const void* x, const void* wgate, int T, int H, float* sg, hipStream_t st);
int launch_mfma_probe(const void* operands, int iters, int workgroups, long long* clocks, hipStream_t st);
// Tiled MFMA kernels (many rows per expert) and streaming kernels (few rows per expert).
int launch_tile_gateup(const GemmArgs& a, int tile_rows, hipStream_t st);
int launch_tile_down(const GemmArgs& a, int tile_rows, hipStream_t st);
int tile_down_ksplit(int Kdim);   // K parts of the down projection when tile_rows == 64
int pick_tile_shape(int rows, int N, int Kdim, bool gateup, bool allow_kcut, bool leave_room);   // one weight set, known rows
// Streaming kernels that stage the weights through wave-private LDS rings (whole-line requests).
int launch_stream_lds_gateup(const GemmArgs& a, hipStream_t st);
int launch_stream_lds_down(const GemmArgs& a, hipStream_t st);

}  // namespace moe
