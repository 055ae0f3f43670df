// C entry points of the MoE-layer library: argument checks and the choice of kernel shapes.
// Semantics of every call are stated in include/moe.h.
#include <atomic>
#include "../../include/moe.h"
#include "../../include/moe_tuning.h"
#include "common.h"

using namespace moe;

namespace {

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

bool dims_ok(int H) { return H > 0 && H % 64 == 0; }

// Which kernels serve an FFN with `mean_rows` expected rows per expert.  The choice uses only
// layer-wide sizes (never the block bounds), so a row's result does not depend on the block cut.
// policy: 0 = automatic; 3 and 5 = MFMA tiles of 128 token rows by 256 weight rows; 4 = 256 by 256;
//         8 = 128 by 64, the down projection cut along K (few rows in all, one weight set);
//         9 = weight streaming through wave-private LDS rings (few rows per expert);
//         10 = 128 by 128; 11 = 160 by 256.  Any other number is refused.
// Bits 8 and 9 of the policy word restrict a call to one of its two kernels (0x100: gate/up
// only, 0x200: down projection only), so that each can be timed on its own.  Bit 10 (0x400, shared
// expert with automatic shapes): its first kernel takes no tile shape that fills a CU completely,
// so that small kernels of other streams (gating, micro-batch construction) run beside it.
constexpr int SHARED_SMALL_T = 512;     // up to here the workspace has room for a K-cut down projection
constexpr int SHARED_KPARTS_MAX = 8;    // parts of its down projection along K

struct Plan { bool valid; bool stream; int tile_rows; bool do_gateup; bool do_down; };
Plan make_plan(int mean_rows, int n_experts_layer, int policy_word) {
  Plan p{};
  const int phase = (policy_word >> 8) & 3;
  const int policy = policy_word & 0xff;
  p.valid = (policy_word & ~0x7ff) == 0;
  p.do_gateup = phase == 0 || (phase & 1);
  p.do_down = phase == 0 || (phase & 2);
  switch (policy) {
    case 0: break;
    case 3: p.tile_rows = 128; return p;
    case 4: p.tile_rows = 256; return p;
    case 5: p.tile_rows = 129; return p;
    case 8: p.tile_rows = 64; return p;
    case 9: p.stream = true; return p;
    case 10: p.tile_rows = 130; return p;
    case 11: p.tile_rows = 160; return p;
    default: p.valid = false; return p;
  }
  // One weight set on all rows (the shared expert): MFMA tiles whose shape each kernel picks from
  // its tile count (pick_tile_shape).  Routed experts, measured with cold caches at the Qwen shape:
  // streaming through LDS rings wins up to a mean of about 26 rows per expert (T = 384), the MFMA
  // tiles beyond (their height picked from the layer-wide mean).
  const bool few_experts = n_experts_layer < 16;
  p.stream = !few_experts && mean_rows <= 26;
  p.tile_rows = 0;
  return p;
}

int ffn_forward(const GemmArgs& gu, const GemmArgs& dn, const Plan& p, hipStream_t st) {
  int rc = 0;
  if (p.stream) {
    if (p.do_gateup && (rc = launch_stream_lds_gateup(gu, st)) != 0) return rc;
    if (p.do_down) rc = launch_stream_lds_down(dn, st);
    return rc;
  }
  if (p.do_gateup && (rc = launch_tile_gateup(gu, p.tile_rows, st)) != 0) return rc;
  if (p.do_down) rc = launch_tile_down(dn, p.tile_rows, st);
  return rc;
}

int expert_group_forward_impl(int group_lo, int group_hi, const int32_t* ids, const void* A, const int32_t* gather,
                              int gather_div,
                              const int32_t* expert_offsets, const void* Wg, const void* Wu, const void* Wd, int P,
                              int H, int E, int I, void* Yp, void* workspace, size_t workspace_bytes, int policy,
                              void* stream) {
  if (P < 0 || !dims_ok(H) || !dims_ok(I) || E < 1 || E > 256) return MOE_ERR_SHAPE;
  if (group_lo < 0 || group_hi > E || group_lo >= group_hi) return MOE_ERR_SHAPE;
  if ((long long)P * (H > I ? H : I) >= (1ll << 31)) return MOE_ERR_SHAPE;
  if (P == 0) return MOE_OK;
  if (!A || !expert_offsets || !Wg || !Wu || !Wd || !Yp || !workspace) return MOE_ERR_NULL;
  if (workspace_bytes < (size_t)P * (size_t)I * 2) return MOE_ERR_WORKSPACE;   // h, bf16 [P,I]
  const int mean_rows = (P + E - 1) / E;
  const Plan plan = make_plan(mean_rows, E, policy);
  if (!plan.valid) return MOE_ERR_SHAPE;
  GemmArgs gu{};
  gu.A = (const bf16_t*)A; gu.B0 = (const bf16_t*)Wg; gu.B1 = (const bf16_t*)Wu; gu.C = (bf16_t*)workspace;
  gu.offsets = expert_offsets; gu.lo = group_lo; gu.hi = group_hi; gu.ids = ids; gu.rows_fixed = 0; gu.rows_total = P;
  gu.mean_rows = mean_rows; gu.N = I; gu.Kdim = H;
  GemmArgs dn = gu;
  gu.gather = gather; gu.gather_div = gather_div;   // only the first kernel reads token rows
  dn.A = (const bf16_t*)workspace; dn.B0 = (const bf16_t*)Wd; dn.B1 = nullptr; dn.C = (bf16_t*)Yp;
  dn.N = H; dn.Kdim = I;
  return ffn_forward(gu, dn, plan, (hipStream_t)stream);
}
}  // namespace

// Scratch memory of moe_permute_static: the per-chunk expert histogram of the counting sort, which
// moe_permute keeps in the caller's workspace.  Every GPU the library runs on holds its own copy of
// the array at its own address until the process ends.  In host code the array's name is not a
// device address: the address on the current device is asked for once per device
// (hipGetSymbolAddress) and kept; only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[MOE_PERMUTE_STATIC_SCRATCH_BYTES];
static std::atomic<void*> scratch_on_device[64];   // by device id

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MOE_ERR_LAUNCH;
  void* p = scratch_on_device[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return MOE_ERR_LAUNCH;
    scratch_on_device[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return MOE_OK;
}

#ifndef MOE_BUILD_ID
#define MOE_BUILD_ID "unstamped"
#endif

extern "C" {

const char* moe_build_id(void) { return MOE_BUILD_ID; }

int moe_tile_clock_buffer(int64_t* clocks, int workgroups) {
  if (clocks != nullptr && workgroups < 1) return MOE_ERR_SHAPE;
  moe::set_tile_clock_buffer(reinterpret_cast<long long*>(clocks), clocks == nullptr ? 0 : workgroups);
  return MOE_OK;
}

int moe_probe_mfma(const void* operands, size_t operand_bytes, int iters, int workgroups, int64_t* clocks, void* stream) {
  if (operands == nullptr || clocks == nullptr) return MOE_ERR_NULL;
  if (operand_bytes < MOE_PROBE_OPERAND_BYTES || iters < 1 || iters > (1 << 20) || workgroups < 1 || workgroups > 65535)
    return MOE_ERR_SHAPE;
  return moe::launch_mfma_probe(operands, iters, workgroups, reinterpret_cast<long long*>(clocks), (hipStream_t)stream) == 0
             ? MOE_OK : MOE_ERR_LAUNCH;
}

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_NULL: return "a required pointer is NULL";
    case MOE_ERR_SHAPE: return "a size or an expert range is outside the supported limits";
    case MOE_ERR_WORKSPACE: return "workspace too small";
    case MOE_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

size_t moe_permute_workspace_bytes(int T, int K, int E) {
  if (T <= 0 || K <= 0 || E <= 0) return 0;
  const size_t chunks = ((size_t)T * (size_t)K + 63) / 64;   // pairs of each expert per 64-pair chunk
  return align256(chunks * (size_t)E * 4);
}
size_t moe_expert_workspace_bytes(int P, int I) {
  if (P <= 0 || I <= 0) return 0;
  return align256((size_t)P * (size_t)I * 2);
}
// h [T,Is] bf16, then (small batches only) the fp32 partial outputs of a down projection cut along K
size_t moe_shared_workspace_bytes(int T, int H, int Is) {
  if (T <= 0 || H <= 0 || Is <= 0) return 0;
  size_t n = align256((size_t)T * (size_t)Is * 2);
  if (T <= SHARED_SMALL_T) n += (size_t)SHARED_KPARTS_MAX * (size_t)T * (size_t)H * 4;
  return n;
}
size_t moe_workspace_bytes(int T, int H, int E, int K, int I, int Is) {
  size_t a = moe_permute_workspace_bytes(T, K, E);
  size_t b = moe_expert_workspace_bytes(T * K, I);
  size_t c = moe_shared_workspace_bytes(T, H, Is);
  size_t m = a > b ? a : b;
  return m > c ? m : c;
}

int moe_route(const void* x, const void* Wr, const float* bias, int T, int H, int E, int K, int renorm,
              int32_t* topk_ids, float* topk_w, void* stream) {
  if (T < 0 || !dims_ok(H) || H > 8192 || E < 1 || E > 256 || K < 1 || K > 16 || K > E) return MOE_ERR_SHAPE;
  if (T == 0) return MOE_OK;
  if (!x || !Wr || !topk_ids || !topk_w) return MOE_ERR_NULL;
  return launch_route(x, Wr, bias, nullptr, 0, T, H, E, K, renorm, topk_ids, topk_w, (hipStream_t)stream);
}

int moe_route_segments(const void* x, const void* Wr, const float* bias_rows, const int32_t* seg_offsets, int n_seg,
                       int T, int H, int E, int K, int renorm, int32_t* topk_ids, float* topk_w, void* stream) {
  if (T < 0 || !dims_ok(H) || H > 8192 || E < 1 || E > 256 || K < 1 || K > 16 || K > E) return MOE_ERR_SHAPE;
  if (n_seg < 1 || n_seg > 4096) return MOE_ERR_SHAPE;
  if (T == 0) return MOE_OK;
  if (!x || !Wr || !bias_rows || !seg_offsets || !topk_ids || !topk_w) return MOE_ERR_NULL;
  return launch_route(x, Wr, bias_rows, seg_offsets, n_seg, T, H, E, K, renorm, topk_ids, topk_w,
                      (hipStream_t)stream);
}

int moe_permute(const int32_t* topk_ids, const void* x, int T, int H, int E, int K, int32_t* expert_offsets,
                int32_t* src_of_row, int32_t* row_of_pair, void* Xp, void* workspace, size_t workspace_bytes,
                void* stream) {
  if (T < 0 || !dims_ok(H) || E < 1 || E > 256 || K < 1 || K > 16 || K > E) return MOE_ERR_SHAPE;
  if ((long long)T * K * H >= (1ll << 31)) return MOE_ERR_SHAPE;
  if (!expert_offsets) return MOE_ERR_NULL;
  if (T > 0 && (!topk_ids || !src_of_row || !row_of_pair || !workspace)) return MOE_ERR_NULL;
  if (T > 0 && Xp && !x) return MOE_ERR_NULL;   // Xp == NULL: index arrays only, x is not read
  if (T > 0 && workspace_bytes < (((size_t)T * K + 63) / 64) * (size_t)E * 4) return MOE_ERR_WORKSPACE;
  return launch_permute(topk_ids, x, T, H, E, K, expert_offsets, src_of_row, row_of_pair, Xp, workspace,
                        (hipStream_t)stream);
}

int moe_permute_static(const int32_t* topk_ids, const void* x, int T, int H, int E, int K, int32_t* expert_offsets,
                       int32_t* src_of_row, int32_t* row_of_pair, void* Xp, void* stream) {
  if (T < 0 || !dims_ok(H) || E < 1 || E > 256 || K < 1 || K > 16 || K > E) return MOE_ERR_SHAPE;
  if ((long long)T * K * H >= (1ll << 31)) return MOE_ERR_SHAPE;
  if (!expert_offsets) return MOE_ERR_NULL;
  if (T > 0 && (!topk_ids || !src_of_row || !row_of_pair)) return MOE_ERR_NULL;
  if (T > 0 && Xp && !x) return MOE_ERR_NULL;
  if ((((size_t)T * K + 63) / 64) * (size_t)E * 4 > (size_t)MOE_PERMUTE_STATIC_SCRATCH_BYTES) return MOE_ERR_WORKSPACE;
  void* table = nullptr;
  const int rc = static_scratch(&table);
  if (rc != MOE_OK) return rc;
  // (the histogram kernel writes every table entry it later reads, so what an earlier call left
  // behind needs no clearing)
  return launch_permute(topk_ids, x, T, H, E, K, expert_offsets, src_of_row, row_of_pair, Xp, table,
                        (hipStream_t)stream);
}

int moe_expert_group_forward_ex(int group_lo, int group_hi, const void* Xp, const int32_t* expert_offsets,
                                const void* Wg, const void* Wu, const void* Wd, int P, int H, int E, int I,
                                void* Yp, void* workspace, size_t workspace_bytes, int policy, void* stream) {
  return expert_group_forward_impl(group_lo, group_hi, nullptr, Xp, nullptr, 1, expert_offsets, Wg, Wu, Wd, P, H, E, I, Yp,
                                   workspace, workspace_bytes, policy, stream);
}

int moe_expert_group_forward_gather(int group_lo, int group_hi, const void* x, const int32_t* src_of_row, int K,
                                    const int32_t* expert_offsets, const void* Wg, const void* Wu, const void* Wd,
                                    int P, int H, int E, int I, void* Yp, void* workspace, size_t workspace_bytes,
                                    int policy, void* stream) {
  if (K < 1 || K > 16 || (P > 0 && P % K != 0)) return MOE_ERR_SHAPE;
  if (P > 0 && !src_of_row) return MOE_ERR_NULL;
  return expert_group_forward_impl(group_lo, group_hi, nullptr, x, src_of_row, K, expert_offsets, Wg, Wu, Wd, P, H, E, I,
                                   Yp, workspace, workspace_bytes, policy, stream);
}

int moe_expert_list_forward(const int32_t* expert_ids, int n_ids, const void* tokens, const int32_t* src_of_row, int K,
                            const int32_t* expert_offsets, const void* Wg, const void* Wu, const void* Wd, int P,
                            int H, int E, int I, void* Yp, void* workspace, size_t workspace_bytes, int policy,
                            void* stream) {
  if (n_ids < 1 || n_ids > E) return MOE_ERR_SHAPE;
  if (!expert_ids) return MOE_ERR_NULL;
  if (src_of_row && (K < 1 || K > 16 || (P > 0 && P % K != 0))) return MOE_ERR_SHAPE;
  // positions [0, n_ids) of the list take the place of the id range; the range checks see [0, n_ids)
  return expert_group_forward_impl(0, n_ids, expert_ids, tokens, src_of_row, src_of_row ? K : 1, expert_offsets, Wg, Wu,
                                   Wd, P, H, E, I, Yp, workspace, workspace_bytes, policy, stream);
}

int moe_fused_shared_sets(int T, int H, int E, int K, int I, int Is) {
  if (T <= 0 || K < 1 || E < 1 || I <= 0 || Is <= 0 || !dims_ok(H) || !dims_ok(I) || Is % I != 0) return 0;
  const int ns = Is / I;
  if (ns > MOE_SHARED_SETS_MAX || E + ns > 256) return 0;
  const long long P = (long long)T * K;
  if ((P + (long long)ns * T) * (H > I ? H : I) >= (1ll << 31)) return 0;
  const Plan plan = make_plan((int)((P + E - 1) / E), E, 0);
  return plan.stream ? 0 : ns;     // batches served by weight streaming keep the separate calls
}

size_t moe_fused_workspace_bytes(int T, int K, int I, int Is) {
  if (T <= 0 || K <= 0 || I <= 0 || Is <= 0 || Is % I != 0) return 0;
  return align256(((size_t)T * K + (size_t)(Is / I) * T) * (size_t)I * 2);
}

int moe_expert_group_forward_fused(int group_lo, int group_hi, const void* x, const int32_t* src_of_row, int K,
                                   const int32_t* expert_offsets, const void* Wg, const void* Wu, const void* Wd,
                                   const void* Wsg, const void* Wsu, const void* Wsd, const void* wgate, int T, int H,
                                   int E, int I, int Is, void* Yp, void* S_parts, float* sg, void* workspace,
                                   size_t workspace_bytes, int policy, void* stream) {
  if (T < 0 || K < 1 || K > 16 || !dims_ok(H) || !dims_ok(I) || E < 1 || E > 256) return MOE_ERR_SHAPE;
  if (group_lo < 0 || group_hi > E || group_lo >= group_hi) return MOE_ERR_SHAPE;
  if (T == 0) return MOE_OK;
  const int ns = moe_fused_shared_sets(T, H, E, K, I, Is);
  if (ns == 0) return MOE_ERR_SHAPE;
  if (!x || !src_of_row || !expert_offsets || !Wg || !Wu || !Wd || !Wsg || !Wsu || !Wsd || !Yp || !S_parts || !workspace)
    return MOE_ERR_NULL;
  if (wgate && !sg) return MOE_ERR_NULL;
  const int P = T * K;
  const int rows = P + ns * T;
  if (workspace_bytes < (size_t)rows * (size_t)I * 2) return MOE_ERR_WORKSPACE;   // h of the routed rows, then of every shared set
  const int mean_rows = (P + E - 1) / E;
  const Plan plan = make_plan(mean_rows, E, policy);
  if (!plan.valid || plan.stream || plan.tile_rows == 64) return MOE_ERR_SHAPE;
  GemmArgs gu{};
  gu.A = (const bf16_t*)x; gu.B0 = (const bf16_t*)Wg; gu.B1 = (const bf16_t*)Wu; gu.C = (bf16_t*)workspace;
  gu.offsets = expert_offsets; gu.lo = group_lo; gu.hi = group_hi; gu.ids = nullptr; gu.rows_total = rows;
  gu.mean_rows = mean_rows; gu.N = I; gu.Kdim = H;
  gu.n_shared = ns; gu.shared_rows = T; gu.rows_routed = P;
  GemmArgs dn = gu;
  gu.gather = src_of_row; gu.gather_div = K;
  gu.Bs0 = (const bf16_t*)Wsg; gu.Bs1 = (const bf16_t*)Wsu; gu.shared_b_step = (long)I * H; gu.ldb_shared = H;
  gu.As = (const bf16_t*)x;                 // set s of the shared expert reads the tokens in order
  dn.A = (const bf16_t*)workspace; dn.B0 = (const bf16_t*)Wd; dn.B1 = nullptr; dn.C = (bf16_t*)Yp;
  dn.N = H; dn.Kdim = I;
  dn.Bs0 = (const bf16_t*)Wsd; dn.shared_b_step = I; dn.ldb_shared = Is;   // set s: columns [s*I, (s+1)*I) of Wsd [H,Is]
  dn.Cs = (bf16_t*)S_parts;
  int rc = ffn_forward(gu, dn, plan, (hipStream_t)stream);
  if (rc != 0) return rc;
  if (wgate && plan.do_down) return launch_gate_dot(x, wgate, T, H, sg, (hipStream_t)stream);
  return MOE_OK;
}

int moe_expert_group_forward(int group_lo, int group_hi, const void* Xp, const int32_t* expert_offsets,
                             const void* Wg, const void* Wu, const void* Wd, int P, int H, int E, int I, void* Yp,
                             void* workspace, size_t workspace_bytes, void* stream) {
  return moe_expert_group_forward_ex(group_lo, group_hi, Xp, expert_offsets, Wg, Wu, Wd, P, H, E, I, Yp, workspace,
                                     workspace_bytes, 0, stream);
}

int moe_shared_forward_ex(const void* x, const void* Wsg, const void* Wsu, const void* Wsd, const void* wgate, int T,
                          int H, int Is, void* S, float* sg, void* workspace, size_t workspace_bytes, int policy,
                          void* stream) {
  if (T < 0 || !dims_ok(H) || !dims_ok(Is)) return MOE_ERR_SHAPE;
  if ((long long)T * (H > Is ? H : Is) >= (1ll << 31)) return MOE_ERR_SHAPE;
  if (T == 0) return MOE_OK;
  if (!x || !Wsg || !Wsu || !Wsd || !S || !workspace) return MOE_ERR_NULL;
  if (wgate && !sg) return MOE_ERR_NULL;
  if (workspace_bytes < (size_t)T * (size_t)Is * 2) return MOE_ERR_WORKSPACE;   // h, bf16 [T,Is]
  const Plan plan = make_plan(T, 1, policy);
  if (!plan.valid) return MOE_ERR_SHAPE;
  const size_t h_bytes = align256((size_t)T * (size_t)Is * 2);
  const size_t part_bytes = (size_t)tile_down_ksplit(Is) * (size_t)T * (size_t)H * 4;
  float* part = nullptr;
  if (!plan.stream && tile_down_ksplit(Is) > 1) {
    if (plan.tile_rows == 64) {          // asked for by the caller: the room must be there
      if (workspace_bytes < h_bytes + part_bytes) return MOE_ERR_WORKSPACE;
      part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + h_bytes);
    } else if (plan.tile_rows == 0 && T <= SHARED_SMALL_T) {   // automatic: sizes the helper reports include it
      if (workspace_bytes < h_bytes + part_bytes) return MOE_ERR_WORKSPACE;
      part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + h_bytes);
    }
  }
  GemmArgs gu{};
  gu.A = (const bf16_t*)x; gu.B0 = (const bf16_t*)Wsg; gu.B1 = (const bf16_t*)Wsu; gu.C = (bf16_t*)workspace;
  gu.offsets = nullptr; gu.lo = 0; gu.hi = 1; gu.rows_fixed = T; gu.rows_total = T; gu.mean_rows = T;
  gu.N = Is; gu.Kdim = H;
  GemmArgs dn = gu;
  dn.A = (const bf16_t*)workspace; dn.B0 = (const bf16_t*)Wsd; dn.B1 = nullptr; dn.C = (bf16_t*)S;
  dn.N = H; dn.Kdim = Is; dn.Cpart = part;
  gu.leave_room = (policy >> 10) & 1;
  int rc = ffn_forward(gu, dn, plan, (hipStream_t)stream);
  if (rc != 0) return rc;
  if (wgate && plan.do_down) return launch_gate_dot(x, wgate, T, H, sg, (hipStream_t)stream);
  return MOE_OK;
}

int moe_shared_forward(const void* x, const void* Wsg, const void* Wsu, const void* Wsd, const void* wgate, int T,
                       int H, int Is, void* S, float* sg, void* workspace, size_t workspace_bytes, void* stream) {
  return moe_shared_forward_ex(x, Wsg, Wsu, Wsd, wgate, T, H, Is, S, sg, workspace, workspace_bytes, 0, stream);
}

int moe_combine(const void* Yp, const int32_t* row_of_pair, const float* topk_w, const void* S, const float* sg,
                int T, int H, int K, void* out, void* stream) {
  if (T < 0 || !dims_ok(H) || K < 1 || K > 16) return MOE_ERR_SHAPE;
  if (T == 0) return MOE_OK;
  if (!Yp || !row_of_pair || !topk_w || !out) return MOE_ERR_NULL;
  if ((S == nullptr) != (sg == nullptr)) return MOE_ERR_NULL;
  return launch_combine(Yp, row_of_pair, topk_w, S, 1, sg, T, H, K, out, (hipStream_t)stream);
}

int moe_combine_parts(const void* Yp, const int32_t* row_of_pair, const float* topk_w, const void* S_parts, int n_parts,
                      const float* sg, int T, int H, int K, void* out, void* stream) {
  if (T < 0 || !dims_ok(H) || K < 1 || K > 16 || n_parts < 1 || n_parts > MOE_SHARED_SETS_MAX) return MOE_ERR_SHAPE;
  if (T == 0) return MOE_OK;
  if (!Yp || !row_of_pair || !topk_w || !out || !S_parts || !sg) return MOE_ERR_NULL;
  return launch_combine(Yp, row_of_pair, topk_w, S_parts, n_parts, sg, T, H, K, out, (hipStream_t)stream);
}

int moe_residual_norm(const void* x, const void* y, int T, int H, float eps, void* out, void* stream) {
  if (T < 0 || !dims_ok(H) || H > 8192 || !(eps >= 0.0f)) return MOE_ERR_SHAPE;
  if (T == 0) return MOE_OK;
  if (!x || !y || !out) return MOE_ERR_NULL;
  return launch_residual_norm(x, y, T, H, eps, out, (hipStream_t)stream);
}

}  // extern "C"
