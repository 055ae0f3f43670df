/*
 * moe.h - C ABI of the MI355X (gfx950) MoE-layer forward library.
 *
 * The calls follow the split the FaaSMoE paper makes (Sec. 3 "Architecture"): a control plane
 * (the orchestrator: gating, construction of one micro-batch per expert block, aggregation) and
 * an execution plane (expert blocks: stateless functions that hold a configurable number of
 * experts and compute on the tokens they are handed).  moe_route, moe_permute and moe_combine
 * are the control plane; moe_expert_group_forward is one expert-block invocation;
 * moe_shared_forward runs the model's shared experts (Sec. 5 "Model Selection": 60 routed and
 * 4 shared experts per layer), which no routed-expert block contains.
 *
 * Conventions for every call
 *  - Every pointer is a DEVICE pointer owned by the caller.  The library allocates nothing,
 *    frees nothing and keeps no pointer after the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *    kernels on it; they never synchronise and never read device memory on the host.
 *  - Activations and weights are bf16 (16-bit, upper half of an IEEE fp32), row-major, innermost
 *    dimension contiguous; accumulation is fp32.  Indices are int32.
 *  - Return value: MOE_OK (0), or a negative MOE_ERR_* code, in which case nothing was enqueued.
 *  - No hidden state: the result of a call is a function of its arguments alone (Sec. 3: expert
 *    blocks are stateless; the orchestrator keeps no cross-request state), so a call may be
 *    repeated, and calls on disjoint outputs may be issued in any order, on several streams and
 *    from several host threads (the library keeps nothing but a per-device note that a kernel's LDS
 *    limit has been raised, set atomically).
 *  - Shape limits: H, I, Is multiples of 64; 1 <= K <= 16; K <= E <= 256; T*K < 2^31 / max(H,I);
 *    moe_route, moe_route_segments and moe_residual_norm: H <= 8192 (a token row lives in registers).
 *
 * Symbols: T tokens, H hidden size, E routed experts, K experts per token, P = T*K
 * (token, slot) pairs, I routed-expert intermediate size, Is shared-expert intermediate size.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK 0
#define MOE_ERR_NULL (-1)      /* a required pointer is NULL */
#define MOE_ERR_SHAPE (-2)     /* a size or an expert range is outside the limits above */
#define MOE_ERR_WORKSPACE (-3) /* workspace_bytes is smaller than the call needs */
#define MOE_ERR_LAUNCH (-4)    /* the HIP runtime refused a kernel launch */

/* Human-readable text for a status code (static storage, never NULL). */
const char* moe_status_string(int status);

/* Id of the sources this library was built from: SHA-256, as hex text, over the kernel sources and
 * this header (static storage, never NULL; "unstamped" for a build that did not pass one).  Callers
 * that keep measurements of the kernels (profiler counters) store it beside them. */
const char* moe_build_id(void);

/*
 * Gating (Sec. 2.1: the gating network selects the top-k experts per token; Sec. 3: it runs in
 * the orchestrator).
 *   logit[t,e] = <x[t,:], Wr[e,:]> + bias[e]      fp32, in a fixed summation order (below)
 *   p[t,:]     = softmax over e of logit[t,:]      fp32
 *   topk_ids[t,0..K-1] = the K experts with the largest logits, descending; equal logits (and
 *                        -0 / +0) go to the lower expert id
 *   topk_w[t,j] = p[t, topk_ids[t,j]], divided by their sum over j when renorm != 0
 * Summation order of the dot product: element h belongs to partial sum (h/8) mod 64; each
 * partial takes its elements in ascending h by fused multiply-add starting from +0; the 64
 * partials are folded by a butterfly a[j] += a[j xor s] for s = 1,2,4,8,16,32; the bias is added
 * last.  bf16 products are exact in fp32, so the logits are reproducible bit for bit.
 * Row t of the outputs depends on row t of x only, so slices of a batch (one per tenant, each
 * with its own bias) may be routed by separate calls.
 *   x [T,H] bf16; Wr [E,H] bf16; bias [E] fp32 or NULL; topk_ids [T,K] int32; topk_w [T,K] fp32.
 * T == 0 is a no-op.
 */
int moe_route(const void* x, const void* Wr, const float* bias, int T, int H, int E, int K,
              int renorm, int32_t* topk_ids, float* topk_w, void* stream);

/*
 * Gating of a batch assembled from several tenants' requests by a shared orchestrator (Sec. 3:
 * the Shared orchestrator serves all tenants and batches across them): the same computation as
 * moe_route, with one bias row per segment of the batch.  Token t of segment s, seg_offsets[s] <= t
 * < seg_offsets[s+1], is routed with bias_rows[s,:]; the result equals n_seg calls of moe_route on
 * the slices, bit for bit, in one launch.
 *   bias_rows [n_seg,E] fp32 (device); seg_offsets [n_seg+1] int32 (device), ascending, first 0,
 *   last T (tokens at or past the last bound, if any, take the last row); 1 <= n_seg <= 4096.
 * The bounds are read on the device and not validated; the other arguments as in moe_route.
 */
int moe_route_segments(const void* x, const void* Wr, const float* bias_rows, const int32_t* seg_offsets,
                       int n_seg, int T, int H, int E, int K, int renorm, int32_t* topk_ids,
                       float* topk_w, void* stream);

/*
 * Micro-batch construction (Sec. 3: after gating the orchestrator builds one routing request per
 * expert block; Sec. 4.1 "token-level micro-batching": a block is invoked once per layer pass, on
 * the batch of every token that gating sent to one of its experts).  A stable counting sort of the
 * P pairs p = t*K + j by expert id:
 *   expert_offsets[e] .. expert_offsets[e+1]-1 are the rows of expert e (expert_offsets[E] = P);
 *   row_of_pair[p] = row that pair p lands on; src_of_row[r] = the pair on row r (its inverse);
 *   inside one expert the rows keep ascending p;  Xp[r,:] = x[src_of_row[r] / K, :].
 * The batch of an expert block [lo,hi) is therefore the contiguous row range
 * expert_offsets[lo] .. expert_offsets[hi]-1 of Xp.
 *   topk_ids [T,K] int32 with values in [0,E) (values outside are not detected);
 *   x [T,H] bf16; expert_offsets [E+1]; src_of_row [P]; row_of_pair [P]; Xp [P,H] bf16.
 * Xp may be NULL: then only the three index arrays are written (x is not read and may be NULL
 * too), for callers that hand the block invocations x and src_of_row instead of a permuted copy
 * (moe_expert_group_forward_gather).
 * workspace: moe_permute_workspace_bytes(T, K, E) bytes of scratch (pairs of each expert per chunk of
 * 64 pairs); contents are meaningless after the call.
 */
int moe_permute(const int32_t* topk_ids, const void* x, int T, int H, int E, int K,
                int32_t* expert_offsets, int32_t* src_of_row, int32_t* row_of_pair, void* Xp,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * moe_permute for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same sort
 * with the same outputs, bit for bit; the table that moe_permute keeps in `workspace` lives in a
 * buffer inside the library instead (a static device array of MOE_PERMUTE_STATIC_SCRATCH_BYTES
 * that each GPU holds until the process ends).  The call allocates and frees nothing.
 * Limit: ((T*K + 63) / 64) * E * 4 <= MOE_PERMUTE_STATIC_SCRATCH_BYTES (e.g. T*K <= 65 536 pairs at
 * E = 256, 279 552 at E = 60); beyond it the call returns MOE_ERR_WORKSPACE and enqueues nothing.
 * All calls on one GPU share that buffer: two calls that overlap in time on the same GPU (different
 * streams) race on it and give undefined index arrays; calls ordered on one stream, or on different
 * GPUs, are safe.  The buffer needs no clearing between calls.  Arguments as for moe_permute.
 */
#define MOE_PERMUTE_STATIC_SCRATCH_BYTES (1 << 20)
int moe_permute_static(const int32_t* topk_ids, const void* x, int T, int H, int E, int K,
                       int32_t* expert_offsets, int32_t* src_of_row, int32_t* row_of_pair, void* Xp,
                       void* stream);

/*
 * One expert-block invocation (Sec. 3: an expert block packages a configurable number of
 * experts behind one function and computes statelessly on the tokens assigned to it).
 * For every expert e in [group_lo, group_hi) and every row r of that expert:
 *   h[r,:]  = silu(Xp[r,:] . Wg[e]^T) * (Xp[r,:] . Wu[e]^T)        silu(a) = a / (1 + exp(-a))
 *   Yp[r,:] = h[r,:] . Wd[e]^T
 * The gate weight is NOT applied here (the block sees tokens only); moe_combine applies it.
 * Only rows expert_offsets[group_lo] .. expert_offsets[group_hi]-1 of Yp are written; experts
 * without rows cost nothing and their weights are not read.  The result for a row does not
 * depend on how [0,E) is cut into blocks (Sec. 3: block size does not change model semantics).
 *   Xp [P,H] bf16; expert_offsets [E+1] int32 ON THE DEVICE (read by the kernels);
 *   Wg, Wu [E,I,H] bf16; Wd [E,H,I] bf16 (the full tensors, not the block's slice);
 *   Yp [P,H] bf16.
 * Guaranteed: of the three weight tensors a call dereferences only the slices of experts in
 * [group_lo, group_hi) that have rows, i.e. bytes [e*I*H*2, (e+1)*I*H*2) past each base pointer
 * for those e.  A caller that keeps only a block's weights on the device (on-demand residency,
 * Sec. 3) may therefore pass base pointers moved back by group_lo experts from a buffer holding
 * just that block; the same holds for the gather and the id-list forms below.
 * workspace: moe_expert_workspace_bytes(P, I) bytes, holding h (bf16 [P,I]).  Blocks that run
 * concurrently may share one workspace: each touches only its own rows.
 */
int moe_expert_group_forward(int group_lo, int group_hi, const void* Xp,
                             const int32_t* expert_offsets, const void* Wg, const void* Wu,
                             const void* Wd, int P, int H, int E, int I, void* Yp,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * Shared experts (Sec. 5: 4 shared experts per layer, here as one SwiGLU FFN whose
 * intermediate size Is is the four concatenated) on every token, and the raw logit of their
 * sigmoid gate:
 *   S[t,:] = ( silu(x[t,:] . Wsg^T) * (x[t,:] . Wsu^T) ) . Wsd^T ;   sg[t] = <x[t,:], wgate>
 *   x [T,H]; Wsg, Wsu [Is,H]; Wsd [H,Is]; wgate [H] (bf16) or NULL (then sg is not written);
 *   S [T,H] bf16; sg [T] fp32.
 * workspace: moe_shared_workspace_bytes(T, H, Is) bytes (h as bf16 [T,Is]; for T <= 512 also the
 * fp32 partial sums of a down projection that is cut along K).
 */
int moe_shared_forward(const void* x, const void* Wsg, const void* Wsu, const void* Wsd,
                       const void* wgate, int T, int H, int Is, void* S, float* sg,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Aggregation (Sec. 3 and Sec. 4.2: the orchestrator aggregates the tokens that come back from
 * the expert blocks):
 *   out[t,:] = sum over j = 0..K-1, in that order, of topk_w[t,j] * Yp[row_of_pair[t*K+j],:]
 *              + sigmoid(sg[t]) * S[t,:]                       (fp32, rounded once to bf16)
 * S and sg may both be NULL (no shared expert).  The sum order is fixed, so `out` is bitwise
 * independent of how the experts were cut into blocks and of the order the blocks ran in.
 *   Yp [T*K,H] bf16; row_of_pair [T*K]; topk_w [T,K] fp32; S [T,H] bf16; sg [T] fp32;
 *   out [T,H] bf16.
 */
int moe_combine(const void* Yp, const int32_t* row_of_pair, const float* topk_w, const void* S,
                const float* sg, int T, int H, int K, void* out, void* stream);

/*
 * Step between two MoE layers when layers are chained without the attention blocks that sit
 * between them in the model (Sec. 3: the orchestrator runs, per transformer layer, attention, then
 * gating and the expert blocks; attention is outside this library):
 *   u = x[t,:] + y[t,:] (fp32);   out[t,:] = bf16( u / sqrt(mean_h(u^2) + eps) )     no learned scale
 * It keeps activations bounded over a stack of layers.  x, y, out [T,H] bf16; out may alias x or y;
 * H <= 8192.
 */
int moe_residual_norm(const void* x, const void* y, int T, int H, float eps, void* out, void* stream);

/*
 * The same invocation without a permuted copy of the tokens: row r of the block's batch is read
 * as x[src_of_row[r] / K, :] while the first kernel stages it (the gather of the micro-batch
 * construction, folded into the consumer).  Same result, bit for bit, as
 * moe_expert_group_forward on Xp.  policy: 0 = the library picks the kernel shape; other values are
 * the tuning knob described in moe_tuning.h.
 *   x [T,H] bf16 with T = P / K; src_of_row [P] int32 on the device, values in [0,P).
 */
int moe_expert_group_forward_gather(int group_lo, int group_hi, const void* x,
                                    const int32_t* src_of_row, int K,
                                    const int32_t* expert_offsets, const void* Wg, const void* Wu,
                                    const void* Wd, int P, int H, int E, int I, void* Yp,
                                    void* workspace, size_t workspace_bytes, int policy,
                                    void* stream);

/*
 * A block invocation that also hosts the model's shared experts (Sec. 5 "Model Selection": 4 shared
 * experts per layer beside the 60 routed ones; Sec. 3: a block packages a configurable set of
 * experts behind one function).  The shared FFN of intermediate size Is is taken as Is / I experts
 * of the routed experts' size I (gate/up rows [s*I, (s+1)*I) of Wsg, Wsu and columns [s*I, (s+1)*I)
 * of Wsd are shared expert s), each applied to every token.  Their tiles join the routed experts'
 * tiles in the same two kernel launches, so the launch has no idle tail between the routed and the
 * shared part and compute-bound shared tiles run beside memory-bound tiles of small experts.
 *   Yp rows of the experts in [group_lo, group_hi): as moe_expert_group_forward_gather, bit for bit;
 *   S_parts[s,t,:] = FFN of shared expert s on x[t,:]  (bf16 [n_sets,T,H]; their sum over s is the
 *                    shared FFN's output, which moe_combine_parts forms in fp32);
 *   sg[t] = <x[t,:], wgate> (fp32) when wgate is not NULL.
 * Supported when moe_fused_shared_sets(T,H,E,K,I,Is) returns n_sets > 0: Is a multiple of I with
 * at most MOE_SHARED_SETS_MAX sets, E + n_sets <= 256, and a batch large enough for the MFMA tile
 * kernels (more than 26 rows per routed expert on average); otherwise MOE_ERR_SHAPE, and the
 * caller uses moe_expert_group_forward(_gather) and moe_shared_forward.  When the routed experts
 * are cut into several blocks, one of the calls carries the shared experts and the others are
 * plain block calls.  x [T,H]; src_of_row [T*K]; weights as in the separate calls.
 * workspace: moe_fused_workspace_bytes(T, K, I, Is) bytes.  policy: 0, or one of 3, 4, 5, 10, 11 and the
 * 0x100 / 0x200 bits of moe_tuning.h.
 */
#define MOE_SHARED_SETS_MAX 8
int moe_fused_shared_sets(int T, int H, int E, int K, int I, int Is);
size_t moe_fused_workspace_bytes(int T, int K, int I, int Is);
int moe_expert_group_forward_fused(int group_lo, int group_hi, const void* x, const int32_t* src_of_row,
                                   int K, const int32_t* expert_offsets, const void* Wg,
                                   const void* Wu, const void* Wd, const void* Wsg, const void* Wsu,
                                   const void* Wsd, const void* wgate, int T, int H, int E, int I,
                                   int Is, void* Yp, void* S_parts, float* sg, void* workspace,
                                   size_t workspace_bytes, int policy, void* stream);

/*
 * moe_combine for shared-expert outputs that come as n_parts separate tensors (S_parts
 * [n_parts,T,H] bf16, from moe_expert_group_forward_fused):
 *   out[t,:] = sum_j topk_w[t,j] * Yp[row_of_pair[t*K+j],:]
 *              + sigmoid(sg[t]) * (S_parts[0,t,:] + S_parts[1,t,:] + ...)     (fp32, parts in ascending
 *   order, one rounding to bf16).  1 <= n_parts <= MOE_SHARED_SETS_MAX; S_parts and sg are required.
 */
int moe_combine_parts(const void* Yp, const int32_t* row_of_pair, const float* topk_w,
                      const void* S_parts, int n_parts, const float* sg, int T, int H, int K,
                      void* out, void* stream);

/*
 * An expert block given as a list of expert ids instead of an id range (Sec. 5 names adaptive,
 * hot-expert-aware block formation as the next step: blocks formed by load need not be ranges).
 * expert_ids [n_ids] int32 ON THE DEVICE, distinct values in [0,E) (not checked); the call
 * computes exactly the rows of those experts, with the same result for each row as any other
 * block cut.  tokens is Xp [P,H] when src_of_row is NULL, else x [P/K,H] read through
 * src_of_row as in moe_expert_group_forward_gather.  policy: 0, or a value of moe_tuning.h.
 */
int moe_expert_list_forward(const int32_t* expert_ids, int n_ids, const void* tokens,
                            const int32_t* src_of_row, int K, const int32_t* expert_offsets,
                            const void* Wg, const void* Wu, const void* Wd, int P, int H, int E,
                            int I, void* Yp, void* workspace, size_t workspace_bytes, int policy,
                            void* stream);

/* Workspace sizes in bytes (multiples of 256). */
size_t moe_permute_workspace_bytes(int T, int K, int E);
size_t moe_expert_workspace_bytes(int P, int I);
size_t moe_shared_workspace_bytes(int T, int H, int Is);
/* Largest of the three: one buffer of this size serves every call of a layer issued on one
 * stream. */
size_t moe_workspace_bytes(int T, int H, int E, int K, int I, int Is);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
