/*
 * moe_tuning.h - the kernel-shape knob of the MoE-layer library, for measurement and tuning.
 *
 * Not needed to use the library: the calls of moe.h pick their kernels themselves (policy 0).  This
 * header documents the `policy` word that some of them accept, declares the two calls of moe.h
 * that exist in a second form only to take it (the values may change between builds), and two
 * measurement aids: the rate the matrix pipes sustain on given operand values (moe_probe_mfma) and
 * the clocks the MFMA tile kernels record about themselves on request (moe_tile_clock_buffer).
 */
#ifndef MOE_TUNING_H_
#define MOE_TUNING_H_

#include "moe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * moe_expert_group_forward and moe_shared_forward (moe.h) with the kernel shape picked by the caller
 * instead of by the library.  policy: 0 = automatic (what the plain calls use); 3 and 5 = MFMA tiles
 * of 128 token rows by 256 weight rows; 4 = 256 by 256; 8 = 128 by 64 (for the shared expert, whose
 * workspace has room for them, the down projection is cut into up to 8 parts along K whose fp32
 * partial sums a second kernel adds in ascending order; with policy 8 and T > 512 the shared call
 * needs the workspace of moe_shared_workspace_bytes plus 8*T*H*4 bytes); 9 = weight-streaming
 * kernels that stage the weights through wave-private LDS rings (few rows per expert); 10 = MFMA
 * tiles of 128 by 128; 11 = 160 by 256.  Any other number is refused with MOE_ERR_SHAPE.
 * Every policy computes the same function; results may differ in the last bf16 bit between
 * policies because the fp32 summation order differs.  Use one policy for all blocks of a layer.
 * Adding 0x100 to policy runs only the first kernel of the call (gate/up projections and SwiGLU
 * into the workspace), adding 0x200 only the second (down projection from the workspace, and for
 * the shared expert the gate logit): the two halves of one call, so each can be timed alone.
 * Adding 0x400 to the policy of moe_shared_forward_ex (automatic shapes) keeps its first kernel off
 * the one tile shape that occupies every register of a CU, so that small kernels issued on other
 * streams at the same time (gating, micro-batch construction) are not held up behind it.
 */
int moe_expert_group_forward_ex(int group_lo, int group_hi, const void* Xp,
                                const int32_t* expert_offsets, const void* Wg, const void* Wu,
                                const void* Wd, int P, int H, int E, int I, void* Yp,
                                void* workspace, size_t workspace_bytes, int policy, void* stream);
int moe_shared_forward_ex(const void* x, const void* Wsg, const void* Wsu, const void* Wsd,
                          const void* wgate, int T, int H, int Is, void* S, float* sg,
                          void* workspace, size_t workspace_bytes, int policy, void* stream);

/*
 * Measurement aid (no part of the paper's method): the rate the matrix pipes sustain on given operand
 * values with nothing else running, and the shader clock the chip holds meanwhile.  Dense MFMA work
 * on operands with realistic bit activity makes the chip lower its clock, so the published peak is
 * out of reach of any kernel on such data; a benchmark can state that ceiling beside its result.
 * operands: device, MOE_PROBE_OPERAND_BYTES bytes read as bf16 (eight 16-byte MFMA operand fragments
 * per lane of a 256-lane workgroup; any values: zeros, random numbers, rows of a real tensor).
 * Each of `workgroups` workgroups (one per compute unit up to the number of compute units) runs four
 * waves that each issue iters x 16 independent 32x32x16 bf16 MFMAs: 2 * 32*32*16 * 16 * iters * 4 *
 * workgroups floating-point operations per launch; the caller times the launch.
 * clocks: device, 2 * workgroups int64, written: per workgroup the ticks of the shader clock and of
 * the constant 100 MHz clock over its loop (their ratio x 100 MHz = the shader clock held).
 * Enqueues one kernel on `stream`, allocates nothing, does not synchronize.  Returns MOE_ERR_NULL,
 * MOE_ERR_SHAPE (operand_bytes too small, iters outside 1 ... 2^20, workgroups outside 1 ... 65535)
 * or MOE_ERR_LAUNCH.
 */
#define MOE_PROBE_OPERAND_BYTES 32768
int moe_probe_mfma(const void* operands, size_t operand_bytes, int iters, int workgroups,
                   int64_t* clocks, void* stream);

/*
 * Measurement aid: the shader clock the chip holds while the MFMA tile kernels of this library run.
 * After moe_tile_clock_buffer(clocks, n) every tile-kernel launch made by the calling host thread
 * (the grouped GEMMs of moe_expert_group_forward*, moe_expert_list_forward and moe_shared_forward
 * at prefill-sized batches; the weight-streaming kernels do not record) writes, for each of its
 * workgroups b < n, four int64 at clocks[4*b]: ticks of the shader clock and ticks of the constant
 * 100 MHz clock between the workgroup's start and end (ratio x 100 MHz = the clock held), the
 * shader-clock ticks it spent inside the K loops of its tiles, and the number of its tiles.
 * Workgroups that find no tile write nothing; a later launch overwrites an earlier one's record.
 * clocks: device memory of 4*n int64, owned by the caller, which keeps it alive until the launches
 * have finished or the buffer is switched off with moe_tile_clock_buffer(NULL, 0).  The setting is
 * per host thread; the kernels read the clocks in either case (two scalar reads per tile) and only
 * skip the store when it is off.
 * Returns MOE_ERR_SHAPE for a buffer with n < 1.
 */
int moe_tile_clock_buffer(int64_t* clocks, int workgroups);

#ifdef __cplusplus
}
#endif
#endif /* MOE_TUNING_H_ */
