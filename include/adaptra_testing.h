/*
 * adaptra_testing.h -- switches and probes for tests and measurements.
 *
 * Nothing here is part of the product path of adaptra.h: a caller that only evaluates
 * schedules never needs this header.  The functions live in the same shared library so that
 * the parity tests can force each kernel of the path and the benchmark can time the dominant
 * kernel and the machine's integer rate with the library's own launches.
 */
#ifndef ADAPTRA_TESTING_H
#define ADAPTRA_TESTING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel selection for every later call of the evaluation entry points, process-wide (one
 * atomic word: a call reads it once, at its start).
 *   0  automatic (default): up to 32 stages, the register/LDS kernel with scenarios on the
 *      lanes from 48 scenarios on (from 33 with at least 32768 candidates), below that -- and
 *      from 33 to 64 stages always -- the kernel with candidates on the lanes, in its read-ahead
 *      form (the measured crossover); the general kernel for what fits
 *      neither (per-scenario stage times at more than 32 stages, warm-ups deeper than the LDS
 *      ring of 128 slots)
 *   1  general kernel only (any S, M, warm-up depth)
 *   2  scenario-lanes kernel wherever its limits allow, regardless of lane efficiency
 *   3  candidate-lanes kernel wherever its limits allow, in its plain form
 *   4  the same, in its read-ahead form (what automatic mode uses)
 * Returns the previous mode, or -1 for an unknown mode (nothing changes). */
int adaptra_set_kernel_mode(int mode);

/* Timing of the resolve kernels (the max-plus recurrence) alone, for the CALLING THREAD's
 * later calls: when both arguments are non-NULL hipEvent_t handles, adaptra_eval,
 * adaptra_best and adaptra_eval_best record `before` on their stream just ahead of those
 * launches and `after` right behind them.  The handles stay the caller's; they must outlive
 * the calls that record them.  Pass NULL, NULL to switch it off (do so before destroying the
 * events).  Always returns ADAPTRA_OK. */
int adaptra_set_resolve_events(void *before, void *after);

/* Instruction mixes of adaptra_valu_probe.  Each is a kernel without memory traffic (the last
 * one aside) in which every wavefront issues the same vector instruction, or short group, over
 * and over on eight independent registers, so that its issue rate can be read off the duration. */
#define ADAPTRA_PROBE_ADD_MAX         0   /* v_add_u32 (scalar addend) + v_max_i32, as the compiler writes the recurrence's two ops */
#define ADAPTRA_PROBE_ADD_VGPR        1   /* v_add_u32, vector operands only */
#define ADAPTRA_PROBE_ADD_SGPR        2   /* v_add_u32 with a scalar operand */
#define ADAPTRA_PROBE_ADD_INLINE      3   /* v_add_u32 with an inline constant */
#define ADAPTRA_PROBE_ADD_LITERAL     4   /* v_add_u32 with a 32-bit literal */
#define ADAPTRA_PROBE_ADD_E64         5   /* v_add_u32 in the 64-bit encoding */
#define ADAPTRA_PROBE_SUB             6   /* v_sub_u32 */
#define ADAPTRA_PROBE_ADD_CO          7   /* v_add_co_u32 (writes vcc) */
#define ADAPTRA_PROBE_ADD3            8   /* v_add3_u32 */
#define ADAPTRA_PROBE_MAX             9   /* v_max_i32, vector operands only */
#define ADAPTRA_PROBE_MAX_SGPR       10   /* v_max_i32 with a scalar operand */
#define ADAPTRA_PROBE_MAX_E64        11   /* v_max_i32 in the 64-bit encoding */
#define ADAPTRA_PROBE_MAX_U32        12   /* v_max_u32 */
#define ADAPTRA_PROBE_MIN            13   /* v_min_i32 */
#define ADAPTRA_PROBE_MAX3           14   /* v_max3_i32 */
#define ADAPTRA_PROBE_MED3           15   /* v_med3_i32 */
#define ADAPTRA_PROBE_AND            16   /* v_and_b32 */
#define ADAPTRA_PROBE_OR             17   /* v_or_b32 */
#define ADAPTRA_PROBE_XOR            18   /* v_xor_b32 */
#define ADAPTRA_PROBE_LSHL           19   /* v_lshlrev_b32 by an inline constant */
#define ADAPTRA_PROBE_MOV            20   /* v_mov_b32 */
#define ADAPTRA_PROBE_CNDMASK        21   /* v_cndmask_b32 on vcc, vcc set once */
#define ADAPTRA_PROBE_CNDMASK_SGPR   22   /* v_cndmask_b32 on a scalar register pair */
#define ADAPTRA_PROBE_CNDMASK_BFE    23   /* s_bfe_i64 vcc + v_cndmask_b32: the select of a link without slack */
#define ADAPTRA_PROBE_CMP_CNDMASK    24   /* v_cmp_gt_i32 vcc + v_cndmask_b32: a max written as compare and select */
#define ADAPTRA_PROBE_ADD_MAX_ALT    25   /* v_add_u32 and v_max_i32 on vector operands, alternating: add, max, add, max */
#define ADAPTRA_PROBE_ADD_MAX_BATCH  26   /* the same instructions, eight adds then eight maxes */
#define ADAPTRA_PROBE_ADD_MAX_BATCH_NOP 27 /* eight adds then eight maxes, an s_nop behind every instruction */
#define ADAPTRA_PROBE_ADD_MAX_ALT_DENSE 28 /* alternating, without the s_nop between two statements */
#define ADAPTRA_PROBE_READLANE       29   /* v_readlane_b32 */
#define ADAPTRA_PROBE_FORWARD_STEP   30   /* the hot kernel's forward step: add, select, max, two ring address adds, ds_write_b32,
                                               ds_read_b32 and its three scalar ops */
#define ADAPTRA_PROBE_MIXES          31

/* Enqueue a probe kernel of `blocks` x 256 threads; every wavefront issues
 * *valu_instructions / (blocks x 4) vector instructions of the chosen mix.
 *   scratch             DEVICE int32 (never written in practice)
 *   valu_instructions   HOST, may be NULL: vector instructions issued by the whole launch
 *                       (wavefront instructions, 64 lane operations each)
 * Asynchronous on `stream`.  ADAPTRA_EINVAL for an unknown mix or sizes below 1. */
int adaptra_valu_probe(int32_t mix, int32_t blocks, int32_t iters, int32_t *scratch, void *stream,
                       int64_t *valu_instructions);

#ifdef __cplusplus
}
#endif
#endif /* ADAPTRA_TESTING_H */
