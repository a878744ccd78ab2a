/*
 * libgrat — measurement aid, not an operation of the method: a register-resident MFMA-only loop.
 *
 * The attention kernels are priced against the chip's published dense matrix rate.  What the same
 * matrix instruction sustains on a given machine with nothing else going on (no memory traffic,
 * no vector arithmetic, no waits) depends on the clock the chip holds under that load; this entry
 * point lets a benchmark measure it next to the kernels it reports on.
 */
#ifndef GRAT_PROBE_H
#define GRAT_PROBE_H

#include "grat.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueues one launch of `blocks` workgroups of 256 threads (4 waves).  Every wave issues
 * iters * 8 matrix instructions of the kind the attention kernels use for `dtype`
 * (GRAT_BF16: v_mfma_f32_32x32x16_bf16, GRAT_F16: v_mfma_f32_32x32x16_f16; 32 768 flop each) on
 * four independent accumulators.  Work per launch: blocks * 4 * iters * 8 * 32 768 flop; the
 * caller times the launch (events on hip_stream).
 *
 * Operands differ from lane to lane, element to element and instruction to instruction.  Of the
 * eight instructions of an iteration, six work on full 8-bit significands (pseudo-random integers
 * -128..127 over 16): accumulators 0..2 take A_v B_v and then A_v (-B_v), which returns them to
 * exactly 0 (every partial sum is a multiple of 1/256 below 2^24).  Accumulator 3 takes two
 * products of small integers per iteration: lane l (0..63) holds, as element e (0..7),
 *   A = (37 l + 11 e + 5) mod 9 - 4,  B0 = (53 l + 17 e + 2) mod 9 - 4,  B1 = (57 l + 13 e + 7) mod 9 - 4,
 * in the instruction's operand layout A[i][k] and B[k][j] with i = j = l mod 32 and
 * k = 8 (l div 32) + e.  Afterwards every lane adds up its 64 accumulator values (integers, exact)
 * into d_sink[block * 256 + thread]; the 64 sums of a wave therefore add up to
 * iters * sum_ij (A B0 + A B1)_ij — a check that the loop ran its count.
 *
 *   d_sink  DEVICE pointer, blocks * 256 int64, overwritten
 *   blocks  1 .. 65 536;  iters  1 .. 4096 (keeps every accumulator below 2^24)
 *
 * Errors: GRAT_ERR_NULL (d_sink), GRAT_ERR_BAD_DIMS (blocks, iters out of range),
 * GRAT_ERR_UNSUPPORTED (dtype GRAT_F32: no matrix path), GRAT_ERR_HIP; nothing is launched on an
 * error other than GRAT_ERR_HIP.  Allocates nothing, does not synchronise.
 */
grat_status grat_probe_mfma(grat_dtype dtype, int64_t* d_sink, int32_t blocks, int32_t iters,
                            void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GRAT_PROBE_H */
