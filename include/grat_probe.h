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
 * What the instruction sustains depends on how its operands toggle, so `data` chooses them.  In
 * every iteration accumulator v (0..3) takes A_v B_v and then A_v B'_v:
 *   data 0  all operands 1.0, B' = B;
 *   data 1  small integers, B' = B: lane l (0..63) holds, as element e (0..7),
 *             A_v = ((37 + 2v) l + 11 e + 5 + 3v) mod 9 - 4,  B_v = ((53 + 2v) l + 17 e + 2 + 3v) mod 9 - 4,
 *           in the instruction's operand layout A[i][k] and B[k][j] with i = j = l mod 32 and
 *           k = 8 (l div 32) + e;
 *   data 2  the stand-in for real activations: for v < 3 pseudo-random n / 64 with n an integer of at
 *           most 8 significant bits spread roughly like 64 N(0,1), and B' = -B, which returns these
 *           accumulators to exactly 0 (every partial sum is a multiple of 1/4096 below 2^24);
 *           v = 3 as under data 1.
 * Afterwards every lane adds up its 64 accumulator values (integers, exact) into
 * d_sink[block * 256 + thread]; the 64 sums of a wave add up to iters * 2 * sum_ij (A_v B_v)_ij
 * summed over the accumulators that count (data 0, 1: all four; data 2: v = 3) — a check that the
 * loop ran its count.
 *
 *   data    0 .. 2
 *   d_sink  DEVICE pointer, blocks * 256 int64, overwritten
 *   blocks  1 .. 65 536;  iters  1 .. 4096 (keeps every accumulator below 2^24)
 *
 * Errors: GRAT_ERR_NULL (d_sink), GRAT_ERR_BAD_DIMS (data, blocks, iters out of range),
 * GRAT_ERR_UNSUPPORTED (dtype GRAT_F32: no matrix path), GRAT_ERR_HIP; nothing is launched on an
 * error other than GRAT_ERR_HIP.  Allocates nothing, does not synchronise.
 */
grat_status grat_probe_mfma(grat_dtype dtype, int32_t data, int64_t* d_sink, int32_t blocks,
                            int32_t iters, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GRAT_PROBE_H */
