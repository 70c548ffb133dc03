/*
 * qgemm_tuning.h -- experiment overrides of the kernel choice inside qgemm.
 *
 * NOT part of the stable interface of qgemm.h: these exist for the tests (every kernel
 * variant can be forced on a small shape) and for timing sweeps that fit the automatic
 * choice.  The overrides are process-wide and apply to every thread's next qgemm /
 * qgemm_noalloc / qg_plan call; setting one while other threads issue calls changes those
 * calls' kernel choice (never their validity: each call reads every override once and
 * refuses a combination that does not cover its shape with QG_EINVAL).  No passage of the
 * paper defines them; the paper's counterpart is its tile-size tuning (Section
 * "Performance of Low-Precision Kernels": about 200 configurations per operator).
 */
#ifndef QGEMM_TUNING_H_
#define QGEMM_TUNING_H_

#include "qgemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Sets override `knob` (0..3) to `value` (0 = automatic) and returns the previous value.
 *   knob 0: forced path (1 = streaming kernel, M <= 64 only; 2 = tiled kernel; 3 = streaming
 *           kernel over blocks of 64 rows; 4 = the paper's prefill variant, Section "End-to-End
 *           Performance": the whole weight is de-quantised to 16 bits first, into a
 *           library-owned buffer of K*N*2 bytes per (device, stream) -- allocated on first
 *           use, replaced after a stream synchronisation when a larger weight arrives, so this
 *           path is not for graph capture and is refused by qgemm_noalloc -- then the tiled
 *           kernel runs on those 16-bit operands with its unpack stage switched off.  Same
 *           rounded weights, same results as path 2; K*N*2 must stay below 2 GiB.  For the
 *           integer and float types it is never chosen automatically: it is slower than the
 *           fused kernel at every M measured, 64 to 12288 rows (qgemm_codebook chooses it for
 *           codes of more than 4 bits from 1024 rows on); 5 = M <= 4 only: matrix-vector kernel on the vector
 *           ALU -- two-element dot products, partial sums added inside the wavefront with lane
 *           permutes -- the measured alternative to the matrix-core streaming kernel; knob 3
 *           then takes its wavefronts per strip, 4 / 8, or 16 with M = 1)
 *   knob 1: forced split-K factor (streaming kernel; tiled kernel with 64- or 128-row tiles)
 *   knob 2: forced row-tile height of the tiled kernel (64 / 128 / 256; 64 on the first
 *           layout only)
 *   knob 3: wavefront arrangement of the streaming kernel: 10 * row tiles + 0 / 1 / 2 for
 *           8 / 4 / 16 wavefronts per strip (10, 11, 12, 21, 41); 14, 15, 26, 46: 8, 16 or 4
 *           wavefronts on 2 adjacent strips; 16: 16 wavefronts on 4 strips.  Its row tiles
 *           must be the ones M needs (1 up to 16 rows, 2 up to 32, 4 up to 64), else QG_EINVAL.
 * Knobs 0, 1 and 3 apply to QG_LAYOUT_TILE128x64 only. */
QG_API int qg_set_knob(int knob, int value);

#ifdef __cplusplus
}
#endif
#endif /* QGEMM_TUNING_H_ */
