/*
 * pcm_measure.h -- measurement aids around the PCM library.  Not part of the training path: nothing
 * here is needed to run a step, and none of it follows a passage of the paper.  The benchmark uses
 * these calls to attribute time to the kernels of a step and to report the matrix-core rate the
 * chip sustains under its power limit.
 *
 * Two libraries:
 *   libpcm.so          exports the stage timer below (the timer hooks sit inside the training calls,
 *                      and cost one branch on a flag while the timer is off);
 *   libpcm_measure.so  exports pcm_measure_mfma_rate, a stand-alone microbenchmark that allocates its
 *                      own buffers and synchronises the device; it shares nothing with libpcm.so.
 */
#ifndef PCM_MEASURE_H_
#define PCM_MEASURE_H_

#include <stdint.h>

#include "pcm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------------------------
 * Stage timing (libpcm.so, host side).  While enabled, the entry points of pcm.h record HIP events
 * on `stream` around their kernels (this creates events and takes a lock on the call path, so timed
 * throughput figures are taken with it disabled); pcm_profile_collect waits for the last recorded
 * event and adds each stage's elapsed time to a running total.  Disabled by default; enabling it
 * does not change any result.
 * ------------------------------------------------------------------------------------------ */
PCM_API int pcm_profile_enable(int on);                 /* returns PCM_OK; resets totals when turned on */
PCM_API int pcm_profile_stage_count(void);
PCM_API const char* pcm_profile_stage_name(int stage);  /* NULL if out of range */
/* host arrays of pcm_profile_stage_count() entries: total milliseconds and launch counts */
PCM_API int pcm_profile_collect(double* total_ms, int64_t* launches);

/* ------------------------------------------------------------------------------------------
 * pcm_measure_mfma_rate (libpcm_measure.so).  Runs bf16 matrix instructions
 * (v_mfma_f32_32x32x16_bf16, fp32 accumulation) from registers on every CU of the current device
 * for about `milliseconds`, with all-zero operands (random_operands = 0) or roughly normal random
 * operands, and reports the sustained rate in TFLOP/s and the mean shader clock in GHz (clock_ghz
 * may be NULL).  Allocates two small device buffers for its own use, frees them before it returns,
 * launches on the default stream and synchronises it.  The chip is power-limited under matrix load
 * and the rate depends on the data, so this is the ceiling a bf16 GEMM on such data can approach;
 * the nominal peak assumes the top clock.
 * ------------------------------------------------------------------------------------------ */
PCM_API int pcm_measure_mfma_rate(int random_operands, int milliseconds, double* tflops, double* clock_ghz);

#ifdef __cplusplus
}
#endif
#endif /* PCM_MEASURE_H_ */
