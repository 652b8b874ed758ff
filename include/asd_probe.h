/*
 * asd_probe.h -- measurement probe used by the benchmark harness (libasd_probe.so).  Not part of
 * the sampling library: nothing in libasd.so calls it.
 */
#ifndef ASD_PROBE_H
#define ASD_PROBE_H

#include <stdint.h>

#if defined(__GNUC__)
#define ASD_PROBE_API __attribute__((visibility("default")))
#else
#define ASD_PROBE_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

/* What the matrix pipe of the current device sustains: a register-only loop of 32x32 MFMAs (dtype 1:
 * v_mfma_f32_32x32x16_bf16, 2: v_mfma_f32_32x32x16_f16, 0: v_mfma_f32_32x32x2_f32) with no memory traffic, run for about
 * ms_target milliseconds (1..5000) on the default stream; *tflops HOST receives the rate of the second
 * half of the run.  random_data != 0: zero-mean random operands, as in real use; 0: constant operands.
 * Returns 0, -1 (bad argument; checked before any device call) or -3 (a HIP call failed).
 * Allocates and frees a few MB; synchronous. */
ASD_PROBE_API int32_t asd_probe_mfma_ceiling(int32_t dtype, int32_t random_data, int32_t ms_target, double* tflops);
/* Message of the last failure on this thread ("" if none). */
ASD_PROBE_API const char* asd_probe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ASD_PROBE_H */
