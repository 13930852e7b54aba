/*
 * pfc_probe.h -- C ABI of libpfc_probe.so: calibration probes for benchmarks.  They do not touch
 * any state of the method and are not part of libpfc.so: what this GPU sustains on a plain float4
 * stream copy and on a bare bf16 MFMA issue loop with non-trivial operand bit patterns, reported
 * beside the nominal peaks so that a roofline fraction can be read against both.
 *
 * Both run `reps` times on `hip_stream` (a hipStream_t, NULL = the default stream), wait for it,
 * and return the rate through the host pointer.  Return value: 0, or a negative code of pfc.h.
 */
#ifndef PFC_PROBE_H_
#define PFC_PROBE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* src, dst: dev, `bytes` bytes each (a multiple of 16); the rate counts read + write, in GB/s. */
int pfc_probe_stream_copy(void* hip_stream, const void* src, void* dst, int64_t bytes,
                          int32_t reps, double* gbs_out);
/* sink: dev, at least one float (never written in practice: it keeps the loop alive); TFLOP/s. */
int pfc_probe_mfma_bf16(void* hip_stream, float* sink, int32_t reps, double* tflops_out);

#ifdef __cplusplus
}
#endif
#endif /* PFC_PROBE_H_ */
