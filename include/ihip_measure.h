/*
 * ihip_measure.h -- measurement hooks of libihip.so: per-kernel event timing and a dense matrix-core
 * rate probe.  They serve the benchmark's protocol (mean launch duration of every kernel on its
 * stream; the sustained MFMA rate next to the vendor's peak) and are no part of the method's
 * boundary, which is ihip.h.
 */
#ifndef IHIP_MEASURE_H
#define IHIP_MEASURE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optional per-kernel timing (the measurement protocol, not the method): while
 * enabled, every kernel the library launches is bracketed by two HIP events on
 * its stream (events are created on first use and recycled).  ihip_profile_read
 * waits for the recorded events, adds them up per kernel name and forgets
 * them: it fills up to max_entries of names (static strings owned by the
 * library), total_ms and launches (host arrays) and returns the number of
 * distinct kernels, or a negative error.  Not for use under graph capture.
 */
int32_t ihip_profile_enable(int32_t on);
int32_t ihip_profile_read(int32_t max_entries, const char **names, double *total_ms, int64_t *launches);

/*
 * Dense matrix-core rate of the current device (the measurement protocol, not
 * the method): runs independent accumulation chains of one bf16 MFMA shape
 * (kind 0: 32x32x16, the prefill attention's; kind 1: 16x16x32, the prefill
 * pruning's) with no memory traffic, `iters` instructions per chain, on every
 * compute unit, twice (the second run is timed with HIP events on `stream`),
 * and writes the rate in TFLOP/s (2 flops per multiply-add) to the host double
 * *tflops.  scratch: device, >= 512 floats, never written in practice.  Blocks
 * until the timed run has finished.  Not for use under graph capture.
 */
int32_t ihip_mfma_rate(int32_t kind, int32_t iters, float *scratch, double *tflops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* IHIP_MEASURE_H */
