/*
 * dmi_bench.h -- harness-side kernels used by bench.py only (libdmi_bench.so).
 * Not part of the capture-and-stage library: they model the serving engine the
 * library runs beside (paper section 6: overhead is measured against the
 * uninstrumented inference step).
 */
#ifndef DMI_BENCH_H
#define DMI_BENCH_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* Occupies `stream` for about `microseconds` with one idle wavefront (bounded
 * wait on the constant-rate wall clock), so that launches enqueued behind it run
 * back to back.  Returns 0 or a hipError_t value. */
int dmi_bench_sleep(void *hip_stream, uint32_t microseconds);

/* Decode-like interfering work: streams n_elems bf16 weights [device] once,
 * multiplies them with a 4096-element bf16 vector x [device] (reused cyclically)
 * and accumulates in fp32 into out[0..n_out) [device, float, n_out >= 4096].
 * HBM-bound like a decode step's weight read.  n_elems must be a multiple of 8
 * and w 16-byte aligned. */
int dmi_bench_stream_gemv(const void *w, uint64_t n_elems, const void *x, float *out, void *hip_stream);

/* Plain device-to-device copy of n_bytes (multiple of 16, both pointers 16-byte
 * aligned): reads n_bytes, writes n_bytes.  The known-size reference the HBM traffic
 * counters of the profiler are scaled by. */
int dmi_bench_copy(void *dst, const void *src, uint64_t n_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
