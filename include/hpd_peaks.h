/*
 * hpd_peaks.h - reference kernels behind the benchmark's "measured_peaks" record: the rates the
 * simplest possible kernels reach on the GPU at hand (a plain read, a plain copy, a loop of
 * independent bf16 MFMAs), reported next to the published peaks that the roofline fractions are
 * quoted against.  They implement nothing of the paper's method and are used by the benchmark
 * only.  Every call enqueues one kernel on `stream` (a hipStream_t as void*, NULL = the null
 * stream) and returns 0, -1 for bad arguments, -4 for a launch error; the caller times them
 * with events.  All pointers are device memory, 16-byte aligned, caller-owned.
 */
#ifndef HPD_PEAKS_H
#define HPD_PEAKS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* reads `bytes` bytes of src once (16-byte loads, a contiguous share per workgroup; a remainder of less
 * than 16 bytes per workgroup of the 32 x compute-unit grid is left out); sink: 4 bytes, practically never written */
int hpd_peak_read(const void* src, size_t bytes, void* sink, void* stream);
/* dst[i] = src[i] over `bytes` bytes (16-byte loads and stores) */
int hpd_peak_copy(void* dst, const void* src, size_t bytes, void* stream);
/* `iters` rounds of four independent v_mfma_f32_32x32x16_bf16 chains per wave, eight waves on every
 * compute unit; *flops_out (host, may be NULL) receives the floating-point operations of the launch */
int hpd_peak_mfma(void* sink, int32_t iters, double* flops_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HPD_PEAKS_H */
