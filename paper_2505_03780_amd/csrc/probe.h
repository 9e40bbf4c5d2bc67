/*
 * probe.h -- C ABI of libprobe_gfx950.so, the benchmark's measurement aids (not part of the attention
 * library): what the device sustains for the two resources that bound the attention path, for quoting
 * a result against the achievable next to the published peak.  The caller times the kernels on its
 * stream.  Return values: 0 (or a positive count) on success, -1 a NULL pointer, -2 a bad size or
 * alignment, -6 the HIP runtime refused the launch.
 */
#ifndef PROBE_H_
#define PROBE_H_
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
/* Enqueues a streaming read of `bytes` bytes (16-byte aligned device buffer, at least 16 bytes);
 * `sink4` is a 4-byte device word that the kernel may touch. */
int probe_hbm_read(const void *buf, size_t bytes, void *sink4, void *hip_stream);
/* Enqueues `iters` rounds of four independent 32x32x16 bf16 MFMAs on eight wavefronts per compute unit
 * and returns the number of floating-point operations enqueued (> 0). */
int64_t probe_mfma_bf16(int iters, void *sink4, void *hip_stream);
#ifdef __cplusplus
}
#endif
#endif /* PROBE_H_ */
