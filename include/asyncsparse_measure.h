/*
 * asyncsparse_measure.h -- measurement support for the benchmark, NOT part of the product ABI (asyncsparse.h).
 *
 * Two probe kernels, built into libasyncsparse_measure.so, that tell what this machine sustains beside the published
 * peaks the roofline fractions are quoted against.  They compute nothing of the method; callers that time them cite
 * no passage of the paper.  Return values: 0 = enqueued, 1 = invalid argument, 5 = a HIP call failed.
 */
#ifndef ASYNCSPARSE_MEASURE_H
#define ASYNCSPARSE_MEASURE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueue a kernel that does nothing but matrix-core instructions (dtype 0: v_mfma_f32_32x32x16_bf16, 1:
 * v_mfma_f32_32x32x2_f32; register operands, two waves per SIMD on every compute unit) for `iters` rounds of 8 per
 * wave, and report in *flop (HOST) how many floating-point operations that is.  Timed by the caller around the
 * launch.  out_device: DEVICE, at least 4 bytes, never written in practice.  stream: hipStream_t or NULL.
 * Asynchronous, allocates nothing.  1 <= iters <= 2^24.
 */
int asp_probe_mfma(int32_t dtype, int64_t iters, void *out_device, void *stream, double *flop);

/*
 * Enqueue a kernel that only reads `bytes` (rounded down to 16, at least 16) of DEVICE memory at src_device
 * (16-byte aligned) with 16-byte loads: the read-only stream that a gather-bound kernel is compared with.
 * out_device: DEVICE, at least 4 bytes.  Asynchronous, allocates nothing.
 */
int asp_probe_read(const void *src_device, int64_t bytes, void *out_device, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ASYNCSPARSE_MEASURE_H */
