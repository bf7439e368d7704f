/*
 * fupr_measure - two kernels of known work and nothing else, for the roofline
 * figures a benchmark reports beside the published peaks of the GPU.  They are
 * not part of the method and live in a library of their own
 * (libfupr_measure.so), so that the product library exports only the method.
 *
 * Device pointers are marked [dev]; both calls are asynchronous on `stream`
 * (a hipStream_t passed as void*, NULL = the default stream) and allocate
 * nothing; the caller times them.  Return value: 0, or a negative code
 * (-1 NULL pointer, -3 unknown dtype, -9 other invalid argument, -2 size,
 * -7 alignment, -8 the HIP runtime refused the launch).
 */
#ifndef FUPR_MEASURE_H
#define FUPR_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * `workgroups` workgroups of 4 waves, each wave issuing iters * 8 independent
 * MFMAs on registers only.  dt: 1 = bf16, 2 = fp16.  shape: 16 = 16 x 16 x 32
 * (4 accumulator registers per MFMA), 32 = 32 x 32 x 16 (16 accumulator
 * registers).  out [dev] receives workgroups * 256 floats (so that the work
 * cannot be dropped); *flops [host] receives the floating-point operations enqueued.
 */
int32_t fupr_measure_mfma(int32_t dt, int32_t shape, int32_t iters, int32_t workgroups, void* out,
                          double* flops, void* stream);

/* dst[0..bytes) = src[0..bytes), 16 bytes per lane; bytes a multiple of 16, both
 * pointers [dev], 16-byte aligned, not overlapping. */
int32_t fupr_measure_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FUPR_MEASURE_H */
