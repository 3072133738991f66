/*
 * kst_yardstick.h -- measuring aids of libkst.so, kept apart from the product's
 * interface (kst.h): what the chip sustains with nothing in the way, to be printed
 * beside the published peaks by the benchmark.  They compute nothing of the method.
 * Same conventions as kst.h: device pointers owned by the caller, work enqueued on
 * the caller's stream, a status returned.
 */
#ifndef KST_YARDSTICK_H
#define KST_YARDSTICK_H

#include "kst.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * kst_yardstick_mfma: every SIMD of every CU runs `iters` rounds of four
 * independent matrix-core instructions of the shape the matrix-core paths use
 * (KST_F32: 32x32x2 fp32; KST_BF16: 32x32x16 bf16, fp32 accumulate) and nothing
 * else.  sink (device, at least kst_yardstick_mfma_sink_elems() floats) receives
 * one sum per lane so that the loop is kept; its values carry no meaning.
 * kst_yardstick_mfma_flops = the floating-point operations one such launch does
 * (0 for an unknown dtype or iters < 1).  iters must be in 1 .. 2^22.
 *
 * kst_yardstick_copy: dst[0..bytes) = src[0..bytes) with 16-byte loads and
 * streaming 16-byte stores; bytes must be a multiple of 16, both pointers device
 * pointers aligned to 16 bytes, the ranges disjoint.
 *
 * Both enqueue on `stream` and return without synchronising.
 */
size_t kst_yardstick_mfma_sink_elems(void);
double kst_yardstick_mfma_flops(kst_dtype dtype, int iters);
kst_status kst_yardstick_mfma(kst_dtype dtype, int iters, float *sink, size_t sink_elems,
                              hipStream_t stream);
kst_status kst_yardstick_copy(const void *src, void *dst, size_t bytes, hipStream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* KST_YARDSTICK_H */
