/*
 * libhif4 — comparison tools for the quantisation-error study of the HiF4 paper (Section III-A:
 * mean squared error of HiF4, NVFP4 and MXFP4 on Gaussian matrices with standard deviations
 * 0.01 * 2^x).  Not part of the HiF4 path: these entry points exist so that the study, and the
 * SQNR figures of the benchmark, can run on the GPU next to hif4_quantize / hif4_dequantize.
 *
 * Same conventions as hif4.h: device pointers owned by the caller, no allocation, no state,
 * host-side validation, kernels enqueued on the caller's stream, status codes of hif4.h.
 * Inputs are finite BF16 matrices, row-major, K contiguous, rows on 16-byte boundaries.
 */
#ifndef HIF4_COMPARE_H
#define HIF4_COMPARE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * MXFP4 quantise-dequantise (Section I; OCP Microscaling): groups of 32 along K share the scale
 * 2^(floor(log2 max|x|) - 2), clipped to 2^-127 .. 2^127; elements are E2M1 (0, 0.5, 1, 1.5, 2,
 * 3, 4, 6), nearest with ties to the even mantissa, saturated at +-6.  K a multiple of 32.
 *   y       out  fp64 [rows][K] dense, the dequantised values; may be NULL
 *   sq_err  i/o  one fp64: sum over all elements of (x - y)^2 is ADDED to it; may be NULL
 */
int hif4cmp_mxfp4_fake_quant(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx,
                             double *y, double *sq_err, void *stream);

/*
 * NVFP4 quantise-dequantise (Section I / III-A): groups of 16 along K, an FP8-E4M3 scale equal
 * to the nearest E4M3 of (group peak / 6), E2M1 elements as above.  With per-tensor scaling the
 * whole tensor is first multiplied by 2688 / max|x| (2688 = 448 * 6) and the result divided by
 * it again: pass the device address of that maximum as a BF16 pattern in a uint32
 * (hif4cmp_abs_max writes it), or NULL for the direct cast.  K a multiple of 16.
 */
int hif4cmp_nvfp4_fake_quant(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx,
                             const uint32_t *tensor_peak, double *y, double *sq_err, void *stream);

/* *peak = max(*peak, BF16 pattern of max|x|): set *peak to 0 first.  K a multiple of 8. */
int hif4cmp_abs_max(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, uint32_t *peak, void *stream);

/* *sq_err += sum (x - y)^2 over two BF16 matrices of the same shape, in fp64.  K a multiple of 8. */
int hif4cmp_sq_err_bf16(const void *x_bf16, const void *y_bf16, int64_t rows, int64_t K, int64_t ldx, int64_t ldy,
                        double *sq_err, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HIF4_COMPARE_H */
