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

/*
 * Speed reference: a GEMM on CDNA4's native MXFP4 matrix instruction
 * (v_mfma_scale_f32_32x32x64_f8f6f4 with both operands E2M1 and one E8M0 scale per 32 values),
 * on the same tile kernel that hif4_gemm uses for decoded operands.  It shows what the hardware's
 * own 4-bit block format reaches on a shape; it computes C = dq(A) * dq(W)^T for MXFP4-quantised
 * operands, not a HiF4 product.
 *
 * hif4ref_mxfp4_pack quantises a finite BF16 matrix [rows][ldx] to MXFP4 (rule as in
 * hif4cmp_mxfp4_fake_quant) in the layout the kernel reads:
 *   cells  : 16 bytes per group of 32 along K, element i in nibble i (sign, two exponent bits,
 *            one mantissa bit); cell (row, group g) at index g * rows + row;  rows * K / 2 bytes
 *   scales : the biased exponents of the group scales; the byte of group j of K step ks (256
 *            wide) of a row sits at ((ks * 2 + j % 2) * rows + row) * 4 + j / 2;  rows * K / 32 bytes
 * K must be a multiple of 256 for both calls.  Pointers 16-byte aligned.
 */
int hif4ref_mxfp4_pack(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, void *cells, void *scales, void *stream);

/* C[M][N] (BF16 or fp32 per out_dtype of hif4.h, row stride ldc) from two packed operands. */
int hif4ref_mxfp4_gemm(const void *a_cells, const void *a_scales, const void *w_cells, const void *w_scales,
                       int64_t M, int64_t N, int64_t K, void *c, int64_t ldc, int out_dtype, void *stream);

/*
 * Measurement aid: 256 workgroups of 8 waves each run `iters` rounds of 8 independent MFMAs on
 * operands with random bit patterns and nothing else, i.e. 2048 * iters * 8 instructions of
 * 32768 flop (kind 0: v_mfma_f32_32x32x16_bf16) or 131072 flop (kind 1: the FP4 form of
 * v_mfma_scale_f32_32x32x64_f8f6f4); kind 2 runs 16 v_mfma_f32_16x16x32_bf16 per round, the same
 * flops as kind 0.  Timed by the benchmark, it gives the rate the matrix pipeline sustains under
 * its power limit, the ceiling next to which GEMM rates are read.
 *   out  device, 131072 floats, receives checksums nobody needs; out[0] instead receives the shader clock, in MHz, that
 *        the first wave of the launch ran at (its cycle counter over the fixed 100 MHz counter): under a power
 *        limit the clock falls with the work done per cycle
 */
int hif4ref_mfma_loop(int kind, int iters, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HIF4_COMPARE_H */
