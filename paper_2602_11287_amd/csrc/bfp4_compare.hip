// The other two 4-bit block formats of the HiF4 paper's quantisation-error study (Section
// III-A: MSE of HiF4, NVFP4 and MXFP4 on Gaussian matrices), as fake-quantisers on the GPU, and
// the squared-error sums the study needs.  Comparison tools: nothing in the HiF4 path uses them.
//
// MXFP4 (Section I; OCP Microscaling): groups of 32 along K, shared scale
// 2^(floor(log2 amax) - 2), elements E2M1, nearest-even, saturated at +-6.
// NVFP4 (Section I / III-A): groups of 16, FP8-E4M3 scale that brings the group peak to 6,
// elements E2M1; with per-tensor scaling the tensor is first multiplied by 2688 / max|x|.
// All arithmetic is fp64 in the order a straightforward host implementation takes (one
// rounding per multiply or divide), so results can be checked value by value; finite inputs.
#include "hif4_common.h"

namespace hif4 {

__device__ __forceinline__ double bf16_to_double(uint32_t b) { return (double)u2f(b << 16); }

// Nearest E2M1 magnitude grid point (0, 0.5, 1, 1.5, 2, 3, 4, 6), ties to the even mantissa.
__device__ __forceinline__ double round_e2m1(double v)
{
    const double a = fabs(v);
    double r;
    if (a < 2.0) r = rint(a * 2.0) * 0.5;
    else if (a < 4.0) r = rint(a);
    else r = fmin(rint(a * 0.5) * 2.0, 6.0);
    return copysign(r, v);
}

// floor(log2 v) of a positive normal double, from its exponent field.
__device__ __forceinline__ int floor_log2(double v)
{
    return (int)((__builtin_bit_cast(uint64_t, v) >> 52) & 0x7FF) - 1023;
}

// Nearest FP8-E4M3 value (bias 7, subnormals, largest 448, no infinity) of v >= 0.
__device__ __forceinline__ double round_e4m3(double v)
{
    int e = floor_log2(fmax(v, 0x1p-20));
    e = e < -6 ? -6 : e; // subnormals share the spacing of 2^-6
    const double step = ldexp(1.0, e - 3);
    return fmin(rint(v / step) * step, 448.0);
}

__device__ __forceinline__ void add_block_sum(double v, double *out)
{
    // wave sum by shuffles, then one atomic per wave
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(out, v);
}

// One thread per group of G elements.  FORMAT 0: MXFP4 (G = 32), 1: NVFP4 (G = 16).
template <int FORMAT>
__global__ __launch_bounds__(256) void fake_quant_kernel(const uint16_t *__restrict__ x, int64_t groups, int64_t gpr,
                                                         int64_t ldx, const uint32_t *__restrict__ tensor_peak,
                                                         double *__restrict__ y, double *__restrict__ sq_err)
{
    constexpr int G = FORMAT == 0 ? 32 : 16;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double err = 0.0;
    if (gid < groups) {
        const int64_t row = gid / gpr, g = gid - row * gpr;
        const uint4 *src = reinterpret_cast<const uint4 *>(x + row * ldx + g * G);
        uint32_t w[G / 2];
#pragma unroll
        for (int i = 0; i < G / 8; ++i) {
            const uint4 v = src[i];
            w[4 * i] = v.x, w[4 * i + 1] = v.y, w[4 * i + 2] = v.z, w[4 * i + 3] = v.w;
        }
        double t = 1.0; // per-tensor factor of NVFP4
        if (FORMAT == 1 && tensor_peak) {
            const double peak = bf16_to_double(*tensor_peak & 0x7FFFu);
            t = peak > 0.0 ? 2688.0 / peak : 1.0;
        }
        double v[G];
        double amax = 0.0;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            v[i] = bf16_to_double((w[i / 2] >> (16 * (i & 1))) & 0xFFFFu) * t;
            amax = fmax(amax, fabs(v[i]));
        }
        double scale;
        if (FORMAT == 0) {
            int sh = floor_log2(amax > 0.0 ? amax : 1.0) - 2;
            sh = sh < -127 ? -127 : (sh > 127 ? 127 : sh);
            scale = ldexp(1.0, sh);
        } else {
            scale = round_e4m3(amax / 6.0);
        }
        const double safe = scale > 0.0 ? scale : 1.0;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const double q = round_e2m1(v[i] / safe);
            const double deq = (scale > 0.0 ? q * scale : 0.0) / t;
            if (y) y[row * gpr * G + g * G + i] = deq;
            const double d = bf16_to_double((w[i / 2] >> (16 * (i & 1))) & 0xFFFFu) - deq;
            err += d * d;
        }
    }
    if (sq_err) add_block_sum(err, sq_err);
}

// max |x| of a BF16 matrix as a BF16 pattern (patterns of non-negative values order like
// integers); *peak must hold 0, or the running maximum, before the launch.
__global__ __launch_bounds__(256) void abs_max_kernel(const uint16_t *__restrict__ x, int64_t chunks, int64_t cpr, int64_t ldx,
                                                      uint32_t *__restrict__ peak)
{
    uint32_t m = 0;
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < chunks; c += (int64_t)gridDim.x * 256) {
        const int64_t row = c / cpr;
        const uint4 v = *reinterpret_cast<const uint4 *>(x + row * ldx + (c - row * cpr) * 8);
        const uint32_t p = pk_max_u16(pk_max_u16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu), pk_max_u16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu));
        m = umax(m, umax(p & 0xFFFFu, p >> 16));
    }
    for (int off = 32; off > 0; off >>= 1) m = umax(m, (uint32_t)__shfl_down((int)m, off, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(peak, m);
}

// sum (x - y)^2 over two BF16 matrices, added to *sq_err.
__global__ __launch_bounds__(256) void sq_err_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ y, int64_t chunks,
                                                     int64_t cpr, int64_t ldx, int64_t ldy, double *__restrict__ sq_err)
{
    double err = 0.0;
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < chunks; c += (int64_t)gridDim.x * 256) {
        const int64_t row = c / cpr, at = (c - row * cpr) * 8;
        const uint4 a = *reinterpret_cast<const uint4 *>(x + row * ldx + at);
        const uint4 b = *reinterpret_cast<const uint4 *>(y + row * ldy + at);
        const uint32_t aw[4] = { a.x, a.y, a.z, a.w }, bw[4] = { b.x, b.y, b.z, b.w };
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const double d = bf16_to_double((aw[i / 2] >> (16 * (i & 1))) & 0xFFFFu) - bf16_to_double((bw[i / 2] >> (16 * (i & 1))) & 0xFFFFu);
            err += d * d;
        }
    }
    add_block_sum(err, sq_err);
}

int launch_fake_quant(int format, const void *x, int64_t rows, int64_t K, int64_t ldx, const uint32_t *tensor_peak, double *y,
                      double *sq_err, hipStream_t stream)
{
    const int G = format == 0 ? 32 : 16;
    const int64_t gpr = K / G, groups = rows * gpr;
    if (groups == 0) return HIF4_OK;
    const dim3 grid((unsigned)((groups + 255) / 256)), block(256);
    const uint16_t *xs = static_cast<const uint16_t *>(x);
    if (format == 0) hipLaunchKernelGGL(fake_quant_kernel<0>, grid, block, 0, stream, xs, groups, gpr, ldx, nullptr, y, sq_err);
    else hipLaunchKernelGGL(fake_quant_kernel<1>, grid, block, 0, stream, xs, groups, gpr, ldx, tensor_peak, y, sq_err);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_abs_max(const void *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *peak, hipStream_t stream)
{
    const int64_t cpr = K / 8, chunks = rows * cpr;
    if (chunks == 0) return HIF4_OK;
    const int64_t blocks = (chunks + 255) / 256;
    const dim3 grid((unsigned)(blocks < 2048 ? blocks : 2048)), block(256);
    hipLaunchKernelGGL(abs_max_kernel, grid, block, 0, stream, static_cast<const uint16_t *>(x), chunks, cpr, ldx, peak);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_sq_err(const void *x, const void *y, int64_t rows, int64_t K, int64_t ldx, int64_t ldy, double *sq_err,
                  hipStream_t stream)
{
    const int64_t cpr = K / 8, chunks = rows * cpr;
    if (chunks == 0) return HIF4_OK;
    const int64_t blocks = (chunks + 255) / 256;
    const dim3 grid((unsigned)(blocks < 2048 ? blocks : 2048)), block(256);
    hipLaunchKernelGGL(sq_err_kernel, grid, block, 0, stream, static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(y),
                       chunks, cpr, ldx, ldy, sq_err);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

} // namespace hif4
