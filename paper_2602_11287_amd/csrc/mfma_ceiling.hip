// What the matrix pipeline sustains on this chip when nothing else is in the way: a loop of
// independent MFMAs on operands with random bit patterns (trivial operands such as zeros or
// small integers draw less power and clock higher, which overstates the ceiling a GEMM on real
// data can reach).  A measurement aid for the benchmark, not part of any HiF4 path.
#include "hif4_common.h"

namespace hif4 {

__device__ __forceinline__ uint32_t lcg(uint32_t &s)
{
    s = s * 1664525u + 1013904223u;
    return s;
}

// The first thread of the launch replaces its sum in out[0] by the shader clock it ran at, in MHz: cycles of the
// shader clock over ticks of the fixed 100 MHz counter, both read before the loop and after the sums (`t` keeps the
// second reading behind the last MFMA).  Under a power limit the clock falls with the work per cycle, so this is the
// clock a matrix-bound kernel on real data can expect, not the nominal one.
__device__ __forceinline__ void store_loop_clock(float *out, long long c0, long long w0, float t)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    asm volatile("" : : "v"(t)); // the sums are complete before the clocks are read again
    const long long c1 = clock64(), w1 = wall_clock64();
    out[0] = w1 > w0 ? (float)(c1 - c0) * 100.0f / (float)(w1 - w0) : 0.0f;
}

// KIND 0: v_mfma_f32_32x32x16_bf16.  KIND 1: v_mfma_scale_f32_32x32x64_f8f6f4 with both
// operands FP4 (E2M1) and unit scales.  Eight accumulators per wave (the GEMM kernels' shape:
// 4 x 2 tiles), 8 waves per workgroup, one workgroup per CU-sized slot.
template <int KIND>
__global__ __launch_bounds__(512) void mfma_loop_kernel(float *out, int iters, uint32_t seed)
{
    const long long c0 = clock64(), w0 = wall_clock64(); // shader clock cycles; a fixed 100 MHz counter
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    uint32_t s = seed + threadIdx.x * 7919u + blockIdx.x * 104729u;
    uint4 av[4], bv[2];
    // BF16: clear the top exponent bit, so that magnitudes stay at or below 2 and the sums finite
    const uint32_t keep = KIND == 0 ? 0xBFFFBFFFu : 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < 4; ++i) av[i] = make_uint4(lcg(s) & keep, lcg(s) & keep, lcg(s) & keep, lcg(s) & keep);
#pragma unroll
    for (int i = 0; i < 2; ++i) bv[i] = make_uint4(lcg(s) & keep, lcg(s) & keep, lcg(s) & keep, lcg(s) & keep);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint4 a = av[i / 2], b = bv[i % 2];
            if constexpr (KIND == 0) {
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), acc[i], 0, 0, 0);
            } else {
#if defined(__HIP_DEVICE_COMPILE__)
                typedef int v8i __attribute__((ext_vector_type(8)));
                const v8i A = { (int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0 }, B = { (int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0 };
                acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, acc[i], 4, 4, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
#endif
            }
        }
    }
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) t += acc[i][r];
    out[blockIdx.x * 512 + threadIdx.x] = t;
    store_loop_clock(out, c0, w0, t);
}

// KIND 2 of the MFMA-only loop: v_mfma_f32_16x16x32_bf16, sixteen accumulators of 16 x 16 per wave and
// iteration (the same flops per iteration as the eight 32 x 32 x 16 of KIND 0).
__global__ __launch_bounds__(512) void mfma_loop16_kernel(float *out, int iters, uint32_t seed)
{
    const long long c0 = clock64(), w0 = wall_clock64();
    f32x4_t acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = f32x4_t{ 0.f, 0.f, 0.f, 0.f };
    uint32_t s = seed + threadIdx.x * 7919u + blockIdx.x * 104729u;
    uint4 av[4], bv[4];
    constexpr uint32_t keep = 0xBFFFBFFFu; // magnitudes at or below 2
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        av[i] = make_uint4(lcg(s) & keep, lcg(s) & keep, lcg(s) & keep, lcg(s) & keep);
        bv[i] = make_uint4(lcg(s) & keep, lcg(s) & keep, lcg(s) & keep, lcg(s) & keep);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[i / 4]), __builtin_bit_cast(bf16x8_t, bv[i % 4]), acc[i], 0, 0, 0);
    }
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) t += acc[i][r];
    out[blockIdx.x * 512 + threadIdx.x] = t;
    store_loop_clock(out, c0, w0, t);
}

int launch_mfma_loop(int kind, int iters, float *out, hipStream_t stream)
{
    const dim3 grid(256), block(512);
    if (kind == 0) hipLaunchKernelGGL(mfma_loop_kernel<0>, grid, block, 0, stream, out, iters, 1u);
    else if (kind == 2) hipLaunchKernelGGL(mfma_loop16_kernel, grid, block, 0, stream, out, iters, 1u);
    else hipLaunchKernelGGL(mfma_loop_kernel<1>, grid, block, 0, stream, out, iters, 1u);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

} // namespace hif4
