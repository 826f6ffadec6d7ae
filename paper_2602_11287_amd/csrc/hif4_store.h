// Epilogues of the GEMM kernels: the fp32 accumulators of a wave, in the layout of its matrix instruction, to C as
// fp32 or BF16 (nearest, ties to even).  What matters here is the instruction count: a lane has up to 128 results,
// and an address computed from scratch plus a bounds test per result (two 64-bit multiplications, a compare and a
// branch each) cost a workgroup several microseconds after its last K step.  So a wave whose whole part of the tile
// lies inside C - the common case, decided once per wave - computes one address per lane, steps it from row to row by
// the row stride and reaches the columns of further MFMA tiles through the store's immediate offset; only the waves on
// the edges of C test every result.
#pragma once
#include "hif4_common.h"

namespace hif4 {

__device__ __forceinline__ uint16_t bf16_rne_bits(float v)
{
    const uint32_t u = f2u(v);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

template <bool OUT_F32>
__device__ __forceinline__ void store_result(char *p, float v)
{
    if (OUT_F32) *reinterpret_cast<float *>(p) = v;
    else *reinterpret_cast<uint16_t *>(p) = bf16_rne_bits(v);
}

// v_mfma_f32_16x16x32_bf16: acc[i][j][r] is row 16 i + 4 q + r, column 16 j + n of the wave's part, for lane (n, q) =
// (lane % 16, lane / 16).  (wrow0, wcol0): first row and column of the wave's part in C (wave-uniform); rows_end, N:
// the bounds.  The decision is taken per block of 16 rows, so a part that crosses the last row of C (or of an expert)
// still stores its full blocks the short way.
template <bool OUT_F32, int TM, int TN>
__device__ __forceinline__ void store_acc_16x16(const f32x4_t (&acc)[TM][TN], void *c, int64_t ldc, int wrow0, int wcol0, int rows_end, int N)
{
    constexpr int ES = OUT_F32 ? 4 : 2;
    const int lane = threadIdx.x % 64, n = lane % 16, q = lane / 16;
    const int64_t rstep = ldc * ES; // bytes from row to row
    const bool cols_inside = wcol0 + 16 * TN <= N; // wave-uniform
    char *p = static_cast<char *>(c) + ((int64_t)(wrow0 + 4 * q) * ldc + wcol0 + n) * ES; // row 4 q of block 0, column n
#pragma unroll
    for (int i = 0; i < TM; ++i, p += 16 * rstep) {
        if (wrow0 + 16 * i >= rows_end) break; // wave-uniform: no rows from here on
        if (cols_inside && wrow0 + 16 * (i + 1) <= rows_end) {
            char *pr = p;
#pragma unroll
            for (int r = 0; r < 4; ++r, pr += rstep)
#pragma unroll
                for (int j = 0; j < TN; ++j) store_result<OUT_F32>(pr + j * 16 * ES, acc[i][j][r]);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (wrow0 + 16 * i + 4 * q + r < rows_end && wcol0 + 16 * j + n < N) store_result<OUT_F32>(p + r * rstep + j * 16 * ES, acc[i][j][r]);
        }
    }
}

// v_mfma_f32_32x32x16_bf16: acc[i][j][r] is row 32 i + 8 (r / 4) + 4 h + r % 4, column 32 j + l of the wave's part, for
// lane (l, h) = (lane % 32, lane / 32).
// (at(i, j): the accumulator of row block i, column block j)
template <bool OUT_F32, int TM, int TN, typename At>
__device__ __forceinline__ void store_acc_32x32_at(At at, void *c, int64_t ldc, int wrow0, int wcol0, int rows_end, int N)
{
    constexpr int ES = OUT_F32 ? 4 : 2;
    const int lane = threadIdx.x % 64, l = lane % 32, h = lane / 32;
    const int64_t rstep = ldc * ES;
    const bool cols_inside = wcol0 + 32 * TN <= N; // wave-uniform
    char *p = static_cast<char *>(c) + ((int64_t)(wrow0 + 4 * h) * ldc + wcol0 + l) * ES; // row 4 h of block 0, column l
#pragma unroll
    for (int i = 0; i < TM; ++i, p += 32 * rstep) {
        if (wrow0 + 32 * i >= rows_end) break; // wave-uniform
        if (cols_inside && wrow0 + 32 * (i + 1) <= rows_end) {
            char *pr = p;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4, pr += 4 * rstep) // rows 8 g4 + 4 h .. + 3 of the block; the other half of the lanes holds the next 4
#pragma unroll
                for (int r = 0; r < 4; ++r, pr += rstep)
#pragma unroll
                    for (int j = 0; j < TN; ++j) store_result<OUT_F32>(pr + j * 32 * ES, at(i, j)[4 * g4 + r]);
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (wrow0 + 32 * i + 8 * (r / 4) + 4 * h + r % 4 < rows_end && wcol0 + 32 * j + l < N)
                        store_result<OUT_F32>(p + (8 * (r / 4) + r % 4) * rstep + j * 32 * ES, at(i, j)[r]);
        }
    }
}

template <bool OUT_F32, int TM, int TN>
__device__ __forceinline__ void store_acc_32x32(const f32x16_t (&acc)[TM][TN], void *c, int64_t ldc, int wrow0, int wcol0, int rows_end, int N)
{
    store_acc_32x32_at<OUT_F32, TM, TN>([&](int i, int j) -> const f32x16_t & { return acc[i][j]; }, c, ldc, wrow0, wcol0, rows_end, N);
}

// one column of 32 x 32 blocks
template <bool OUT_F32, int TM>
__device__ __forceinline__ void store_acc_32x32(const f32x16_t (&acc)[TM], void *c, int64_t ldc, int wrow0, int wcol0, int rows_end, int N)
{
    store_acc_32x32_at<OUT_F32, TM, 1>([&](int i, int) -> const f32x16_t & { return acc[i]; }, c, ldc, wrow0, wcol0, rows_end, N);
}

} // namespace hif4
