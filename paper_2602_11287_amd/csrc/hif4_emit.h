// GEMM epilogue that writes the result as HiF4 (units along N, the reduction axis of the next
// layer): the fp32 tile in the MFMA accumulators is rounded to BF16 exactly as the BF16 output
// would be, parked in LDS row-major, and encoded by Algorithm 1 of the HiF4 paper (Section II-B)
// with the arithmetic of the streaming encoder.  The result equals hif4_quantize applied to the
// BF16 output of the same main loop, bit for bit, without C crossing HBM as BF16.
#pragma once
#include "hif4_encode.h"

namespace hif4 {

// LDS bytes the epilogue needs for a BM x BN tile: rows padded by 16 bytes against bank conflicts.
template <int BM, int BN>
constexpr size_t emit_lds_bytes()
{
    return (size_t)BM * (BN * 2 + 16);
}

// Second half of the epilogue: the BF16 tile parked in LDS (row stride BN + 8 elements) -> HiF4 planes.
template <int BM, int BN, int NT, int MODE>
__device__ __forceinline__ void emit_encode_parked(const uint16_t *tile, int row0, int rows_end, int col0, int N,
                                                   uint32_t *__restrict__ c_codes, uint32_t *__restrict__ c_meta)
{
    constexpr int RS = BN + 8;
    const int tid = threadIdx.x;
    // four adjacent lanes per unit, as in the streaming encoder: lane l owns groups of 8 number l and l + 4
    constexpr int UPR = BN / 64, UNITS = BM * UPR, UPP = NT / 4; // units per row, per tile, per pass
    const int l = tid & 3;
    const int64_t n8 = N / 8, n64 = N / 64;
#pragma unroll 1
    for (int u0 = 0; u0 < UNITS; u0 += UPP) {
        int u = u0 + tid / 4;
        const bool in_tile = UNITS % UPP == 0 || u < UNITS; // a tile with fewer units than a pass takes: the rest idle
        u = in_tile ? u : UNITS - 1;
        const int row = u / UPR, ucol = u % UPR;
        uint4 w[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) w[c] = *reinterpret_cast<const uint4 *>(tile + row * RS + ucol * 64 + (c * 4 + l) * 8);
        uint32_t out[2];
        const uint32_t m = encode_share<4, MODE>(w, l, out);
        const int grow = row0 + row, gunit = col0 / 64 + ucol;
        if (in_tile && grow < rows_end && gunit < n64) {
#pragma unroll
            for (int c = 0; c < 2; ++c) c_codes[grow * n8 + gunit * 8 + c * 4 + l] = out[c];
            if (l == 0) c_meta[grow * n64 + gunit] = m;
        }
    }
}

// acc: TM x TN accumulators of this wave (wave (wm, wn) of WM x WN, tiles of 32 x 32; lane holds
// column lane % 32 and rows 8 * (r / 4) + 4 * (lane / 32) + r % 4 of each tile).  All threads of
// the workgroup call this after their last LDS read of the main loop.  Rows at or past rows_end
// and columns at or past N (a multiple of 64) are not stored.
template <int BM, int BN, int WM, int WN, int MODE, int TM, int TN>
__device__ __forceinline__ void emit_hif4_tile(const f32x16_t (&acc)[TM][TN], void *lds, int row0, int rows_end, int col0, int N,
                                               uint32_t *__restrict__ c_codes, uint32_t *__restrict__ c_meta)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int RS = BN + 8; // row stride in BF16 elements
    uint16_t *tile = static_cast<uint16_t *>(lds);
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int wm = wave / WN, wn = wave % WN, half = lane / 32, l32 = lane % 32;

    __syncthreads(); // every wave is past its operand reads of the last K step
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * (BM / WM) + i * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                const int col = wn * (BN / WN) + jn * 32 + l32;
                const uint32_t u = f2u(acc[i][jn][r]);
                tile[row * RS + col] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
            }
    __syncthreads();

    emit_encode_parked<BM, BN, NT, MODE>(tile, row0, rows_end, col0, N, c_codes, c_meta);
}

// The same for accumulators of v_mfma_f32_16x16x32_bf16: TM x TN tiles of 16 x 16 per wave, lane holds column
// lane % 16 and rows 4 * (lane / 16) + r of each tile.
template <int BM, int BN, int WM, int WN, int MODE, int TM, int TN>
__device__ __forceinline__ void emit_hif4_tile16(const f32x4_t (&acc)[TM][TN], void *lds, int row0, int rows_end, int col0, int N,
                                                 uint32_t *__restrict__ c_codes, uint32_t *__restrict__ c_meta)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int RS = BN + 8;
    uint16_t *tile = static_cast<uint16_t *>(lds);
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int wm = wave / WN, wn = wave % WN, q = lane / 16, n = lane % 16;

    __syncthreads(); // every wave is past its operand reads of the last K step
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = wm * (BM / WM) + i * 16 + 4 * q + r;
                const int col = wn * (BN / WN) + jn * 16 + n;
                const uint32_t u = f2u(acc[i][jn][r]);
                tile[row * RS + col] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
            }
    __syncthreads();
    emit_encode_parked<BM, BN, NT, MODE>(tile, row0, rows_end, col0, N, c_codes, c_meta);
}

} // namespace hif4
