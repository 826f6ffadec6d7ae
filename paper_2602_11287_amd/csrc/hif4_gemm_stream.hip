// Weight-only HiF4 GEMM for a few dozen rows of A and a wide weight matrix (batched token
// generation on a big linear layer): C[M][N] = A[M][K] (BF16) * W[N][K]^T (HiF4), M <= 64.  The work is streaming W
// from HBM once (0.5625 bytes per weight) and expanding it (Eq. 2 of the HiF4 paper, Section
// II-A); each 64-wide K step of a column is the unit dot product of Eq. 4 (Section III-B) with a
// BF16 left operand, accumulated in fp32.
//
// A workgroup of 4 waves owns 64 output columns, a wave 16 of them over the whole of K, so no
// partial sums cross waves.  v_mfma_f32_16x16x32_bf16: lane (n, q) = (lane % 16, lane / 16)
// supplies 8 consecutive k of weight row n, i.e. one dword of codes expanded in registers in
// natural element order, and 8 consecutive k of activation row n.  K advances by pairs of units
// (128 values): lane (n, q) loads the 16 code bytes [16 q, 16 q + 16) of row n's 64, so a row is
// read as one contiguous run, and MFMA t (0..3) of the pair takes group 4 q + t of the pair's 16
// groups of 8.  The activations are the same for every wave and workgroup: a chunk of CP pairs
// is brought into LDS by direct global -> LDS loads (plain BF16, no reordering needed), laid out
// [pair][row block][group][row] so that both the 64-lane loads and the 16-lane operand reads
// touch consecutive 16-byte cells, double-buffered with one barrier per chunk.  Packed weights
// are fetched two chunks ahead into registers.
#include "hif4_expand.h"

namespace hif4 {

// see hif4_gemm_cells.hip: inline assembly so that the compiler's wait-count pass does not see
// an LDS-writing load (it would serialise every LDS read behind it)
__device__ __forceinline__ void stream_load_to_lds_16(const void *src, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_byte), "v"(src) : "memory");
}

#ifndef HIF4_STREAM_CP4
#define HIF4_STREAM_CP4 2
#endif
#ifndef HIF4_STREAM_CP12
#define HIF4_STREAM_CP12 4
#endif
// pairs of units per chunk of activations (one barrier per chunk), by the number of 16-row blocks
constexpr int stream_chunk_pairs(int mb) { return mb > 2 ? HIF4_STREAM_CP4 : HIF4_STREAM_CP12; }

template <int MB, bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_stream_kernel(const uint16_t *__restrict__ a, int64_t lda,
                                                          const uint32_t *__restrict__ w_codes,
                                                          const uint32_t *__restrict__ w_meta, void *c, int64_t ldc,
                                                          int M, int N, int K)
{
    constexpr int CP = stream_chunk_pairs(MB);         // pairs of units per chunk
    constexpr int CHUNK_CELLS = CP * MB * 256; // 16-byte cells of A per chunk: [pair][row block][16 groups][16 rows]
    constexpr int LOADS = CP * MB * 4;         // 64-cell direct loads per chunk, dealt to the 4 waves
    constexpr int LPW = LOADS / 4;
    extern __shared__ uint4 lds[]; // 2 chunks

    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int n_l = lane % 16, q = lane / 16;
    const int col = blockIdx.x * 64 + wave * 16 + n_l;
    const int colc = col < N ? col : N - 1;
    const int upr = K / 64, npairs = upr / 2, nchunks = (npairs + CP - 1) / CP;
    const uint32_t *wrow = w_codes + (int64_t)colc * (K / 8) + 4 * q;
    const uint32_t *mrow = w_meta + (int64_t)colc * upr + (q >> 1);

    struct Packed {
        uint4 c[CP];
        uint32_t m[CP];
    };
    // the packed weights of chunk ch for this lane; pairs past the end of K repeat the last one (never used)
    auto fetch_w = [&](Packed &pk, int ch) {
#pragma unroll
        for (int i = 0; i < CP; ++i) {
            int p = ch * CP + i;
            p = p < npairs ? p : npairs - 1;
            pk.c[i] = *reinterpret_cast<const uint4 *>(wrow + (int64_t)p * 16);
            pk.m[i] = mrow[2 * p];
        }
    };
    // direct loads of the activations of chunk ch into buffer `buf`: load id -> (pair, row block, 4 groups),
    // lane -> (group, row); rows past M repeat the last row, pairs past the end of K the last pair
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)lds;
    auto stage_a = [&](int buf, int ch) {
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int id = wave * LPW + i, pp = id / (4 * MB), rest = id % (4 * MB), mb = rest / 4, gq = rest % 4;
            int p = ch * CP + pp;
            p = p < npairs ? p : npairs - 1;
            int row = mb * 16 + n_l;
            row = row < M ? row : M - 1;
            const uint16_t *src = a + (int64_t)row * lda + (int64_t)p * 128 + (4 * gq + q) * 8;
            const uint32_t cell = (uint32_t)(buf * CHUNK_CELLS + ((pp * MB + mb) * 16 + 4 * gq) * 16);
            stream_load_to_lds_16(src, lds_base + (uint32_t)__builtin_amdgcn_readfirstlane((int)(cell * 16)));
        }
    };

    f32x4_t acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x4_t{ 0.f, 0.f, 0.f, 0.f };

    Packed w0, w1; // chunks ch and ch + 1
    stage_a(0, 0);
    fetch_w(w0, 0);
    fetch_w(w1, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    auto work = [&](const Packed &pk, int buf, int ch) {
        const uint4 *cells = lds + buf * CHUNK_CELLS;
#pragma unroll
        for (int i = 0; i < CP; ++i) {
            if (ch * CP + i < npairs) { // uniform
                const uint32_t cw[4] = { pk.c[i].x, pk.c[i].y, pk.c[i].z, pk.c[i].w };
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, decode_chunk(cw[t], pk.m[i], 4 * (q & 1) + t));
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const uint4 av = cells[((i * MB + mb) * 16 + 4 * q + t) * 16 + n_l];
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av), bfrag, acc[mb], 0, 0, 0);
                    }
                }
            }
        }
    };

    for (int ch = 0; ch < nchunks; ch += 2) {
        // chunk ch from buffer 0 and w0; its successor's activations land in buffer 1 meanwhile
        stage_a(1, ch + 1);
        work(w0, 0, ch);
        fetch_w(w0, ch + 2);
        // the direct loads above are older than the CP * 2 loads of fetch_w: wait for them only
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 * CP) : "memory");
        __syncthreads();
        stage_a(0, ch + 2);
        work(w1, 1, ch + 1);
        fetch_w(w1, ch + 3);
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 * CP) : "memory");
        __syncthreads();
    }

    // lane (n, q) holds column n, rows 16 mb + 4 q + r
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 16 * mb + 4 * q + r;
            if (row < M && col < N) {
                const float v = acc[mb][r];
                if (OUT_F32) static_cast<float *>(c)[(int64_t)row * ldc + col] = v;
                else static_cast<uint16_t *>(c)[(int64_t)row * ldc + col] = (uint16_t)((f2u(v) + 0x7FFFu + ((f2u(v) >> 16) & 1u)) >> 16);
            }
        }
}

template <int MB>
static int launch_stream_mb(const void *a, int64_t lda, const uint8_t *w_codes, const uint32_t *w_meta, int64_t M, int64_t N,
                            int64_t K, void *c, int64_t ldc, int out_dtype, hipStream_t stream)
{
    constexpr int CP = stream_chunk_pairs(MB);
    constexpr size_t lds_bytes = (size_t)2 * CP * MB * 256 * sizeof(uint4);
    const dim3 grid((unsigned)((N + 63) / 64)), block(256);
    const uint16_t *ap = static_cast<const uint16_t *>(a);
    const uint32_t *wc = reinterpret_cast<const uint32_t *>(w_codes);
    hipError_t e;
    if (out_dtype == HIF4_OUT_F32) {
        auto k = gemm_stream_kernel<MB, true>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, ap, lda, wc, w_meta, c, ldc, (int)M, (int)N, (int)K);
    } else {
        auto k = gemm_stream_kernel<MB, false>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, ap, lda, wc, w_meta, c, ldc, (int)M, (int)N, (int)K);
    }
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// M <= 64, K a multiple of 128 (whole pairs of units).
int launch_gemm_stream(const void *a, int64_t lda, const uint8_t *w_codes, const uint32_t *w_meta, int64_t M, int64_t N, int64_t K,
                       void *c, int64_t ldc, int out_dtype, hipStream_t stream)
{
    if (M <= 16) return launch_stream_mb<1>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
    if (M <= 32) return launch_stream_mb<2>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
    return launch_stream_mb<4>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
}

} // namespace hif4
