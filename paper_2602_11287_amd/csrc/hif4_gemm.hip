// HiF4 GEMM for gfx950:  C[M][N] = A[M][K] * W[N][K]^T, fp32 accumulation on the BF16
// matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Why BF16 MFMA: a decoded HiF4 value is (4+M) * mag * 2^x with at most six significant
// bits, so it is exact in BF16 and the 64-term sum of Eq. 4 (Section III-B of the HiF4
// paper) needs no per-unit rescale of the accumulators.  An int8 or fp8 MFMA holds the
// intra-unit integers exactly but leaves the product of the two E6M2 scales to be applied
// to every accumulator after every 64-wide K step (3 VALU operations per output per unit
// against 64 MACs), which costs more than the 2x MFMA rate gives.
//
// Structure: a workgroup owns a BM x BN tile of C and walks K one unit (64) at a time.
// For each step every thread expands one packed unit (32 bytes of codes + 4 bytes of
// metadata, straight from global memory) to 64 BF16 values and writes them to LDS; the
// waves then read MFMA operands from LDS.  LDS is double-buffered, so the expansion of
// step k+1 overlaps the matrix work of step k.
//
// K order inside a unit: the sum over k may run in any order as long as both operands
// use the same one.  A group of 8 elements j (one dword of codes) becomes one 16-byte LDS
// cell holding its elements in the order 0,1,2,3,4,5,6,7 -> (0,1),(2,3),(4,5),(6,7) as
// BF16 pairs; MFMA sub-step s (of 4) takes cell 2s from lanes 0..31 and cell 2s+1 from
// lanes 32..63.  Cells are stored [j][row], so both the expansion writes and the operand
// reads of a wave touch consecutive 16-byte cells.
#include "hif4_common.h"

namespace hif4 {

// ------------------------------------------------------------------ expansion

// One dword of codes (group of 8 number j of a unit with metadata m) -> 8 BF16 in a uint4.
// `sbase` is the fp32 pattern of (4+M) * 2^(E-52) for the unit, or a NaN pattern.
__device__ __forceinline__ uint4 expand_chunk(uint32_t c, uint32_t m, uint32_t sbase, int j)
{
    const uint32_t e8 = (m >> (8 + j)) & 1u;
    const uint32_t e16a = (m >> (16 + 2 * j)) & 1u, e16b = (m >> (17 + 2 * j)) & 1u;
    const float sa = u2f(sbase + ((e8 + e16a) << 23)), sb = u2f(sbase + ((e8 + e16b) << 23));
    const uint32_t lo = c & 0x07070707u, hi = (c >> 4) & 0x07070707u;
    const uint32_t sl = (c << 4) & 0x80808080u, sh = c & 0x80808080u;
    float f[8];
    f[0] = (float)(lo & 0xFFu) * sa;
    f[1] = (float)((lo >> 8) & 0xFFu) * sa;
    f[2] = (float)((lo >> 16) & 0xFFu) * sa;
    f[3] = (float)(lo >> 24) * sa;
    f[4] = (float)(hi & 0xFFu) * sb;
    f[5] = (float)((hi >> 8) & 0xFFu) * sb;
    f[6] = (float)((hi >> 16) & 0xFFu) * sb;
    f[7] = (float)(hi >> 24) * sb;
    uint32_t r[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const uint32_t pair = __builtin_amdgcn_perm(f2u(f[2 * t + 1]), f2u(f[2 * t]), 0x07060302u);
        const uint32_t sg = __builtin_amdgcn_perm(0u, t < 2 ? sl : sh, (t & 1) ? 0x030C020Cu : 0x010C000Cu);
        r[t] = pair | sg;
    }
    return make_uint4(r[0], r[1], r[2], r[3]);
}

// fp32 pattern of the unit scale (4+M) * 2^(E-48-4), NaN for the NaN unit.
__device__ __forceinline__ uint32_t unit_scale_bits(uint32_t m)
{
    const uint32_t s = ((((m >> 2) & 0x3Fu) + (127u - 50u)) << 23) | ((m & 3u) << 21);
    return (m & 0xFFu) == 0xFFu ? 0x7FC00000u : s;
}

// ------------------------------------------------------------------ kernel

struct GemmArgs {
    const uint32_t *a_codes; // packed A: [M][K/8] dwords, or BF16 A when A_BF16
    const uint32_t *a_meta;  // [M][K/64]
    const uint32_t *w_codes; // [E][N][K/8]
    const uint32_t *w_meta;  // [E][N][K/64]
    const int32_t *offs;     // grouped: device int32[E+1]; else nullptr
    void *c;
    int64_t lda; // BF16 A only: row stride in elements
    int64_t ldc;
    int M, N, K, E;
    int tiles_n;
};

template <int BM, int BN, int WM, int WN, bool A_BF16, bool OUT_F32, bool GROUPED>
__global__ __launch_bounds__(64 * WM * WN) void gemm_kernel(GemmArgs g)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32; // MFMA tiles per wave
    constexpr int CELLS = 8 * (BM + BN);                // 16-byte cells per buffer
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave tiles are multiples of 32");
    extern __shared__ uint4 lds[]; // 2 buffers x CELLS

    const int tid = threadIdx.x;
    const int wave = tid / 64, lane = tid % 64;
    const int wm = wave / WN, wn = wave % WN;

    // ---- which tile
    int row0, rows_end; // this tile covers rows [row0, min(row0 + BM, rows_end)) of A and C
    const uint32_t *w_codes = g.w_codes;
    const uint32_t *w_meta = g.w_meta;
    const int tile_n = blockIdx.x % g.tiles_n;
    int tile_m = blockIdx.x / g.tiles_n;
    if (GROUPED) {
        // walk the experts until the m-tile index falls inside one (uniform across the block)
        int e = 0, acc = 0, found = 0;
        row0 = 0;
        rows_end = 0;
        for (; e < g.E; ++e) {
            const int lo = g.offs[e], hi = g.offs[e + 1];
            const int nt = (hi - lo + BM - 1) / BM;
            if (tile_m < acc + nt) {
                row0 = lo + (tile_m - acc) * BM;
                rows_end = hi;
                found = 1;
                break;
            }
            acc += nt;
        }
        if (!found) return; // grid is an upper bound on the number of tiles
        w_codes += (int64_t)e * g.N * (g.K / 8);
        w_meta += (int64_t)e * g.N * (g.K / 64);
    } else {
        row0 = tile_m * BM;
        rows_end = g.M;
    }
    const int col0 = tile_n * BN;
    const int upr = g.K / 64; // units per row

    // ---- expansion role of this thread: unit `u` of the tile (A rows first, then W rows)
    constexpr int UPT = (BM + BN + NT - 1) / NT; // units per thread per K step
    const uint32_t *src_codes[UPT];
    const uint32_t *src_meta[UPT];
    const uint16_t *src_bf16[UPT];
    int cell0[UPT];
    bool active[UPT];
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
        const int u = tid + i * NT;
        active[i] = u < BM + BN;
        if (u < BM) {
            int r = row0 + u;
            r = r < rows_end ? r : rows_end - 1; // rows past the edge repeat the last one; never stored
            src_codes[i] = g.a_codes + (int64_t)r * (g.K / 8);
            src_meta[i] = g.a_meta + (int64_t)r * upr;
            src_bf16[i] = reinterpret_cast<const uint16_t *>(g.a_codes) + (int64_t)r * g.lda;
            cell0[i] = u;
        } else {
            int r = col0 + (u - BM);
            r = r < g.N ? r : g.N - 1;
            src_codes[i] = w_codes + (int64_t)r * (g.K / 8);
            src_meta[i] = w_meta + (int64_t)r * upr;
            src_bf16[i] = nullptr;
            cell0[i] = 8 * BM + (u - BM);
        }
    }
    // cell (j, row) of the A part sits at j*BM + row; of the W part at 8*BM + j*BN + row

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    uint4 pc[UPT][A_BF16 ? 8 : 2]; // next step: packed codes of a unit, or 64 BF16 of a plain A row
    uint32_t pm[UPT];

    auto fetch = [&](int ks) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            if (!active[i]) continue;
            if (A_BF16 && (tid + i * NT) < BM) {
                const uint4 *p = reinterpret_cast<const uint4 *>(src_bf16[i] + (int64_t)ks * 64);
#pragma unroll
                for (int j = 0; j < 8; ++j) pc[i][j] = p[j];
            } else {
                const uint4 *p = reinterpret_cast<const uint4 *>(src_codes[i] + ks * 8);
                pc[i][0] = p[0];
                pc[i][1] = p[1];
                pm[i] = src_meta[i][ks];
            }
        }
    };
    auto expand_to = [&](uint4 *buf) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            if (!active[i]) continue;
            if (A_BF16 && (tid + i * NT) < BM) { // plain BF16 activations: cells are straight copies
#pragma unroll
                for (int j = 0; j < 8; ++j) buf[cell0[i] + j * BM] = pc[i][j];
                continue;
            }
            const uint32_t sbase = unit_scale_bits(pm[i]);
            const uint32_t cw[8] = { pc[i][0].x, pc[i][0].y, pc[i][0].z, pc[i][0].w,
                                     pc[i][1].x, pc[i][1].y, pc[i][1].z, pc[i][1].w };
            const int stride = (tid + i * NT) < BM ? BM : BN;
#pragma unroll
            for (int j = 0; j < 8; ++j) buf[cell0[i] + j * stride] = expand_chunk(cw[j], pm[i], sbase, j);
        }
    };

    const int nk = upr;
    if (nk > 0) {
        fetch(0);
        expand_to(lds);
    }
    __syncthreads();

    const int half = lane / 32, l32 = lane % 32;
    for (int ks = 0; ks < nk; ++ks) {
        uint4 *cur = lds + (ks & 1) * CELLS;
        uint4 *nxt = lds + ((ks + 1) & 1) * CELLS;
        if (ks + 1 < nk) fetch(ks + 1);

        const uint4 *abase = cur + wm * (BM / WM) + l32;
        const uint4 *bbase = cur + 8 * BM + wn * (BN / WN) + l32;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int j = 2 * s + half;
            bf16x8_t af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = __builtin_bit_cast(bf16x8_t, abase[j * BM + i * 32]);
#pragma unroll
            for (int i = 0; i < TN; ++i) bfr[i] = __builtin_bit_cast(bf16x8_t, bbase[j * BN + i * 32]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int jn = 0; jn < TN; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[jn], acc[i][jn], 0, 0, 0);
        }
        if (ks + 1 < nk) expand_to(nxt);
        __syncthreads();
    }

    // ---- epilogue: lane holds column l32 of each 32x32 tile, rows 8*(r/4) + 4*half + r%4
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
            const int col = col0 + wn * (BN / WN) + jn * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + wm * (BM / WM) + i * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                if (row < rows_end && col < g.N) {
                    const float v = acc[i][jn][r];
                    if (OUT_F32) {
                        static_cast<float *>(g.c)[(int64_t)row * g.ldc + col] = v;
                    } else {
                        static_cast<uint16_t *>(g.c)[(int64_t)row * g.ldc + col] = (uint16_t)((f2u(v) + 0x7FFFu + ((f2u(v) >> 16) & 1u)) >> 16);
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------ skinny weight-only GEMM

// C[M][N] = A[M][K] (BF16) * W[N][K]^T (HiF4) for M <= 16 * MB: bound by streaming W once
// from HBM.  A workgroup owns 16 output columns; its 8 waves split K by pairs of units and
// add their partial tiles through LDS.  v_mfma_f32_16x16x32_bf16: lane (n, q) = (lane % 16,
// lane / 16) supplies 8 consecutive k of weight row n (one dword of codes, expanded in
// registers, never through LDS) and of activation row n; for the pair of units (2p, 2p+1)
// lane q loads the 16 code bytes [16 q, 16 q + 16) of the 64-byte pair, so a weight row's
// bytes are read as one contiguous run.
template <int MB, bool OUT_F32>
__global__ __launch_bounds__(512) void gemm_skinny_kernel(const uint16_t *__restrict__ a, int64_t lda,
                                                          const uint32_t *__restrict__ w_codes,
                                                          const uint32_t *__restrict__ w_meta, void *c, int64_t ldc,
                                                          int M, int N, int K)
{
    constexpr int KS = 8;
    __shared__ float red[KS][MB][256];
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int n_l = lane % 16, q = lane / 16;
    const int col = blockIdx.x * 16 + n_l;
    const int colc = col < N ? col : N - 1;
    const int upr = K / 64, npairs = (upr + 1) / 2;
    const uint32_t *wrow = w_codes + (int64_t)colc * (K / 8);
    const uint32_t *mrow = w_meta + (int64_t)colc * upr;

    f32x4_t acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x4_t{ 0.f, 0.f, 0.f, 0.f };

    for (int p = wave; p < npairs; p += KS) {
        const int u = 2 * p + (q >> 1);
        const bool valid = u < upr;
        const int uc = valid ? u : upr - 1;
        uint4 cw = *reinterpret_cast<const uint4 *>(wrow + uc * 8 + (q & 1) * 4);
        uint32_t meta = mrow[uc];
        if (!valid) { cw = make_uint4(0, 0, 0, 0); meta = 0; } // an odd unit count: the missing half adds zeros
        const uint32_t sbase = unit_scale_bits(meta);
        const uint32_t cwa[4] = { cw.x, cw.y, cw.z, cw.w };
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = 4 * (q & 1) + t;
            const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, expand_chunk(cwa[t], meta, sbase, j));
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int row = mb * 16 + n_l;
                uint4 av = make_uint4(0, 0, 0, 0);
                if (valid && row < M) av = *reinterpret_cast<const uint4 *>(a + (int64_t)row * lda + (int64_t)uc * 64 + j * 8);
                acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av), bfrag, acc[mb], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][mb][r * 64 + lane] = acc[mb][r];
    __syncthreads();
    // thread -> (mb, r, lane): output row mb*16 + 4*(lane/16) + r, column lane%16
    for (int idx = tid; idx < MB * 256; idx += 512) {
        const int mb = idx / 256, rem = idx % 256, r = rem / 64, ln = rem % 64;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < KS; ++w) v += red[w][mb][rem];
        const int row = mb * 16 + 4 * (ln / 16) + r, cc = blockIdx.x * 16 + (ln % 16);
        if (row < M && cc < N) {
            if (OUT_F32) static_cast<float *>(c)[(int64_t)row * ldc + cc] = v;
            else static_cast<uint16_t *>(c)[(int64_t)row * ldc + cc] = (uint16_t)((f2u(v) + 0x7FFFu + ((f2u(v) >> 16) & 1u)) >> 16);
        }
    }
}

template <int MB>
static int launch_skinny(const void *a, int64_t lda, const uint8_t *w_codes, const uint32_t *w_meta, int64_t M, int64_t N,
                         int64_t K, void *c, int64_t ldc, int out_dtype, hipStream_t stream)
{
    const dim3 grid((unsigned)((N + 15) / 16)), block(512);
    const uint16_t *ap = static_cast<const uint16_t *>(a);
    const uint32_t *wc = reinterpret_cast<const uint32_t *>(w_codes);
    if (out_dtype == HIF4_OUT_F32)
        hipLaunchKernelGGL((gemm_skinny_kernel<MB, true>), grid, block, 0, stream, ap, lda, wc, w_meta, c, ldc, (int)M, (int)N, (int)K);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<MB, false>), grid, block, 0, stream, ap, lda, wc, w_meta, c, ldc, (int)M, (int)N, (int)K);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

__global__ void zero_kernel(void *c, int64_t M, int64_t N, int64_t ldc, int elem_bytes)
{
    const int64_t col = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (col >= N) return;
    for (int64_t row = blockIdx.y; row < M; row += gridDim.y) {
        if (elem_bytes == 4) static_cast<uint32_t *>(c)[row * ldc + col] = 0u;
        else static_cast<uint16_t *>(c)[row * ldc + col] = 0;
    }
}

// ------------------------------------------------------------------ launch

int launch_encode(const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode,
                  hipStream_t stream);

template <int BM, int BN, int WM, int WN, bool A_BF16, bool GROUPED>
static int launch_tiles(const GemmArgs &g, int out_dtype, int m_tiles, hipStream_t stream)
{
    constexpr size_t lds_bytes = 2 * 8 * (BM + BN) * sizeof(uint4);
    const dim3 grid((unsigned)((int64_t)m_tiles * g.tiles_n)), block(64 * WM * WN);
    hipError_t e;
    if (out_dtype == HIF4_OUT_F32) {
        auto k = gemm_kernel<BM, BN, WM, WN, A_BF16, true, GROUPED>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, g);
    } else {
        auto k = gemm_kernel<BM, BN, WM, WN, A_BF16, false, GROUPED>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, g);
    }
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
                const uint32_t *w_meta, const int32_t *offs, int E, int64_t M, int64_t N, int64_t K, void *c,
                int64_t ldc, int out_dtype, void *workspace, hipStream_t stream)
{
    if (K == 0) { // empty sum: C = 0 (a fill kernel, so that the call can be captured in a graph)
        const dim3 grid((unsigned)((N + 255) / 256), (unsigned)(M < 65535 ? M : 65535)), block(256);
        hipLaunchKernelGGL(zero_kernel, grid, block, 0, stream, c, M, N, ldc, out_dtype == HIF4_OUT_F32 ? 4 : 2);
        return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
    }
    if (a_kind == HIF4_A_BF16_KEEP && !offs && M <= 64) { // decode-shaped: stream the weights once
        if (M <= 16) return launch_skinny<1>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
        if (M <= 32) return launch_skinny<2>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
        return launch_skinny<4>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
    }
    GemmArgs g;
    if (a_kind == HIF4_A_BF16_KEEP) {
        g.a_codes = static_cast<const uint32_t *>(a); // BF16 rows, staged as they are
        g.a_meta = nullptr;
    } else if (a_kind == HIF4_A_BF16_QUANTIZE) {
        // quantise A into the workspace: codes plane, then the meta plane at the next 16-byte boundary
        uint8_t *codes = static_cast<uint8_t *>(workspace);
        const size_t cbytes = ((size_t)M * (size_t)K / 2 + 15) & ~(size_t)15;
        uint32_t *meta = reinterpret_cast<uint32_t *>(codes + cbytes);
        if (int rc = launch_encode(a, M, K, lda, codes, meta, HIF4_ROUND_RNE, stream)) return rc;
        g.a_codes = reinterpret_cast<const uint32_t *>(codes);
        g.a_meta = meta;
    } else {
        g.a_codes = static_cast<const uint32_t *>(a);
        g.a_meta = a_meta;
    }
    g.w_codes = reinterpret_cast<const uint32_t *>(w_codes);
    g.w_meta = w_meta;
    g.offs = offs;
    g.c = c;
    g.lda = lda;
    g.ldc = ldc;
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    g.E = E;
    if (offs) {
        constexpr int BM = 128, BN = 256;
        g.tiles_n = (int)((N + BN - 1) / BN);
        const int m_tiles = (int)(M / BM) + E; // upper bound of sum_e ceil(rows_e / BM)
        if (a_kind == HIF4_A_BF16_KEEP) return launch_tiles<BM, BN, 2, 4, true, true>(g, out_dtype, m_tiles, stream);
        return launch_tiles<BM, BN, 2, 4, false, true>(g, out_dtype, m_tiles, stream);
    }
    constexpr int BM = 256, BN = 256;
    g.tiles_n = (int)((N + BN - 1) / BN);
    const int m_tiles = (int)((M + BM - 1) / BM);
    if (a_kind == HIF4_A_BF16_KEEP) return launch_tiles<BM, BN, 2, 4, true, false>(g, out_dtype, m_tiles, stream);
    return launch_tiles<BM, BN, 2, 4, false, false>(g, out_dtype, m_tiles, stream);
}

} // namespace hif4
