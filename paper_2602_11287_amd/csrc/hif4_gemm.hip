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
// cell holding its elements in the order 0,2,1,3,4,6,5,7 (see expand_chunk) as BF16
// pairs; MFMA sub-step s (of 4) takes cell 2s from lanes 0..31 and cell 2s+1 from
// lanes 32..63.  Cells are stored [j][row], so both the expansion writes and the operand
// reads of a wave touch consecutive 16-byte cells.
#include "hif4_common.h"

#ifndef HIF4_GEMM_SCHED
#define HIF4_GEMM_SCHED 1
#endif

namespace hif4 {

// ------------------------------------------------------------------ expansion

// One dword of codes (group of 8 number j of a unit with metadata m) -> 8 BF16 in a uint4,
// in the cell order e0,e2 | e1,e3 | e4,e6 | e5,e7 (the K order inside a cell is free as long
// as both operands share it; this one puts the two sign bits of every pair 16 bits apart in
// the codes dword, so one shift and one bit-field insert place both).
// `sbase` is the fp32 pattern of (4+M) * 2^(E-52) for the unit, or a NaN pattern.
__device__ __forceinline__ uint4 expand_chunk(uint32_t c, uint32_t m, uint32_t sbase, int j)
{
    const uint32_t e8 = (m >> (8 + j)) & 1u;
    const uint32_t e16a = (m >> (16 + 2 * j)) & 1u, e16b = (m >> (17 + 2 * j)) & 1u;
    const float sa = u2f(sbase + ((e8 + e16a) << 23)), sb = u2f(sbase + ((e8 + e16b) << 23));
    uint32_t lo = c & 0x07070707u, hi = (c >> 4) & 0x07070707u; // magnitudes of elements 0..3 / 4..7, one per byte
    asm volatile("" : "+v"(lo), "+v"(hi));                      // keep them as bytes: v_cvt_f32_ubyteN reads them in place
    const float f0 = (float)(lo & 0xFFu) * sa, f1 = (float)((lo >> 8) & 0xFFu) * sa;
    const float f2 = (float)((lo >> 16) & 0xFFu) * sa, f3 = (float)(lo >> 24) * sa;
    const float f4 = (float)(hi & 0xFFu) * sb, f5 = (float)((hi >> 8) & 0xFFu) * sb;
    const float f6 = (float)((hi >> 16) & 0xFFu) * sb, f7 = (float)(hi >> 24) * sb;
    // exact values: the BF16 form is the top half of the fp32 pattern.  Signs: element t at
    // bit 8t+3, element 4+t at bit 8t+7 of c.
    constexpr uint32_t MAG = 0x7FFF7FFFu;
    uint4 r;
    r.x = bfi(MAG, __builtin_amdgcn_perm(f2u(f2), f2u(f0), 0x07060302u), c << 12);
    r.y = bfi(MAG, __builtin_amdgcn_perm(f2u(f3), f2u(f1), 0x07060302u), c << 4);
    r.z = bfi(MAG, __builtin_amdgcn_perm(f2u(f6), f2u(f4), 0x07060302u), c << 8);
    r.w = bfi(MAG, __builtin_amdgcn_perm(f2u(f7), f2u(f5), 0x07060302u), c);
    return r;
}

// The same expansion cut into five pieces, so that the GEMM main loop can place one piece
// after each MFMA: chunk_begin (masks and the two group scales), then four pairs.
struct ChunkState {
    uint32_t c, lo, hi;
    float sa, sb;
};

__device__ __forceinline__ ChunkState chunk_begin(uint32_t c, uint32_t m, uint32_t sbase, int j)
{
    ChunkState st;
    const uint32_t e8 = (m >> (8 + j)) & 1u;
    const uint32_t e16a = (m >> (16 + 2 * j)) & 1u, e16b = (m >> (17 + 2 * j)) & 1u;
    st.sa = u2f(sbase + ((e8 + e16a) << 23));
    st.sb = u2f(sbase + ((e8 + e16b) << 23));
    st.c = c;
    st.lo = c & 0x07070707u;
    st.hi = (c >> 4) & 0x07070707u;
    asm volatile("" : "+v"(st.lo), "+v"(st.hi));
    return st;
}

template <int T>
__device__ __forceinline__ uint32_t chunk_pair(const ChunkState &st)
{
    constexpr uint32_t MAG = 0x7FFF7FFFu;
    if (T == 0) return bfi(MAG, __builtin_amdgcn_perm(f2u((float)((st.lo >> 16) & 0xFFu) * st.sa), f2u((float)(st.lo & 0xFFu) * st.sa), 0x07060302u), st.c << 12);
    if (T == 1) return bfi(MAG, __builtin_amdgcn_perm(f2u((float)(st.lo >> 24) * st.sa), f2u((float)((st.lo >> 8) & 0xFFu) * st.sa), 0x07060302u), st.c << 4);
    if (T == 2) return bfi(MAG, __builtin_amdgcn_perm(f2u((float)((st.hi >> 16) & 0xFFu) * st.sb), f2u((float)(st.hi & 0xFFu) * st.sb), 0x07060302u), st.c << 8);
    return bfi(MAG, __builtin_amdgcn_perm(f2u((float)(st.hi >> 24) * st.sb), f2u((float)((st.hi >> 8) & 0xFFu) * st.sb), 0x07060302u), st.c);
}

// 8 consecutive plain BF16 values -> the same cell order.
__device__ __forceinline__ uint4 permute_bf16_cell(uint4 v)
{
    uint4 r;
    r.x = __builtin_amdgcn_perm(v.y, v.x, 0x05040100u); // e0, e2
    r.y = __builtin_amdgcn_perm(v.y, v.x, 0x07060302u); // e1, e3
    r.z = __builtin_amdgcn_perm(v.w, v.z, 0x05040100u); // e4, e6
    r.w = __builtin_amdgcn_perm(v.w, v.z, 0x07060302u); // e5, e7
    return r;
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

    // ---- expansion role of this thread: unit `u` of the tile (A rows first, then W rows).
    // With fewer units than threads the surplus threads repeat the last units (same bytes to
    // the same cells), which keeps the loop body free of branches.
    static_assert(BM + BN <= NT, "one unit per thread and K step");
    const int u = tid < BM + BN ? tid : tid - (NT - BN);
    const bool is_a = u < BM;
    const uint32_t *src_codes;
    const uint32_t *src_meta;
    int cell0, cstride;
    if (is_a) {
        int r = row0 + u;
        r = r < rows_end ? r : rows_end - 1; // rows past the edge repeat the last one; never stored
        src_codes = A_BF16 ? g.a_codes + (int64_t)r * (g.lda / 2) : g.a_codes + (int64_t)r * (g.K / 8);
        src_meta = A_BF16 ? g.w_meta : g.a_meta + (int64_t)r * upr; // (unused for plain BF16 rows)
        cell0 = u;
        cstride = BM;
    } else {
        int r = col0 + (u - BM);
        r = r < g.N ? r : g.N - 1;
        src_codes = w_codes + (int64_t)r * (g.K / 8);
        src_meta = w_meta + (int64_t)r * upr;
        cell0 = 8 * BM + (u - BM);
        cstride = BN;
    }
    // cell (j, row) of the A part sits at j*BM + row; of the W part at 8*BM + j*BN + row
    const bool plain = A_BF16 && is_a; // wave-uniform: BM is a multiple of 64

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Two register sets of packed input, two K steps ahead of the matrix work.
    constexpr int NPC = A_BF16 ? 8 : 2;
    struct Packed { uint4 c[NPC]; uint32_t m; };
    const int nk = upr;

    auto fetch = [&](Packed &pk, int ks) {
        ks = ks < nk ? ks : nk - 1; // past the end: reload the last step, never used
        if (plain) {
            const uint4 *p = reinterpret_cast<const uint4 *>(src_codes + (int64_t)ks * 32);
#pragma unroll
            for (int j = 0; j < NPC; ++j) pk.c[j] = p[j];
            pk.m = 0;
        } else {
            const uint4 *p = reinterpret_cast<const uint4 *>(src_codes + ks * 8);
            pk.c[0] = p[0];
            pk.c[1] = p[1];
            pk.m = src_meta[ks];
        }
    };
    // cells 2q and 2q+1 of this thread's unit -> LDS
    auto expand_quarter = [&](const Packed &pk, uint4 *buf, int q) {
        if (plain) {
            if (NPC == 8) {
                buf[cell0 + (2 * q) * cstride] = permute_bf16_cell(pk.c[(2 * q) % NPC]);
                buf[cell0 + (2 * q + 1) * cstride] = permute_bf16_cell(pk.c[(2 * q + 1) % NPC]);
            }
        } else {
            const uint32_t sbase = unit_scale_bits(pk.m);
            const uint4 cw = pk.c[q / 2];
            const uint32_t c0 = (q & 1) ? cw.z : cw.x, c1 = (q & 1) ? cw.w : cw.y;
            buf[cell0 + (2 * q) * cstride] = expand_chunk(c0, pk.m, sbase, 2 * q);
            buf[cell0 + (2 * q + 1) * cstride] = expand_chunk(c1, pk.m, sbase, 2 * q + 1);
        }
    };

    const int half = lane / 32, l32 = lane % 32;
    constexpr int NMF = TM * TN;  // MFMAs per quarter step
    constexpr int SPM = 8 / NMF;  // expansion slices (BF16 pairs) placed after each MFMA
    static_assert(NMF * SPM == 8, "the 8 pairs of a quarter are spread evenly over its MFMAs");

    // One K step: matrix work on `cur`, expansion of the following step from `pk` into `nxt`.
    // A step has four quarters (one MFMA K-slab of 16 each); a quarter issues TM*TN = 8 MFMAs
    // and expands two cells (8 BF16 pairs): one pair after each MFMA, fenced, so that the
    // VALU work runs while the matrix pipeline is busy.  Operand reads of the next quarter are
    // issued in the middle of the current one.
    auto k_step = [&](const uint4 *cur, uint4 *nxt, const Packed &pk) {
        const uint4 *abase = cur + wm * (BM / WM) + l32;
        const uint4 *bbase = cur + 8 * BM + wn * (BN / WN) + l32;
        bf16x8_t af[2][TM], bfr[2][TN];
        auto load_frags = [&](int s) {
            const int j = 2 * s + half;
#pragma unroll
            for (int i = 0; i < TM; ++i) af[s & 1][i] = __builtin_bit_cast(bf16x8_t, abase[j * BM + i * 32]);
#pragma unroll
            for (int i = 0; i < TN; ++i) bfr[s & 1][i] = __builtin_bit_cast(bf16x8_t, bbase[j * BN + i * 32]);
        };
        const uint32_t sbase = unit_scale_bits(pk.m);
        load_frags(0);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            ChunkState st;
            uint4 cell;
#pragma unroll
            for (int tm = 0; tm < NMF; ++tm) {
                acc[tm / TN][tm % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s & 1][tm / TN], bfr[s & 1][tm % TN], acc[tm / TN][tm % TN], 0, 0, 0);
#pragma unroll
                for (int sl = 0; sl < SPM; ++sl) {
                    const int t = tm * SPM + sl;  // slice 0..7 of this quarter
                    const int jc = 2 * s + t / 4; // cell being expanded
                    if (plain) {
                        if (NPC == 8 && t % 4 == 0) nxt[cell0 + jc * cstride] = permute_bf16_cell(pk.c[jc % NPC]);
                    } else {
                        if (t % 4 == 0) {
                            const uint4 cw = pk.c[(jc / 4) % NPC];
                            const uint32_t cj = (jc % 4 == 0) ? cw.x : (jc % 4 == 1) ? cw.y : (jc % 4 == 2) ? cw.z : cw.w;
                            st = chunk_begin(cj, pk.m, sbase, jc);
                            cell.x = chunk_pair<0>(st);
                        } else if (t % 4 == 1) {
                            cell.y = chunk_pair<1>(st);
                        } else if (t % 4 == 2) {
                            cell.z = chunk_pair<2>(st);
                        } else {
                            cell.w = chunk_pair<3>(st);
                            nxt[cell0 + jc * cstride] = cell;
                        }
                    }
                }
                if (tm == NMF / 4 && s < 3) load_frags(s + 1);
#if HIF4_GEMM_SCHED
                __builtin_amdgcn_sched_barrier(0);
#endif
            }
        }
    };

    uint4 *buf0 = lds, *buf1 = lds + CELLS;
    Packed set0, set1;
    fetch(set0, 0);
    fetch(set1, 1);
#pragma unroll
    for (int q = 0; q < 4; ++q) expand_quarter(set0, buf0, q);
    fetch(set0, 2);
    __syncthreads();

    for (int ks = 0; ks < nk; ks += 2) {
        k_step(buf0, buf1, set1); // matrix work of step ks, expansion of step ks+1
        fetch(set1, ks + 3);
        __syncthreads();
        if (ks + 1 < nk) {
            k_step(buf1, buf0, set0); // step ks+1, expansion of step ks+2
            fetch(set0, ks + 4);
            __syncthreads();
        }
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
                if (valid && row < M) av = permute_bf16_cell(*reinterpret_cast<const uint4 *>(a + (int64_t)row * lda + (int64_t)uc * 64 + j * 8));
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
