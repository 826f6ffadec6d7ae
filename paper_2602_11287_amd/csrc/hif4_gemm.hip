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
#include "hif4_emit.h"
#include "hif4_expand.h"
#include "hif4_grouped.h"
#include "hif4_store.h"

#ifndef HIF4_GEMM_SCHED
#define HIF4_GEMM_SCHED 1
#endif

namespace hif4 {

// ------------------------------------------------------------------ kernel

struct GemmArgs {
    const uint16_t *a;       // BF16 activations [M][lda]: plain rows, or rows already in cell order
    const uint32_t *w_codes; // [E][N][K/8] dwords
    const uint32_t *w_meta;  // [E][N][K/64]
    const int32_t *offs;     // grouped: device int32[E+1]; else nullptr
    void *c;
    uint32_t *c_meta; // EMIT kernels: c is the codes plane [M][N/2] of the HiF4 result, this its metadata plane
    int64_t lda; // row stride of a, in elements
    int64_t ldc;
    int M, N, K, E;
    int tiles_m, tiles_n;
};

// A_CELL: the 8 BF16 of every group of 8 in `a` are already stored in cell order (the
// library's own decoded copy of a HiF4 operand); otherwise they are permuted on the way in.
// EMIT >= 0: the result is written as HiF4 with units along N (rounding mode EMIT), see hif4_emit.h.
template <int BM, int BN, int WM, int WN, bool A_CELL, bool OUT_F32, bool GROUPED, int EMIT = -1>
__global__ __launch_bounds__(64 * WM * WN, 2) void gemm_kernel(GemmArgs g)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32; // MFMA tiles per wave
    constexpr int PAD = 4;                              // cells; see the staging role below
    constexpr int W_BASE = 8 * BM + PAD;                // first cell of the W part of a buffer
    constexpr int CELLS = 8 * (BM + BN) + 2 * PAD;      // 16-byte cells per buffer
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "wave tiles are multiples of 32");
    static_assert(2 * BM <= NT && 2 * BN <= NT, "two threads per row");
    extern __shared__ uint4 lds[]; // 2 buffers x CELLS

    const int tid = threadIdx.x;
    const int wave = tid / 64, lane = tid % 64;
    const int wm = wave / WN, wn = wave % WN;

    // ---- which tile
    int row0, rows_end; // this tile covers rows [row0, min(row0 + BM, rows_end)) of A and C
    const uint32_t *w_codes = g.w_codes;
    const uint32_t *w_meta = g.w_meta;
    // Block -> tile: see dense_tile_of_block.
    constexpr int XCDS = 8;
    int tile_m, tile_n;
    if (GROUPED) {
        // The tile list of a grouped GEMM ends in an unknown number of empty m-tiles (the grid
        // is an upper bound), so m-tiles are dealt to the XCDs round-robin instead, all n-tiles
        // of an m-tile staying on one XCD (they share its A rows).
        const int i = (int)(blockIdx.x / XCDS);
        tile_m = (i / g.tiles_n) * XCDS + (int)(blockIdx.x % XCDS);
        tile_n = i % g.tiles_n;
        if (tile_m >= g.tiles_m) return;
    } else {
        if (!dense_tile_of_block(g.tiles_m, g.tiles_n, tile_m, tile_n)) return;
    }
    if (GROUPED) {
        int e;
        if (!find_expert_tile<BM>(g.offs, g.E, g.M, tile_m, lane, e, row0, rows_end)) return;
        w_codes += (int64_t)e * g.N * (g.K / 8);
        w_meta += (int64_t)e * g.N * (g.K / 64);
    } else {
        row0 = tile_m * BM;
        rows_end = g.M;
    }
    const int col0 = tile_n * BN;
    const int upr = g.K / 64; // units per row
    const int nk = upr;

    // ---- staging role of this thread, per K step: half a packed unit of a W row (4 dwords of
    // codes -> 4 cells) and half a unit of an A row (64 bytes of BF16 -> 4 cells).  With fewer
    // rows than thread pairs the surplus threads repeat rows (same bytes to the same cells),
    // which keeps the loop body free of branches.
    // Two adjacent lanes share a row (its two 64-byte halves), so the global loads of a wave
    // cover whole 128-byte lines.  In LDS the cells of groups 4..7 are shifted by PAD cells,
    // which moves the writes of the odd lanes to other banks than those of the even lanes.
    const int h = tid & 1;
    const int ra = (tid >> 1) % BM, rw = (tid >> 1) % BN;
    int arow = row0 + ra;
    arow = arow < rows_end ? arow : rows_end - 1; // rows past the edge repeat the last one; never stored
    int wrow = col0 + rw;
    wrow = wrow < g.N ? wrow : g.N - 1;
    const uint16_t *a_src = g.a + (int64_t)arow * g.lda + 32 * h;
    const uint32_t *wc_src = w_codes + (int64_t)wrow * (g.K / 8) + 4 * h;
    const uint32_t *wm_src = w_meta + (int64_t)wrow * upr;
    // cell (j, row) of the A part sits at j*BM + row + PAD*(j/4); the W part follows it
    const int a_cell0 = (4 * h) * BM + ra + PAD * h, w_cell0 = W_BASE + (4 * h) * BN + rw + PAD * h;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Two register sets of staged input, two K steps ahead of the matrix work.
    struct Staged {
        uint4 wc;
        uint32_t wm;
        uint4 a[4];
    };
    auto fetch = [&](Staged &st, int ks) {
        ks = ks < nk ? ks : nk - 1; // past the end: reload the last step, never used
        st.wc = *reinterpret_cast<const uint4 *>(wc_src + ks * 8);
        st.wm = wm_src[ks];
        const uint4 *p = reinterpret_cast<const uint4 *>(a_src + (int64_t)ks * 64);
#pragma unroll
        for (int j = 0; j < 4; ++j) st.a[j] = p[j];
    };
    auto a_cell = [&](const Staged &st, int q) { return A_CELL ? st.a[q] : permute_bf16_cell(st.a[q]); };
    auto w_word = [&](const Staged &st, int q) { return q == 0 ? st.wc.x : q == 1 ? st.wc.y : q == 2 ? st.wc.z : st.wc.w; };

    const int half = lane / 32, l32 = lane % 32;
    // a wave whose rows all lie past the edge of the tile only helps with staging
    const bool wave_has_rows = !GROUPED || row0 + wm * (BM / WM) < rows_end;
    constexpr int NMF = TM * TN; // MFMAs per quarter step
    constexpr int SPM = 8 / NMF; // staging slots after each MFMA
    static_assert(NMF * SPM == 8, "eight staging slots per quarter, spread evenly over its MFMAs");

    // One K step: matrix work on `cur`, staging of the following step from `st` into `nxt`.
    // A step has four phases.  Phase p requests the MFMA operands of quarter p (a K-slab of 16)
    // from LDS and meanwhile runs the MFMAs of quarter p-1, whose operands arrived during the
    // phase before; for p = 0 that is the last quarter of the previous step, still in registers.
    // So the barrier between two steps falls between the operand reads of a quarter and its
    // MFMAs: right after it every wave has a quarter of matrix work to issue while the first
    // operands of the new buffer are on their way (the operand registers start out as zeros, so
    // the first step's phase 0 adds nothing; the last quarter is worked off after the loop).
    // In phase p the thread also expands its W dword p (begin + 4 BF16 pairs) and copies its A
    // cell p: one slot of that work after each MFMA, fenced, so that the VALU work runs while
    // the matrix pipeline is busy.
    bf16x8_t af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[1][i] = bf16x8_t{ 0, 0, 0, 0, 0, 0, 0, 0 };
#pragma unroll
    for (int i = 0; i < TN; ++i) bfr[1][i] = bf16x8_t{ 0, 0, 0, 0, 0, 0, 0, 0 };
    auto mfma = [&](int fb, int tm) {
        if (wave_has_rows)
            acc[tm / TN][tm % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[fb][tm / TN], bfr[fb][tm % TN], acc[tm / TN][tm % TN], 0, 0, 0);
    };
    auto fence = [] {
#if HIF4_GEMM_SCHED
        __builtin_amdgcn_sched_barrier(0);
#endif
    };
    auto k_step = [&](const uint4 *cur, uint4 *nxt, const Staged &st) {
        const uint4 *abase = cur + wm * (BM / WM) + l32;
        const uint4 *bbase = cur + W_BASE + wn * (BN / WN) + l32;
        auto load_frags = [&](int s) {
            if (!wave_has_rows) return;
            const int j = 2 * s + half;
#pragma unroll
            for (int i = 0; i < TM; ++i) af[s & 1][i] = __builtin_bit_cast(bf16x8_t, abase[j * BM + (s / 2) * PAD + i * 32]);
#pragma unroll
            for (int i = 0; i < TN; ++i) bfr[s & 1][i] = __builtin_bit_cast(bf16x8_t, bbase[j * BN + (s / 2) * PAD + i * 32]);
        };
        const uint32_t sbase = unit_scale_bits(st.wm);
        ChunkState cs = chunk_begin(w_word(st, 0), st.wm, sbase, 4 * h);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 cell;
            load_frags(s);
            fence();
#pragma unroll
            for (int tm = 0; tm < NMF; ++tm) {
                mfma((s + 1) & 1, tm);
#pragma unroll
                for (int sl = 0; sl < SPM; ++sl) {
                    const int slot = tm * SPM + sl;
                    if (slot == 0) {
                        cell.x = chunk_pair<0>(cs);
                    } else if (slot == 1) {
                        cell.y = chunk_pair<1>(cs);
                    } else if (slot == 2) {
                        cell.z = chunk_pair<2>(cs);
                    } else if (slot == 3) {
                        cell.w = chunk_pair<3>(cs);
                        nxt[w_cell0 + s * BN] = cell;
                    } else if (slot == 4) {
                        nxt[a_cell0 + s * BM] = a_cell(st, s);
                    } else if (slot == 5) {
                        if (s < 3) cs = chunk_begin(w_word(st, s + 1), st.wm, sbase, 4 * h + s + 1);
                    }
                }
                fence();
            }
        }
    };

    uint4 *buf0 = lds, *buf1 = lds + CELLS;
    Staged set0, set1;
    fetch(set0, 0);
    fetch(set1, 1);
    {
        const uint32_t sbase = unit_scale_bits(set0.wm);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            buf0[w_cell0 + q * BN] = expand_chunk(w_word(set0, q), set0.wm, sbase, 4 * h + q);
            buf0[a_cell0 + q * BM] = a_cell(set0, q);
        }
    }
    fetch(set0, 2);
    __syncthreads();

    for (int ks = 0; ks < nk; ks += 2) {
        k_step(buf0, buf1, set1); // matrix work of step ks, staging of step ks+1
        fetch(set1, ks + 3);
        __syncthreads();
        if (ks + 1 < nk) {
            k_step(buf1, buf0, set0); // step ks+1, staging of step ks+2
            fetch(set0, ks + 4);
            __syncthreads();
        }
    }
#pragma unroll
    for (int tm = 0; tm < NMF; ++tm) mfma(1, tm); // quarter 3 of the last step

    if constexpr (EMIT >= 0) {
        emit_hif4_tile<BM, BN, WM, WN, EMIT>(acc, lds, row0, rows_end, col0, g.N, static_cast<uint32_t *>(g.c), g.c_meta);
        return;
    }
    // ---- epilogue: lane holds column l32 of each 32x32 tile, rows 8*(r/4) + 4*half + r%4
    store_acc_32x32<OUT_F32>(acc, g.c, g.ldc, row0 + wm * (BM / WM), col0 + wn * (BN / WN), rows_end, g.N);
}

// ------------------------------------------------------------------ skinny weight-only GEMM

#ifndef HIF4_SKINNY_NBUF1
#define HIF4_SKINNY_NBUF1 1
#endif
#ifndef HIF4_SKINNY_NBUF2
#define HIF4_SKINNY_NBUF2 1
#endif
#ifndef HIF4_SKINNY_NBUF4
#define HIF4_SKINNY_NBUF4 1
#endif
#ifndef HIF4_SKINNY_WAVES4
#define HIF4_SKINNY_WAVES4 8
#endif
// waves per workgroup and pairs of units in flight per wave, by the number of 16-row blocks (measured
// on MI355X: more pairs in flight cost registers, and occupancy is worth more)
#ifndef HIF4_SKINNY_WAVES12
#define HIF4_SKINNY_WAVES12 8
#endif
constexpr int skinny_waves(int mb) { return mb == 4 ? HIF4_SKINNY_WAVES4 : HIF4_SKINNY_WAVES12; }
constexpr int skinny_nbuf(int mb) { return mb == 1 ? HIF4_SKINNY_NBUF1 : mb == 2 ? HIF4_SKINNY_NBUF2 : HIF4_SKINNY_NBUF4; }

// C[M][N] = A[M][K] (BF16) * W[N][K]^T (HiF4) for M <= 16 * MB: bound by streaming W once
// from HBM.  A workgroup owns 16 output columns; its waves split K into contiguous ranges and
// add their partial tiles through LDS at the end.  v_mfma_f32_16x16x32_bf16: lane (n, q) =
// (lane % 16, lane / 16) supplies 8 consecutive k of weight row n (one dword of codes,
// expanded in registers) and of activation row n.
// K advances by pairs of units (128 values).  For a pair, lane (n, q) loads the 16 code
// bytes [16 q, 16 q + 16) of row n's 64 bytes, so a weight row is read as one contiguous run;
// MFMA t (0..3) of the pair then takes group 4 q + t of the pair's 16 groups of 8.  The
// activations of the pair (16 MB rows x 256 bytes) are loaded with fully coalesced 16-byte
// loads (16 lanes per row), written to a wave-private LDS slab [group][row] in cell order and
// read back in the MFMA operand layout; no workgroup barrier is involved.  One pair is in
// flight per wave in registers while the pair before it is worked on: what hides the memory
// latency is occupancy (about 80 registers and 4 KB of LDS per wave let three workgroups share
// a CU; with four pairs in flight per wave and one workgroup per CU the same kernel was measured
// 20 to 35 % slower).
// A_CELL: the rows of `a` already hold every group of 8 in cell order (the library's decoded copy of HiF4
// activations, see launch_decode_cells): no permutation on the way in.
template <int MB, int WAVES, bool OUT_F32, bool A_CELL = false>
__global__ __launch_bounds__(64 * WAVES) void gemm_skinny_kernel(const uint16_t *__restrict__ a, int64_t lda,
                                                                 const uint32_t *__restrict__ w_codes,
                                                                 const uint32_t *__restrict__ w_meta, void *c,
                                                                 int64_t ldc, int M, int N, int K)
{
    constexpr int NBUF = skinny_nbuf(MB);
    constexpr int ROWS = 16 * MB, RSTRIDE = ROWS + 1; // +1 cell: the 16 lanes of a row write 16 different banks
    constexpr int SLAB = 16 * RSTRIDE;                // cells per pair
    constexpr int NLD = ROWS / 4;                     // activation loads per lane and pair
    extern __shared__ uint4 lds[];
    float *red = reinterpret_cast<float *>(lds); // [WAVES][MB][256], over the slabs once the main loop is through

    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int n_l = lane % 16, q = lane / 16;
    const int col = blockIdx.x * 16 + n_l;
    const int colc = col < N ? col : N - 1;
    const int upr = K / 64, npairs = (upr + 1) / 2;
    const int ppw = (npairs + WAVES - 1) / WAVES;
    const int p_begin = wave * ppw, p_end = p_begin + ppw < npairs ? p_begin + ppw : npairs;
    const uint32_t *wrow = w_codes + (int64_t)colc * (K / 8);
    const uint32_t *mrow = w_meta + (int64_t)colc * upr;
    uint4 *slab = lds + wave * SLAB; // one slab per wave: a pair is written and read back before the next one is written

    struct InFlight {
        uint4 wc;
        uint32_t m;
        uint4 a[NLD];
    };
    // loads of pair p; anything past the end of K (a short last pair, a pair past the range) is zero
    auto issue = [&](InFlight &f, int p) {
        const int u = 2 * p + (q >> 1);
        const bool wvalid = p < p_end && u < upr;
        const int uc = u < upr ? u : upr - 1;
        f.wc = make_uint4(0, 0, 0, 0);
        f.m = 0;
        if (wvalid) {
            f.wc = *reinterpret_cast<const uint4 *>(wrow + uc * 8 + (q & 1) * 4);
            f.m = mrow[uc];
        }
        const int ua = 2 * p + (n_l >> 3); // unit of this lane's 16-byte piece of an activation row
#pragma unroll
        for (int r = 0; r < NLD; ++r) {
            const int row = 4 * r + q;
            f.a[r] = make_uint4(0, 0, 0, 0);
            if (p < p_end && ua < upr && row < M)
                f.a[r] = *reinterpret_cast<const uint4 *>(a + (int64_t)row * lda + (int64_t)p * 128 + n_l * 8);
        }
    };

    f32x4_t acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x4_t{ 0.f, 0.f, 0.f, 0.f };

    InFlight fl[NBUF];
#pragma unroll
    for (int i = 0; i < NBUF; ++i) issue(fl[i], p_begin + i);

    for (int p = p_begin; p < p_end; p += NBUF) {
#pragma unroll
        for (int i = 0; i < NBUF; ++i) {
            if (p + i < p_end) { // wave-uniform
                uint4 *sl = slab;
                // lane (piece n_l, row 4r + q) -> cell [n_l][row]
#pragma unroll
                for (int r = 0; r < NLD; ++r) sl[n_l * RSTRIDE + 4 * r + q] = A_CELL ? fl[i].a[r] : permute_bf16_cell(fl[i].a[r]);
                const uint4 wc = fl[i].wc;
                const uint32_t m = fl[i].m;
                issue(fl[i], p + i + NBUF);
                __builtin_amdgcn_wave_barrier(); // the reads below see the whole wave's writes (LDS is in order)
                const uint32_t sbase = unit_scale_bits(m);
                const uint32_t cwa[4] = { wc.x, wc.y, wc.z, wc.w };
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const bf16x8_t bfrag = __builtin_bit_cast(bf16x8_t, expand_chunk(cwa[t], m, sbase, 4 * (q & 1) + t));
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const uint4 av = sl[(4 * q + t) * RSTRIDE + mb * 16 + n_l];
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av), bfrag, acc[mb], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
    __syncthreads(); // every wave is through with its slab: the partial tiles go on top of them
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[(wave * MB + mb) * 256 + r * 64 + lane] = acc[mb][r];
    __syncthreads();
    // thread -> (mb, r, lane): output row mb*16 + 4*(lane/16) + r, column lane%16
    for (int idx = tid; idx < MB * 256; idx += 64 * WAVES) {
        const int mb = idx / 256, rem = idx % 256, r = rem / 64, ln = rem % 64;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += red[(w * MB + mb) * 256 + rem];
        const int row = mb * 16 + 4 * (ln / 16) + r, cc = blockIdx.x * 16 + (ln % 16);
        if (row < M && cc < N) {
            if (OUT_F32) static_cast<float *>(c)[(int64_t)row * ldc + cc] = v;
            else static_cast<uint16_t *>(c)[(int64_t)row * ldc + cc] = (uint16_t)((f2u(v) + 0x7FFFu + ((f2u(v) >> 16) & 1u)) >> 16);
        }
    }
}

template <int MB, bool A_CELL = false>
static int launch_skinny(const void *a, int64_t lda, const uint8_t *w_codes, const uint32_t *w_meta, int64_t M, int64_t N,
                         int64_t K, void *c, int64_t ldc, int out_dtype, hipStream_t stream)
{
    constexpr int WAVES = skinny_waves(MB);
    constexpr size_t slab_bytes = (size_t)WAVES * 16 * (16 * MB + 1) * sizeof(uint4), red_bytes = (size_t)WAVES * MB * 256 * sizeof(float);
    constexpr size_t lds_bytes = slab_bytes > red_bytes ? slab_bytes : red_bytes;
    static_assert(lds_bytes <= 160 * 1024, "fits the LDS of one CU");
    const dim3 grid((unsigned)((N + 15) / 16)), block(64 * WAVES);
    const uint16_t *ap = static_cast<const uint16_t *>(a);
    const uint32_t *wc = reinterpret_cast<const uint32_t *>(w_codes);
    hipError_t e;
    if (out_dtype == HIF4_OUT_F32) {
        auto k = gemm_skinny_kernel<MB, WAVES, true, A_CELL>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, ap, lda, wc, w_meta, c, ldc, (int)M, (int)N, (int)K);
    } else {
        auto k = gemm_skinny_kernel<MB, WAVES, false, A_CELL>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, ap, lda, wc, w_meta, c, ldc, (int)M, (int)N, (int)K);
    }
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
int launch_encode_to_cells(const void *x, int64_t rows, int64_t K, int64_t ldx, void *cells, int mode, hipStream_t stream);
int launch_encode_to_rows(const void *x, int64_t rows, int64_t K, int64_t ldx, void *y, int mode, hipStream_t stream);
int launch_decode(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, int64_t ldy, hipStream_t stream);
bool fewrows_fits(int64_t M, int64_t N, int64_t K, int64_t lda);
int launch_gemm_fewrows(const void *a, int64_t lda, const uint8_t *w_codes, const uint32_t *w_meta, int64_t M, int64_t N, int64_t K,
                        void *c, int64_t ldc, int out_dtype, hipStream_t stream);
#ifndef HIF4_FEWROWS
#define HIF4_FEWROWS 1
#endif
int launch_encode_to_planes(const void *x, int64_t rows, int64_t K, int64_t ldx, void *planes, int mode, hipStream_t stream);
int launch_decode_cells(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, hipStream_t stream);
int launch_decode_planes(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *planes, hipStream_t stream);
int launch_bf16_to_planes(const void *x, int64_t rows, int64_t K, int64_t ldx, void *planes, hipStream_t stream);
int launch_gemm_stream(const void *a, int64_t lda, const uint8_t *w_codes, const uint32_t *w_meta, int64_t M, int64_t N, int64_t K,
                       void *c, int64_t ldc, int out_dtype, hipStream_t stream);
#ifndef HIF4_STREAM_MIN_COLUMNS
#define HIF4_STREAM_MIN_COLUMNS 12288
#endif
constexpr int64_t STREAM_MIN_COLUMNS = HIF4_STREAM_MIN_COLUMNS;
int launch_gemm_planes(const void *a_planes, const void *w_planes, int64_t M, int64_t N, int64_t K, void *c, uint32_t *c_meta,
                       int64_t ldc, int out_dtype, hipStream_t stream);

bool colwave_fits(int64_t M, int64_t N, int64_t K);
int launch_gemm_colwave(const void *a_planes, const uint8_t *w_codes, const uint32_t *w_meta, const int32_t *offs, int E,
                        int64_t M, int64_t N, int64_t K, void *c, uint32_t *c_meta, int64_t ldc, int out_dtype, int rows_per_tile,
                        hipStream_t stream);

// Internal output kinds beyond HIF4_OUT_BF16 / HIF4_OUT_F32: the result as HiF4 (c = codes plane, c_meta).
enum { OUT_HIF4_RNE = 16, OUT_HIF4_RHA = 17 };

template <int BM, int BN, int WM, int WN, bool A_CELL, bool GROUPED>
static int launch_tiles(GemmArgs g, int out_dtype, int m_tiles, hipStream_t stream)
{
    g.tiles_m = m_tiles;
    constexpr size_t loop_bytes = 2 * (8 * (BM + BN) + 8) * sizeof(uint4);
    constexpr size_t lds_bytes = loop_bytes;
    // grouped: whole rounds of 8 m-tiles; dense: the tiles themselves, split evenly over the 8 XCDs (see the kernel)
    const int64_t padded = GROUPED ? (int64_t)((m_tiles + 7) / 8) * 8 * g.tiles_n : dense_tile_blocks(m_tiles, g.tiles_n);
    if (padded > 0x7FFFFFFF) return HIF4_ERR_SHAPE;
    const dim3 grid((unsigned)((padded + 7) / 8 * 8)), block(64 * WM * WN);
    hipError_t e;
    {
        if (out_dtype == OUT_HIF4_RNE || out_dtype == OUT_HIF4_RHA) { // result written as HiF4
            constexpr size_t emit_bytes = emit_lds_bytes<BM, BN>() > loop_bytes ? emit_lds_bytes<BM, BN>() : loop_bytes;
            static_assert(emit_bytes <= 160 * 1024, "fits the LDS of one CU");
            auto k = out_dtype == OUT_HIF4_RNE ? gemm_kernel<BM, BN, WM, WN, A_CELL, false, GROUPED, HIF4_ROUND_RNE>
                                               : gemm_kernel<BM, BN, WM, WN, A_CELL, false, GROUPED, HIF4_ROUND_RHA>;
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)emit_bytes);
            if (e != hipSuccess) return HIF4_ERR_DEVICE;
            hipLaunchKernelGGL(k, grid, block, emit_bytes, stream, g);
            return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
        }
    }
    if (out_dtype == HIF4_OUT_F32) {
        auto k = gemm_kernel<BM, BN, WM, WN, A_CELL, true, GROUPED>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, g);
    } else {
        auto k = gemm_kernel<BM, BN, WM, WN, A_CELL, false, GROUPED>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, g);
    }
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// Workspace layout.  Both HiF4 kinds of A: the exact BF16 values of the HiF4 activations (2 bytes per
// element; when the call quantises A itself the packed planes never reach memory).  Every part starts
// on a 16-byte boundary.
static inline size_t align16(size_t n) { return (n + 15) & ~(size_t)15; }

size_t gemm_workspace_bytes(int a_kind, int64_t M, int64_t K)
{
    if (M <= 0 || K <= 0) return 0;
    if (a_kind == HIF4_A_HIF4 || a_kind == HIF4_A_BF16_QUANTIZE) return (size_t)M * (size_t)K * 2;
    return 0;
}

// From this many rows of A on, a dense GEMM between two HiF4 operands decodes W once into the
// workspace as well (if the caller gave room for it) and runs the kernel of hif4_gemm_cells.hip
// instead of expanding W inside the main loop.  Measured on MI355X: that main loop (on
// v_mfma_f32_16x16x32_bf16, nothing but matrix work) is 10 to 17 % faster than the one that expands W,
// and the pre-pass that decodes W costs 2.56 bytes per weight once per call, which that margin covers
// from about 3300 rows on whatever the shape (+8 to 12 % from 3328 to 4096 rows on five weight shapes, runs of the
// two paths interleaved), and from 1536 rows on when the decoded W stays within the 256 MB memory-side cache (at
// most 128 Mi weights: +2 to 10 % there; a 28672 x 8192 matrix loses 3 to 5 % below 3328 rows).
#ifndef HIF4_DECODED_W_MIN_ROWS
#define HIF4_DECODED_W_MIN_ROWS 3328
#endif
constexpr int64_t DECODED_W_MIN_ROWS = HIF4_DECODED_W_MIN_ROWS;

// A dense call between HiF4 operands with at most this many rows is one m-tile of that kernel.
#ifndef HIF4_COLWAVE_MAX_ROWS
#define HIF4_COLWAVE_MAX_ROWS 192
#endif
constexpr int64_t COLWAVE_MAX_ROWS = HIF4_COLWAVE_MAX_ROWS;
// Up to 64 rows, two kernels can take a dense call whatever the kind of A (each after a pre-pass that puts A
// into its form): the one that splits K over the waves of 16-column workgroups (gemm_skinny_kernel) and the
// one that expands W into MFMA operands per 32-column strip (hif4_gemm_colwave.hip).  Measured from HIP graphs
// (us, pre-pass included, first kernel : second): 16 x 4096 x 4096 9 : 19, 64 x 4096 x 4096 15 : 19,
// 32 x 11008 x 4096 21 : 22, 64 x 11008 x 4096 34 : 25, 16 x 28672 x 8192 51 : 65, 32 x 28672 x 8192 72 : 67,
// 64 x 28672 x 8192 101 : 74 - the first wins on few rows or few weights.
static bool few_rows_prefer_k_split(int64_t M, int64_t N, int64_t K)
{
    const int64_t weights = N * K;
    return M <= 16 || (M <= 32 && weights <= ((int64_t)48 << 20)) || (M <= 64 && weights <= ((int64_t)24 << 20));
}

// Up to 32 rows against at least 6144 columns: the kernel of hif4_gemm_fewrows.hip.  Measured from HIP graphs over
// distinct weight matrices (us, that kernel : gemm_skinny_kernel), 16 rows: 6144 x 4096 10.8 : 11.2, 8192 x 4096 11.1 : 11.5,
// 11008 x 4096 13.0 : 15.2, 14336 x 4096 15.0 : 19.8, 8192 x 8192 18.0 : 20.6, 28672 x 8192 41.9 : 62.6, 8192 x 28672
// 48.5 : 66.4; 32 rows: 6144 x 4096 14.4 : 14.4, 11008 x 4096 16.9 : 19.7, 8192 x 8192 25.4 : 31.5, 28672 x 8192 51.2 : 74.6,
// 8192 x 28672 79.7 : 88.0; one row: 11008 x 4096 11.1 : 12.4, 28672 x 8192 40.9 : 46.8.  The other way round on fewer
// columns, where its 16-column strips do not fill the chip with waves (16 rows: 4096 x 4096 8.8 : 7.2, 2048 x 7168
// 12.3 : 10.3, 4096 x 11008 17.5 : 15.4; 32 rows: 14.2 : 8.4, 20.9 : 13.5, 32.1 : 20.5; 8 rows and fewer: within 5 %).
#ifndef HIF4_FEWROWS_MIN_COLUMNS
#define HIF4_FEWROWS_MIN_COLUMNS 6144
#endif
static bool fewrows_pays(int64_t M, int64_t N, int64_t K)
{
    (void)K;
    return M <= 32 && N >= HIF4_FEWROWS_MIN_COLUMNS;
}

// Rows of A per workgroup of that kernel for a dense call, 0: not its case.  Up to 192 rows: one tile.
// Beyond, every m-tile expands W again, which pays only while the whole call is small: at most
// HIF4_COLWAVE_DENSE_STRIPS (32-column strip, 128-row tile) pairs, i.e. one round of two waves per SIMD
// (measured against the tile kernel at 256 to 1024 rows and 2048 to 28672 columns).  Tiles of 128 rows
// while those pairs leave SIMDs idle, else the tile height (128, 192, 256) that covers M with the
// least padding, the fewest tiles among equals.
#ifndef HIF4_COLWAVE_DENSE_STRIPS
#define HIF4_COLWAVE_DENSE_STRIPS 2048
#endif
static int colwave_dense_rows(int64_t M, int64_t N)
{
    if (M <= COLWAVE_MAX_ROWS) return (int)M;
    const int64_t s128 = (N + 31) / 32 * ((M + 127) / 128);
    if (s128 > HIF4_COLWAVE_DENSE_STRIPS || M > 2048) return 0;
#ifdef HIF4_COLWAVE_DENSE_TILE
    return HIF4_COLWAVE_DENSE_TILE;
#endif
    if (s128 <= 1024) return 128;
    int best = 128;
    int64_t best_pad = (M + 127) / 128 * 128 - M, best_tiles = (M + 127) / 128;
    for (int rows = 192; rows <= 256; rows += 64) {
        const int64_t tiles = (M + rows - 1) / rows, pad = tiles * rows - M;
        if (pad < best_pad || (pad == best_pad && tiles < best_tiles)) best = rows, best_pad = pad, best_tiles = tiles;
    }
    return best;
}

// Whether a dense call should decode W once, given the room: see DECODED_W_MIN_ROWS; never on the shapes of the
// few-row kernel, which is faster than both.
static bool decoded_w_pays(int64_t M, int64_t N, int64_t K)
{
    if (M >= DECODED_W_MIN_ROWS) return true;
    return M >= 1536 && N * K <= ((int64_t)128 << 20) && colwave_dense_rows(M, N) == 0;
}

size_t gemm_workspace_bytes_decoded_w(int a_kind, int64_t M, int64_t N, int64_t K)
{
    const size_t base = gemm_workspace_bytes(a_kind, M, K);
    // weight-only with more than 64 rows in the range of the kernel of hif4_gemm_colwave.hip: room for a reordered
    // copy of A selects it
    if (a_kind == HIF4_A_BF16_KEEP && N > 0 && K > 0 && (M > 64 ? colwave_dense_rows(M, N) > 0 : M > 0 && !few_rows_prefer_k_split(M, N, K)))
        return (size_t)M * (size_t)K * 2;
    if (N <= 0 || K <= 0 || !decoded_w_pays(M, N, K)) return base;
    if (a_kind == HIF4_A_BF16_KEEP) return align16((size_t)M * (size_t)K * 2) + (size_t)N * (size_t)K * 2; // A as planes, W decoded
    return align16(base) + (size_t)N * (size_t)K * 2;
}

#ifndef HIF4_COLWAVE_ROWS
#define HIF4_COLWAVE_ROWS -1
#endif
// Rows of A per workgroup for the grouped kernel of hif4_gemm_colwave.hip, from the mean number of
// rows per expert (the counts themselves live on the device): an expert should fit one m-tile, so that
// its weights are expanded once, with room for the spread of a random routing.  0: use the tile kernel.
static int colwave_rows(int64_t M, int E)
{
    if (HIF4_COLWAVE_ROWS >= 0) return HIF4_COLWAVE_ROWS;
    const int64_t want = M / (E > 0 ? E : 1) * 11 / 8 + 8;
    return want <= 64 ? 64 : want <= 128 ? 128 : want <= 192 ? 192 : 256;
}

// Which main loop takes a call: a pure function of the call's shape, kind, output form and workspace, so that the
// choice can be tested (and reported) without a GPU.  grouped: the call has per-expert row ranges (E experts);
// ws_ok: the workspace pointer is there and 16-byte aligned.
int gemm_plan(int a_kind, bool grouped, int E, int64_t M, int64_t N, int64_t K, int64_t lda, bool emit, bool ws_ok, size_t ws_bytes)
{
    if (K == 0) return HIF4_PLAN_ZERO_FILL;
    const bool keep = a_kind == HIF4_A_BF16_KEEP;
    const size_t a_bf16 = (size_t)M * (size_t)K * 2; // A as BF16: the decoded copy of HiF4 activations, or a reordered copy of plain ones
    // a few rows against a wide weight matrix: W streamed once, unit scales applied to the units' partial sums
    if (HIF4_FEWROWS && !grouped && !emit && fewrows_pays(M, N, K) && fewrows_fits(M, N, K, keep ? lda : K)) return HIF4_PLAN_FEWROWS;
    const int cw_rows = grouped ? colwave_rows(M, E) : colwave_dense_rows(M, N);
    const bool colwave_ok = cw_rows > 0 && colwave_fits(M, N, K) && (!keep || (ws_ok && ws_bytes >= a_bf16));
    if (keep && !grouped && M <= 64 && !emit && (few_rows_prefer_k_split(M, N, K) || !colwave_ok)) {
        // decode-shaped: 33 to 64 rows against many columns go to the kernel that splits columns only (measured 96
        // against 122 us for 64 x 28672 x 8192, 38 against 43 us at 14336 x 4096, 36 against 30 us at 11008 x 4096),
        // the rest to the one that splits K over the waves of 16-column workgroups
        return M > 32 && K % 128 == 0 && N >= STREAM_MIN_COLUMNS ? HIF4_PLAN_STREAM : HIF4_PLAN_SKINNY;
    }
    // many rows and room for a decoded copy of W: both operands decoded once, main loop without any expansion
    if (!grouped && decoded_w_pays(M, N, K) && (!keep || ws_ok) && ws_bytes >= align16(a_bf16) + (size_t)N * (size_t)K * 2) return HIF4_PLAN_PLANES;
    // HiF4 activations, few rows against not too many weights: the K-split kernel fed with their exact BF16 values
    if (!keep && !grouped && !emit && M <= 64 && few_rows_prefer_k_split(M, N, K)) return HIF4_PLAN_SKINNY;
    // grouped, or a dense call of few rows (one m-tile, or a few on a small N): every weight meets few rows only, so
    // the kernel that expands W straight into MFMA operands takes the call
    if (colwave_ok) return HIF4_PLAN_COLWAVE;
    return HIF4_PLAN_TILES; // W expanded inside the main loop of the 256 x 256 tile kernel
}

// out_dtype: HIF4_OUT_BF16, HIF4_OUT_F32, or 16 + rounding mode for a HiF4 result (c = codes plane, c_meta = its
// metadata plane, ldc unused).  HiF4 activations enter every main loop as their exact BF16 values (at most 6
// significant bits each), written once per call into the workspace in the form the chosen loop reads; when the call
// quantises them itself, Algorithm 1 and Eq. 2 run in one pass and the packed activations never reach memory.
int launch_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
                const uint32_t *w_meta, const int32_t *offs, int E, int64_t M, int64_t N, int64_t K, void *c,
                uint32_t *c_meta, int64_t ldc, int out_dtype, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    const bool emit = out_dtype == OUT_HIF4_RNE || out_dtype == OUT_HIF4_RHA;
    const bool keep = a_kind == HIF4_A_BF16_KEEP, quantize = a_kind == HIF4_A_BF16_QUANTIZE;
    const bool ws_ok = workspace && (reinterpret_cast<uintptr_t>(workspace) & 15) == 0;
    const uint8_t *a_packed = static_cast<const uint8_t *>(a);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    switch (gemm_plan(a_kind, offs != nullptr, E, M, N, K, lda, emit, ws_ok, workspace_bytes)) {
    case HIF4_PLAN_ZERO_FILL: { // empty sum: C = 0 (a fill kernel, so that the call can be captured in a graph)
        const dim3 grid((unsigned)((N + 255) / 256), (unsigned)(M < 65535 ? M : 65535)), block(256);
        if (emit) { // the all-zero unit: codes 0, metadata 0 (E6M2 at its least code, no micro-exponents)
            hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((N / 4 + 255) / 256), grid.y), block, 0, stream, c, M, N / 4, N / 4, 2);
            hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((N / 64 + 255) / 256), grid.y), block, 0, stream, c_meta, M, N / 64, N / 64, 4);
        } else {
            hipLaunchKernelGGL(zero_kernel, grid, block, 0, stream, c, M, N, ldc, out_dtype == HIF4_OUT_F32 ? 4 : 2);
        }
        return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
    }
    case HIF4_PLAN_FEWROWS: { // A as dense rows in natural element order
        if (keep) return launch_gemm_fewrows(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
        if (int rc = quantize ? launch_encode_to_rows(a, M, K, lda, ws, HIF4_ROUND_RNE, stream) : launch_decode(a_packed, a_meta, M, K, ws, K, stream)) return rc;
        return launch_gemm_fewrows(ws, K, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
    }
    case HIF4_PLAN_STREAM: return launch_gemm_stream(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
    case HIF4_PLAN_SKINNY: {
        if (keep) {
            if (M <= 16) return launch_skinny<1>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
            if (M <= 32) return launch_skinny<2>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
            return launch_skinny<4>(a, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
        }
        // A as dense rows, every group of 8 in cell order
        if (int rc = quantize ? launch_encode_to_cells(a, M, K, lda, ws, HIF4_ROUND_RNE, stream) : launch_decode_cells(a_packed, a_meta, M, K, ws, stream)) return rc;
        if (M <= 16) return launch_skinny<1, true>(ws, K, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
        if (M <= 32) return launch_skinny<2, true>(ws, K, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
        return launch_skinny<4, true>(ws, K, w_codes, w_meta, M, N, K, c, ldc, out_dtype, stream);
    }
    case HIF4_PLAN_PLANES: { // both operands as cell planes: A first, W behind it
        uint8_t *wplanes = ws + align16((size_t)M * (size_t)K * 2);
        if (int rc = keep       ? launch_bf16_to_planes(a, M, K, lda, ws, stream)
                     : quantize ? launch_encode_to_planes(a, M, K, lda, ws, HIF4_ROUND_RNE, stream)
                                : launch_decode_planes(a_packed, a_meta, M, K, ws, stream))
            return rc;
        if (int rc = launch_decode_planes(w_codes, w_meta, N, K, wplanes, stream)) return rc;
        return launch_gemm_planes(ws, wplanes, M, N, K, c, c_meta, ldc, out_dtype, stream);
    }
    case HIF4_PLAN_COLWAVE: { // A as cell planes
        if (int rc = keep       ? launch_bf16_to_planes(a, M, K, lda, ws, stream)
                     : quantize ? launch_encode_to_planes(a, M, K, lda, ws, HIF4_ROUND_RNE, stream)
                                : launch_decode_planes(a_packed, a_meta, M, K, ws, stream))
            return rc;
        return launch_gemm_colwave(ws, w_codes, w_meta, offs, E, M, N, K, c, c_meta, ldc, out_dtype, offs ? colwave_rows(M, E) : colwave_dense_rows(M, N), stream);
    }
    default: break;
    }
    // HIF4_PLAN_TILES: plain BF16 rows of A as they are, HiF4 activations as dense rows in cell order
    GemmArgs g;
    if (keep) {
        g.a = static_cast<const uint16_t *>(a);
        g.lda = lda;
    } else {
        if (int rc = quantize ? launch_encode_to_cells(a, M, K, lda, ws, HIF4_ROUND_RNE, stream) : launch_decode_cells(a_packed, a_meta, M, K, ws, stream)) return rc;
        g.a = reinterpret_cast<const uint16_t *>(ws);
        g.lda = K;
    }
    const bool a_cell = !keep;
    g.w_codes = reinterpret_cast<const uint32_t *>(w_codes);
    g.w_meta = w_meta;
    g.offs = offs;
    g.c = c;
    g.c_meta = c_meta;
    g.ldc = ldc;
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    g.E = E;
    if (offs) {
        // Row counts per expert live on the device; the host only knows their mean.  Every W
        // unit is expanded once per m-tile that uses it, and a K step of a tile costs almost the
        // same whether its rows are all there or not (measured: 2.1 us for 256 x 256, dominated by the
        // expansion of the 256 W rows), so the tile should cover an
        // expert's rows in one go: 256 rows unless experts are small on average.  Splitting the
        // call by row count into a 128-row and a 256-row launch was measured slower on the mixed
        // case (two short launches, each with its own tail).  The grid is the upper bound
        // sum_e ceil(rows_e / BM) <= M / BM + E.
        constexpr int BN = 256;
        g.tiles_n = (int)((N + BN - 1) / BN);
        if (M > (int64_t)E * 96) {
            const int m_tiles = (int)(M / 256) + E;
            if (a_cell) return launch_tiles<256, BN, 2, 4, true, true>(g, out_dtype, m_tiles, stream);
            return launch_tiles<256, BN, 2, 4, false, true>(g, out_dtype, m_tiles, stream);
        }
        // small experts: 128 x 128 tiles on four waves, two workgroups per CU with barriers of their
        // own (measured 13 % faster than 128 x 256 on eight waves at 64 rows per expert)
        g.tiles_n = (int)((N + 127) / 128);
        const int m_tiles = (int)(M / 128) + E;
        if (a_cell) return launch_tiles<128, 128, 2, 2, true, true>(g, out_dtype, m_tiles, stream);
        return launch_tiles<128, 128, 2, 2, false, true>(g, out_dtype, m_tiles, stream);
    }
    constexpr int BM = 256, BN = 256;
    g.tiles_n = (int)((N + BN - 1) / BN);
    const int m_tiles = (int)((M + BM - 1) / BM);
    if (a_cell) return launch_tiles<BM, BN, 2, 4, true, false>(g, out_dtype, m_tiles, stream);
    return launch_tiles<BM, BN, 2, 4, false, false>(g, out_dtype, m_tiles, stream);
}

} // namespace hif4
