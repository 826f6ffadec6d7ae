// Dense HiF4 GEMM for many rows: both operands decoded once per call, then a BF16 MFMA main
// loop fed by direct global -> LDS loads.
//
// Why a second path: inside the tile kernel of hif4_gemm.hip every unit of W is expanded by
// each of the M / 256 tiles of C that use it.  With many thousands of rows that repeated VALU
// work (it lowers the clock the matrix pipeline runs at) costs more than decoding W once (2.56
// bytes of traffic per weight), so here the exact BF16 values of A and of W (Eq. 2 of the HiF4
// paper, Section II-A; at most six significant bits each) are written to the workspace first
// and the main loop is a plain BF16 GEMM whose partial sums are those of Eq. 4 (Section III-B)
// per 64-wide K step, accumulated in fp32.
//
// Layout of a decoded copy ("cell planes"): one 16-byte cell holds the 8 values of one group of
// 8 along K in the order 0,2,1,3,4,6,5,7 (expand_chunk); cell (row, group g) sits at index
// g * rows + row.  So the 64 cells a wave moves with one global_load_lds_dwordx4 (rows r..r+63
// of one group) are contiguous in memory and land contiguously in LDS, where a K step of a
// tile is stored [group j of 8][row] as in the other tile kernel.  No VGPR carries staged data,
// no ds_write is issued, and the staging needs no VALU work at all.
#include "hif4_emit.h"
#include "hif4_expand.h"
#include "hif4_store.h"

namespace hif4 {

// 64 lanes x 16 bytes from global memory straight into 1 KB of LDS starting at byte offset
// `lds_byte` (the same for the whole wave): global_load_lds_dwordx4, lane l landing at
// lds_byte + 16 l.  Completion is counted by vmcnt.  Written as inline assembly so that the
// compiler's wait-count insertion does not see an LDS-writing load: with one pending it would
// turn every wait for an LDS read into a wait for all of them, and the operand prefetch of the
// main loop would be lost.  The caller waits for vmcnt(0) itself before the data is read.
// M0 (the LDS base of such a load) is used by nothing else in these kernels; the s_nop is the
// wait state the hardware needs between a write of M0 and an LDS-writing load.
__device__ __forceinline__ void load_to_lds_16(const uint4 *src, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_byte), "v"(src) : "memory");
}

// byte offset of a __shared__ object inside the workgroup's LDS
__device__ __forceinline__ uint32_t lds_offset(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

// ------------------------------------------------------------------ decode to cell planes

// Block = 64 rows x 2 units.  Thread (row = tid % 64, hu = tid / 64) expands half a unit (one
// 16-byte load of codes) to 4 cells; a wave's stores are 64 consecutive cells of one group.
// The 4-byte-per-lane reads of a wave touch 64 different lines, but the 8 loads that share a
// line come from the same block, so they are served by the L1.
// (Streaming stores for the planes were measured: no difference for the whole call, interleaved A/B on five shapes;
// streaming stores for C in the main loop's epilogue cost 3 to 20 %.)
__global__ __launch_bounds__(256) void decode_planes_kernel(const uint32_t *__restrict__ codes,
                                                            const uint32_t *__restrict__ meta, int64_t rows,
                                                            int64_t upr, uint4 *__restrict__ planes)
{
    // one grid axis (row blocks fastest): K is not bounded by the 65535 blocks of a second axis
    const int64_t row_blocks = (rows + 63) / 64;
    const int64_t row = (int64_t)(blockIdx.x % row_blocks) * 64 + threadIdx.x % 64;
    const int hu = threadIdx.x / 64;
    const int64_t unit = (int64_t)(blockIdx.x / row_blocks) * 2 + (hu >> 1);
    if (row >= rows || unit >= upr) return;
    const int hh = hu & 1;
    const uint4 c = *reinterpret_cast<const uint4 *>(codes + (row * upr + unit) * 8 + 4 * hh);
    const uint32_t m = meta[row * upr + unit];
    const uint32_t sbase = unit_scale_bits(m);
    const uint32_t cw[4] = { c.x, c.y, c.z, c.w };
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int j = 4 * hh + t;
        planes[(unit * 8 + j) * rows + row] = expand_chunk(cw[t], m, sbase, j);
    }
}

// Plain BF16 rows (the activations of a weight-only call) -> the same cell planes.  Block = 64 rows x
// 8 groups of 8 (one 128-byte line of every row); thread (row, group) permutes one cell.
__global__ __launch_bounds__(512) void bf16_to_planes_kernel(const uint16_t *__restrict__ x, int64_t rows, int64_t ldx,
                                                             uint4 *__restrict__ planes)
{
    const int64_t row_blocks = (rows + 63) / 64; // one grid axis, row blocks fastest
    const int64_t row = (int64_t)(blockIdx.x % row_blocks) * 64 + threadIdx.x % 64;
    const int64_t g = (int64_t)(blockIdx.x / row_blocks) * 8 + threadIdx.x / 64;
    if (row >= rows) return;
    planes[g * rows + row] = permute_bf16_cell(*reinterpret_cast<const uint4 *>(x + row * ldx + g * 8));
}

int launch_bf16_to_planes(const void *x, int64_t rows, int64_t K, int64_t ldx, void *planes, hipStream_t stream)
{
    if (rows == 0 || K == 0) return HIF4_OK;
    const int64_t blocks = (rows + 63) / 64 * (K / 64);
    if (blocks > 0x7FFFFFFF) return HIF4_ERR_SHAPE;
    const dim3 grid((unsigned)blocks), block(512);
    hipLaunchKernelGGL(bf16_to_planes_kernel, grid, block, 0, stream, static_cast<const uint16_t *>(x), rows, ldx,
                       static_cast<uint4 *>(planes));
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_decode_planes(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *planes,
                         hipStream_t stream)
{
    const int64_t upr = K / 64;
    if (rows == 0 || upr == 0) return HIF4_OK;
    const int64_t blocks = (rows + 63) / 64 * ((upr + 1) / 2);
    if (blocks > 0x7FFFFFFF) return HIF4_ERR_SHAPE;
    const dim3 grid((unsigned)blocks), block(256);
    hipLaunchKernelGGL(decode_planes_kernel, grid, block, 0, stream, reinterpret_cast<const uint32_t *>(codes), meta, rows,
                       upr, static_cast<uint4 *>(planes));
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// ------------------------------------------------------------------ GEMM on cell planes

struct PlaneGemmArgs {
    const uint4 *a; // cell planes of A: [K/8][M]  (MXFP4: [K/32][M])
    const uint4 *w; // cell planes of W: [K/8][N]  (MXFP4: [K/32][N])
    const uint32_t *a_scale, *w_scale; // MXFP4 only: scale planes, see mxfp4_pack_kernel
    void *c;
    uint32_t *c_meta; // EMIT kernels: c is the codes plane of the HiF4 result, this its metadata plane
    int64_t ldc;
    int M, N, K;
    int tiles_m, tiles_n; // tiles of this launch
    int col_base;         // its first column of W / of C (a launch may cover a range of columns only, see launch_planes)
};

// MX = false: BF16 cells, a K step is 64 wide and a quarter is one v_mfma_f32_32x32x16_bf16.
// MX = true (speed reference, not a HiF4 path): MXFP4 cells of 32 E2M1 values with one E8M0
// scale each, a K step is 256 wide and a quarter is one v_mfma_scale_f32_32x32x64_f8f6f4, which
// takes a lane's 32 values and their scale as they are.  Everything else is shared.
// EMIT >= 0: the result is written as HiF4 with units along N (rounding mode EMIT), see hif4_emit.h.
template <int BM, int BN, int WM, int WN, bool OUT_F32, bool MX = false, int EMIT = -1>
__global__ __launch_bounds__(64 * WM * WN) void gemm_planes_kernel(PlaneGemmArgs g)
{
    constexpr int KSTEP = MX ? 256 : 64;
    constexpr int NW = WM * WN;                          // waves
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;  // MFMA tiles per wave
    constexpr int NMF = TM * TN;                         // MFMAs per quarter step
    constexpr int W_BASE = 8 * BM, CELLS = 8 * (BM + BN); // 16-byte cells per buffer: [j][row] of A, then of W
    constexpr int IA = 8 * BM / 64 / NW, IW = 8 * BN / 64 / NW; // 64-cell loads per wave and K step
    static_assert(BM % 64 == 0 && BN % 64 == 0 && (8 * BM / 64) % NW == 0 && (8 * BN / 64) % NW == 0, "whole loads per wave");
    extern __shared__ uint4 lds[]; // 2 buffers x CELLS

    const int tid = threadIdx.x;
    const int wave = tid / 64, lane = tid % 64;
    const int wm = wave / WN, wn = wave % WN;

    int tile_m, tile_n; // see dense_tile_of_block
    if (!dense_tile_of_block(g.tiles_m, g.tiles_n, tile_m, tile_n)) return;
    const int row0 = tile_m * BM, col0 = g.col_base + tile_n * BN;
    const int nk = g.K / KSTEP;

    // ---- staging plan of this wave: load i moves cells (group j, rows rb*64 .. rb*64+63); rows
    // past the edge of the matrix repeat its last row (never stored).
    const uint4 *a_src[IA], *w_src[IW];
    int a_dst[IA], w_dst[IW];
#pragma unroll
    for (int i = 0; i < IA; ++i) {
        const int id = wave * IA + i, j = id / (BM / 64), rb = id % (BM / 64);
        int row = row0 + rb * 64 + lane;
        row = row < g.M ? row : g.M - 1;
        a_src[i] = g.a + (int64_t)j * g.M + row;
        a_dst[i] = j * BM + rb * 64;
    }
#pragma unroll
    for (int i = 0; i < IW; ++i) {
        const int id = wave * IW + i, j = id / (BN / 64), rb = id % (BN / 64);
        int row = col0 + rb * 64 + lane;
        row = row < g.N ? row : g.N - 1;
        w_src[i] = g.w + (int64_t)j * g.N + row;
        w_dst[i] = W_BASE + j * BN + rb * 64;
    }
    const int64_t a_step = (int64_t)8 * g.M, w_step = (int64_t)8 * g.N; // cells per K step
    // enqueue the loads of one K step into `buf` and advance to the next step
    auto stage = [&](uint4 *buf) {
        const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_offset(buf));
#pragma unroll
        for (int i = 0; i < IA; ++i) {
            load_to_lds_16(a_src[i], base + (uint32_t)__builtin_amdgcn_readfirstlane(a_dst[i] * 16));
            a_src[i] += a_step;
        }
#pragma unroll
        for (int i = 0; i < IW; ++i) {
            load_to_lds_16(w_src[i], base + (uint32_t)__builtin_amdgcn_readfirstlane(w_dst[i] * 16));
            w_src[i] += w_step;
        }
    };
    // all of this thread's direct loads have landed in LDS
    auto staged_wait = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int half = lane / 32, l32 = lane % 32;
    // MFMA operands of two quarters (K-slabs of 16, or of 64 for MXFP4).  Quarter s takes cell 2s
    // from lanes 0..31 and cell 2s+1 from lanes 32..63.  The set that the first phase works on
    // starts as zeros.
    uint4 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[1][i] = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < TN; ++i) bfr[1][i] = make_uint4(0, 0, 0, 0);
    // MXFP4 scales: one dword per lane, tile and K step, byte s for quarter s (straight from
    // global memory, one step ahead); `prev` serves the quarter that is worked off after the barrier.
    struct Scales {
        uint32_t a[TM], b[TN];
    };
    Scales sc_prev, sc_cur, sc_next;
#pragma unroll
    for (int i = 0; i < TM; ++i) sc_prev.a[i] = sc_cur.a[i] = sc_next.a[i] = 0x7F7F7F7Fu; // 2^0
#pragma unroll
    for (int i = 0; i < TN; ++i) sc_prev.b[i] = sc_cur.b[i] = sc_next.b[i] = 0x7F7F7F7Fu;
    auto load_scales = [&](Scales &sc, int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int row = row0 + wm * (BM / WM) + i * 32 + l32;
            row = row < g.M ? row : g.M - 1;
            sc.a[i] = g.a_scale[((int64_t)ks * 2 + half) * g.M + row];
        }
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            int row = col0 + wn * (BN / WN) + i * 32 + l32;
            row = row < g.N ? row : g.N - 1;
            sc.b[i] = g.w_scale[((int64_t)ks * 2 + half) * g.N + row];
        }
    };
    // MFMA number tm of quarter q (of the step whose scales are sc) on operand set fb
    auto mfma = [&](int fb, int tm, [[maybe_unused]] int q, [[maybe_unused]] const Scales &sc) {
        f32x16_t &d = acc[tm / TN][tm % TN];
        const uint4 a = af[fb][tm / TN], b = bfr[fb][tm % TN];
        if constexpr (MX) {
#if defined(__HIP_DEVICE_COMPILE__)
            typedef int v8i __attribute__((ext_vector_type(8)));
            const v8i A = { (int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0 }, B = { (int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0 };
            const int sa = (int)sc.a[tm / TN], sb = (int)sc.b[tm % TN];
            // cbsz = blgp = 4: both operands FP4 (E2M1); the op_sel arguments pick the scale byte
            if (q == 0) d = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, d, 4, 4, 0, sa, 0, sb);
            else if (q == 1) d = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, d, 4, 4, 1, sa, 1, sb);
            else if (q == 2) d = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, d, 4, 4, 2, sa, 2, sb);
            else d = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, d, 4, 4, 3, sa, 3, sb);
#endif
        } else {
            d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), d, 0, 0, 0);
        }
    };
    // One K step on `cur`: phase p requests the operands of quarter p and runs the MFMAs of
    // quarter p-1 (for p = 0: the last quarter of the previous step, still in registers), so
    // the barrier between two steps falls between a quarter's operand reads and its MFMAs.
    auto k_step = [&](const uint4 *cur) {
        const uint4 *abase = cur + wm * (BM / WM) + l32;
        const uint4 *bbase = cur + W_BASE + wn * (BN / WN) + l32;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int j = 2 * s + half;
#pragma unroll
            for (int i = 0; i < TM; ++i) af[s & 1][i] = abase[j * BM + i * 32];
#pragma unroll
            for (int i = 0; i < TN; ++i) bfr[s & 1][i] = bbase[j * BN + i * 32];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int tm = 0; tm < NMF; ++tm) mfma((s + 1) & 1, tm, (s + 3) & 3, s == 0 ? sc_prev : sc_cur);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One loop body for both buffers (no branch around the matrix work), so that the
    // accumulators are plain loop-carried registers.
    int cur = 0, nxt = CELLS;
    stage(lds);
    if (MX) load_scales(sc_cur, 0);
    staged_wait();
    __syncthreads();
    for (int ks = 0; ks < nk; ++ks) {
        if (ks + 1 < nk) {
            stage(lds + nxt); // every wave is past its reads of that buffer (the barrier above)
            if (MX) load_scales(sc_next, ks + 1);
        }
        k_step(lds + cur);
        staged_wait();
        __syncthreads();
        const int t2 = cur;
        cur = nxt;
        nxt = t2;
        if (MX) {
            sc_prev = sc_cur;
            sc_cur = sc_next;
        }
    }
#pragma unroll
    for (int tm = 0; tm < NMF; ++tm) mfma(1, tm, 3, sc_prev); // quarter 3 of the last step

    if constexpr (EMIT >= 0) {
        emit_hif4_tile<BM, BN, WM, WN, EMIT>(acc, lds, row0, g.M, col0, g.N, static_cast<uint32_t *>(g.c), g.c_meta);
        return;
    }

    // ---- epilogue: lane holds column l32 of each 32x32 tile, rows 8*(r/4) + 4*half + r%4
    store_acc_32x32<OUT_F32>(acc, g.c, g.ldc, row0 + wm * (BM / WM), col0 + wn * (BN / WN), g.M, g.N);
}


// The same GEMM on v_mfma_f32_16x16x32_bf16.  On this chip the matrix pipeline is limited by
// power under real operand bits, and the 16 x 16 x 32 form sustains more than the 32 x 32 x 16
// form (measured with MFMA-only loops on random bits: 2.0 against 1.7-1.8 PFLOP/s): twice the K
// per instruction means half the accumulator traffic per flop.  Same tile, staging and block
// mapping as above; a wave's 128 x 64 part is 8 x 4 tiles of 16 x 16.  Lane (n, q) = (lane % 16,
// lane / 16) takes row n and cell 4 hs + q of a K step's 8 cells for half step hs (32 of K).
// A half step is two phases of 16 MFMAs (tile rows 0..3, then 4..7); phase P requests its
// operands from LDS and runs the MFMAs of phase P - 1, so the barrier between two K steps again
// falls between the last phase's operand reads and its MFMAs.
template <int BM, int BN, int WM, int WN, bool OUT_F32, int EMIT = -1>
__global__ __launch_bounds__(64 * WM * WN) void gemm_planes16_kernel(PlaneGemmArgs g)
{
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM / 16, TN = BN / WN / 16; // 16 x 16 tiles per wave
    static_assert(TM == 8 && TN >= 2 && TN <= 4, "two phases of four tile rows per half step; 32 to 64 columns per wave");
    constexpr int W_BASE = 8 * BM, CELLS = 8 * (BM + BN);
    constexpr int IA = 8 * BM / 64 / NW, IW = 8 * BN / 64 / NW;
    extern __shared__ uint4 lds[]; // 2 buffers x CELLS

    const int tid = threadIdx.x;
    const int wave = tid / 64, lane = tid % 64;
    const int wm = wave / WN, wn = wave % WN;

    // The workgroups stay: a compute unit runs one of them at a time, and a new one per tile would spend about 12 us
    // outside its K loop (start of the waves, first loads from memory, draining of its stores) for 64 to 128 K steps of
    // 1.4 us.  So a workgroup takes tile after tile (persistent_tile), and the first K step of its next tile is on its
    // way into LDS while it stores the results of this one.
    const int nk = g.K / 64;
    int tile_m, tile_n;
    if (!persistent_tile(0, g.tiles_m, g.tiles_n, tile_m, tile_n)) return;

    const uint4 *a_src[IA], *w_src[IW];
    int a_dst[IA], w_dst[IW];
#pragma unroll
    for (int i = 0; i < IA; ++i) a_dst[i] = (wave * IA + i) / (BM / 64) * BM + (wave * IA + i) % (BM / 64) * 64;
#pragma unroll
    for (int i = 0; i < IW; ++i) w_dst[i] = W_BASE + (wave * IW + i) / (BN / 64) * BN + (wave * IW + i) % (BN / 64) * 64;
    // where the loads of the first K step of the tile at (row0, col0) start; rows past the edge of a matrix repeat its last row
    auto aim = [&](int row0, int col0) {
#pragma unroll
        for (int i = 0; i < IA; ++i) {
            const int id = wave * IA + i, j = id / (BM / 64), rb = id % (BM / 64);
            int row = row0 + rb * 64 + lane;
            row = row < g.M ? row : g.M - 1;
            a_src[i] = g.a + (int64_t)j * g.M + row;
        }
#pragma unroll
        for (int i = 0; i < IW; ++i) {
            const int id = wave * IW + i, j = id / (BN / 64), rb = id % (BN / 64);
            int row = col0 + rb * 64 + lane;
            row = row < g.N ? row : g.N - 1;
            w_src[i] = g.w + (int64_t)j * g.N + row;
        }
    };
    const int64_t a_step = (int64_t)8 * g.M, w_step = (int64_t)8 * g.N;
    auto stage = [&](uint4 *buf) {
        const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_offset(buf));
#pragma unroll
        for (int i = 0; i < IA; ++i) {
            load_to_lds_16(a_src[i], base + (uint32_t)__builtin_amdgcn_readfirstlane(a_dst[i] * 16));
            a_src[i] += a_step;
        }
#pragma unroll
        for (int i = 0; i < IW; ++i) {
            load_to_lds_16(w_src[i], base + (uint32_t)__builtin_amdgcn_readfirstlane(w_dst[i] * 16));
            w_src[i] += w_step;
        }
    };
    auto staged_wait = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    f32x4_t acc[TM][TN];
    const int q = lane / 16, n = lane % 16;
    // operands of two phases (4 tile rows of A each) and of two half steps (4 tile columns of W each)
    uint4 af[2][4], bfr[2][TN];
    auto mfma_phase = [&](int ph) { // the 4 TN MFMAs of phase ph = 2 hs + ab: tile rows 4 ab .. 4 ab + 3, operands of half step hs
        const int hs = ph / 2, ab = ph % 2;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[4 * ab + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, af[ph & 1][i]), __builtin_bit_cast(bf16x8_t, bfr[hs & 1][j]),
                                                                             acc[4 * ab + i][j], 0, 0, 0);
    };
    auto k_step = [&](const uint4 *cur) {
        const uint4 *abase = cur + wm * (BM / WM) + n;
        const uint4 *bbase = cur + W_BASE + wn * (BN / WN) + n;
#pragma unroll
        for (int ph = 0; ph < 4; ++ph) {
            const int hs = ph / 2, ab = ph % 2, j = 4 * hs + q;
#pragma unroll
            for (int i = 0; i < 4; ++i) af[ph & 1][i] = abase[j * BM + (4 * ab + i) * 16];
            if (ab == 0) {
#pragma unroll
                for (int i = 0; i < TN; ++i) bfr[hs & 1][i] = bbase[j * BN + i * 16];
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_phase((ph + 3) & 3);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    int cur = 0, nxt = CELLS;
    aim(tile_m * BM, g.col_base + tile_n * BN);
    stage(lds);
    for (int k = 0;; ++k) {
        const int row0 = tile_m * BM, col0 = g.col_base + tile_n * BN;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = f32x4_t{ 0.f, 0.f, 0.f, 0.f };
        // the sets the first phase works on start as zeros
#pragma unroll
        for (int i = 0; i < 4; ++i) af[1][i] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < TN; ++i) bfr[1][i] = make_uint4(0, 0, 0, 0);
        staged_wait(); // the tile's first K step (requested before the loop, or before the last tile's stores) is in LDS
        __syncthreads();
        for (int ks = 0; ks < nk; ++ks) {
            if (ks + 1 < nk) stage(lds + nxt); // every wave is past its reads of that buffer (the barrier above)
            k_step(lds + cur);
            staged_wait();
            __syncthreads();
            const int t2 = cur;
            cur = nxt;
            nxt = t2;
        }
        mfma_phase(3); // the last phase of the last step
        const bool more = persistent_tile(k + 1, g.tiles_m, g.tiles_n, tile_m, tile_n);

        if constexpr (EMIT >= 0) {
            emit_hif4_tile16<BM, BN, WM, WN, EMIT>(acc, lds, row0, g.M, col0, g.N, static_cast<uint32_t *>(g.c), g.c_meta);
            if (!more) return;
            __syncthreads(); // the parked tile is read: LDS may take the next tile's first K step
            aim(tile_m * BM, g.col_base + tile_n * BN);
            stage(lds + cur);
        } else {
            // both buffers are free (the barrier that ended the K loop): the next tile's first K step goes into `cur`
            // while the results leave from registers
            if (more) {
                aim(tile_m * BM, g.col_base + tile_n * BN);
                stage(lds + cur);
            }
            // ---- epilogue: lane holds column n of each 16 x 16 tile, rows 4 q + r
            store_acc_16x16<OUT_F32>(acc, g.c, g.ldc, row0 + wm * (BM / WM), col0 + wn * (BN / WN), g.M, g.N);
            if (!more) return;
        }
    }
}

#ifndef HIF4_PLANES_MFMA16
#define HIF4_PLANES_MFMA16 1
#endif

// ---- the last, partly filled round of a launch.  A workgroup holds a CU to itself, so a launch of T tiles runs
// in ceil(T / 256) rounds (per XCD: of its share of the tiles on its 32 CUs), and a last round that is two thirds
// empty costs as much as a full one: 4096 x 11008 is 688 tiles, 2.69 rounds of work in 3 rounds of time.  The remedy
// here keeps one workgroup per tile and the order of every output's additions over K (so the bits of the result do
// not depend on it): the columns are cut in two ranges, whole rounds of 256-column tiles first, then the rest in
// narrower tiles (192 or 128 columns, 48 or 32 per wave) that fill one more round, as a second launch behind the first.
// 4096 x 11008: 32 tile columns of 256 (512 tiles, two rounds), then 2816 columns as 15 x 16 tiles of 192.
struct PlanesSplit {
    int main_tile_cols; // tile columns of 256 in the first launch (0: none)
    int tail_bn;        // tile width of the launch that takes the other columns: 256 (one launch for all), 192 or 128
};

// Rounds a launch of `tiles` tiles runs: its blocks are dealt to the 8 XCDs in equal shares (dense_tile_of_block),
// each XCD has 32 CUs and a workgroup holds a CU to itself.
static int64_t planes_rounds(int64_t tiles)
{
    return ((tiles + 7) / 8 + 31) / 32;
}

// Time of a narrower tile's round in units of a 256-column tile's (measured on MI355X, K steps of 256 x 192 and
// 256 x 128 tiles against 256 x 256), and of the gap between the two launches.
#ifndef HIF4_PLANES_REL192
#define HIF4_PLANES_REL192 0.80
#define HIF4_PLANES_REL128 0.60
#define HIF4_PLANES_GAP 0.04
#endif

// Which split a call of M x N takes: the cheapest by that model among no split and, for each narrower width, the
// most whole rounds of 256-column tiles that leave a tail; a split must save at least 3 %.  Pure host function.
PlanesSplit planes_split(int64_t M, int64_t N)
{
    const PlanesSplit none = { 0, 256 };
    const int64_t tm = (M + 255) / 256, tn = (N + 255) / 256;
    if (!HIF4_PLANES_MFMA16 || tm * tn <= 256 || tm * tn > 16 * 256 || tm > 1024) return none; // one round anyway, or a tail that is small change
    const double t_none = (double)planes_rounds(tm * tn);
    PlanesSplit best = none;
    double t_best = t_none * 0.97;
    const int widths[2] = { 192, 128 };
    const double rel[2] = { HIF4_PLANES_REL192, HIF4_PLANES_REL128 };
    // candidates for the first launch: the most tile columns that make the last or last but one whole number of rounds
    const int64_t full = tm * tn / 256;
    int64_t cand[2];
    int nc = 0;
    for (int64_t k = full; k >= 0 && k + 1 >= full; --k) cand[nc++] = k * 256 / tm;
    for (int wi = 0; wi < 2; ++wi)
        for (int ci = 0; ci < nc; ++ci) {
            const int64_t c = cand[ci];
            if (c >= tn) continue;
            const int64_t tail_cols = N - 256 * c, tt = (tail_cols + widths[wi] - 1) / widths[wi];
            const double t = (double)planes_rounds(tm * c) + rel[wi] * (double)planes_rounds(tm * tt) + (c > 0 ? HIF4_PLANES_GAP : 0.0);
            if (t < t_best) best = { (int)c, widths[wi] }, t_best = t;
        }
    return best;
}

template <int BN>
static int launch_planes16(PlaneGemmArgs g, int out_dtype, hipStream_t stream) // tiles_m, tiles_n, col_base are set
{
    constexpr int BM = 256, WM = 2, WN = 4;
    constexpr size_t lds_bytes = 2 * 8 * (BM + BN) * sizeof(uint4);
    constexpr size_t emit_bytes = emit_lds_bytes<BM, BN>() > lds_bytes ? emit_lds_bytes<BM, BN>() : lds_bytes;
    static_assert(emit_bytes <= 160 * 1024, "fits the LDS of one CU");
    if ((int64_t)g.tiles_m * g.tiles_n > 0x7FFFFFF0) return HIF4_ERR_SHAPE;
    // workgroups that stay (see the kernel): 32 per XCD, one per compute unit, or fewer if the tiles are fewer
    const dim3 grid((unsigned)(8 * persistent_slots(g.tiles_m, g.tiles_n, 32))), block(64 * WM * WN);
    auto launch = [&](auto k, size_t bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return HIF4_ERR_DEVICE;
        hipLaunchKernelGGL(k, grid, block, bytes, stream, g);
        return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
    };
    if (out_dtype == 16 + HIF4_ROUND_RNE) return launch(gemm_planes16_kernel<BM, BN, WM, WN, false, HIF4_ROUND_RNE>, emit_bytes);
    if (out_dtype == 16 + HIF4_ROUND_RHA) return launch(gemm_planes16_kernel<BM, BN, WM, WN, false, HIF4_ROUND_RHA>, emit_bytes);
    if (out_dtype == HIF4_OUT_F32) return launch(gemm_planes16_kernel<BM, BN, WM, WN, true>, lds_bytes);
    return launch(gemm_planes16_kernel<BM, BN, WM, WN, false>, lds_bytes);
}

template <bool MX>
static int launch_planes(PlaneGemmArgs g, int64_t M, int64_t N, int64_t K, int out_dtype, hipStream_t stream)
{
    // 8 waves of 128 x 64: measured faster than 4 waves of 128 x 128 (also on 16 x 16 x 32 MFMAs with 256 accumulator
    // registers per lane and the barrier between the two halves of a K step: 4 to 9 % slower), and smaller
    // workgroup tiles (128 x 128 to 256 x 128) do not help calls of 256 to 4096 rows either
    constexpr int BM = 256, BN = 256, WM = 2, WN = 4;
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    g.tiles_m = (int)((M + BM - 1) / BM);
    g.tiles_n = (int)((N + BN - 1) / BN);
    g.col_base = 0;
    if constexpr (!MX) {
        if (HIF4_PLANES_MFMA16) {
            const PlanesSplit sp = planes_split(M, N);
            if (sp.main_tile_cols > 0) {
                g.tiles_n = sp.main_tile_cols;
                if (int rc = launch_planes16<256>(g, out_dtype, stream)) return rc;
                g.col_base = 256 * sp.main_tile_cols;
            }
            g.tiles_n = (int)((N - g.col_base + sp.tail_bn - 1) / sp.tail_bn);
            if (sp.tail_bn == 192) return launch_planes16<192>(g, out_dtype, stream);
            if (sp.tail_bn == 128) return launch_planes16<128>(g, out_dtype, stream);
            return launch_planes16<256>(g, out_dtype, stream);
        }
    }
    constexpr size_t lds_bytes = 2 * 8 * (BM + BN) * sizeof(uint4);
    if (dense_tile_blocks(g.tiles_m, g.tiles_n) > 0x7FFFFFFF) return HIF4_ERR_SHAPE;
    const dim3 grid((unsigned)dense_tile_blocks(g.tiles_m, g.tiles_n)), block(64 * WM * WN);
    hipError_t e;
    if constexpr (!MX) {
        if (out_dtype == 16 + HIF4_ROUND_RNE || out_dtype == 16 + HIF4_ROUND_RHA) { // result written as HiF4
            constexpr size_t emit_bytes = emit_lds_bytes<BM, BN>() > lds_bytes ? emit_lds_bytes<BM, BN>() : lds_bytes;
            static_assert(emit_bytes <= 160 * 1024, "fits the LDS of one CU");
            auto k = out_dtype == 16 + HIF4_ROUND_RNE ? gemm_planes_kernel<BM, BN, WM, WN, false, false, HIF4_ROUND_RNE>
                                                       : gemm_planes_kernel<BM, BN, WM, WN, false, false, HIF4_ROUND_RHA>;
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)emit_bytes);
            if (e != hipSuccess) return HIF4_ERR_DEVICE;
            hipLaunchKernelGGL(k, grid, block, emit_bytes, stream, g);
            return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
        }
    }
    auto k = out_dtype == HIF4_OUT_F32 ? gemm_planes_kernel<BM, BN, WM, WN, true, MX> : gemm_planes_kernel<BM, BN, WM, WN, false, MX>;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return HIF4_ERR_DEVICE;
    hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, g);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// out_dtype as in launch_gemm: 16 + rounding mode writes the result as HiF4 (c = codes plane, c_meta).
int launch_gemm_planes(const void *a_planes, const void *w_planes, int64_t M, int64_t N, int64_t K, void *c, uint32_t *c_meta,
                       int64_t ldc, int out_dtype, hipStream_t stream)
{
    PlaneGemmArgs g;
    g.a = static_cast<const uint4 *>(a_planes);
    g.w = static_cast<const uint4 *>(w_planes);
    g.a_scale = g.w_scale = nullptr;
    g.c = c;
    g.c_meta = c_meta;
    g.ldc = ldc;
    return launch_planes<false>(g, M, N, K, out_dtype, stream);
}

// ------------------------------------------------------------------ MXFP4 speed reference

// BF16 matrix -> MXFP4 in the plane layout of the kernel above.  One thread per group of 32
// along K (Section I of the HiF4 paper; OCP Microscaling): shared scale 2^(floor(log2 amax) - 2)
// clipped to 2^-127 .. 2^127, stored as its biased exponent (E8M0); elements E2M1 (sign, two
// exponent bits, one mantissa bit), nearest with ties to even, saturated at +-6; element i of
// the group in nibble i of the 16-byte cell.  Cell (row, group g) at g * rows + row.  The scale
// bytes of the 8 groups of a 256-wide K step are laid out for the MFMA lanes: dword
// (ks * 2 + h) * rows + row holds groups h, 2 + h, 4 + h, 6 + h of step ks in bytes 0..3.
// Finite inputs.  K is a multiple of 256.
__global__ __launch_bounds__(256) void mxfp4_pack_kernel(const uint16_t *__restrict__ x, int64_t rows, int64_t gpr, int64_t ldx,
                                                         uint4 *__restrict__ cells, uint8_t *__restrict__ scales)
{
    // consecutive threads take consecutive rows of one group: the cell stores are contiguous
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= rows * gpr) return;
    const int64_t g = id / rows, row = id - g * rows;
    const uint4 *src = reinterpret_cast<const uint4 *>(x + row * ldx + g * 32);
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint4 v = src[i];
        w[4 * i] = v.x, w[4 * i + 1] = v.y, w[4 * i + 2] = v.z, w[4 * i + 3] = v.w;
    }
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t a = w[i] & 0x7FFF7FFFu;
        amax = umax(amax, umax(a & 0xFFFFu, a >> 16));
    }
    // floor(log2 amax) = exponent field - 127 for normals; zero counts as 2^0 (scale 2^-2), and
    // anything below 2^-125 ends at the lower clip
    int shared = amax == 0 ? -2 : (int)(amax >> 7) - 127 - 2;
    shared = shared < -127 ? -127 : shared;
    const float inv = u2f((uint32_t)(127 - shared) << 23); // 2^-shared, exponent field in 2..254
    uint32_t out[4] = { 0, 0, 0, 0 };
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const uint32_t b = (w[i / 2] >> (16 * (i & 1))) & 0xFFFFu;
        const float a = u2f((b & 0x7FFFu) << 16) * inv; // exact: a power-of-two scaling
        float r;
        if (a < 2.0f) r = rintf(a * 2.0f) * 0.5f;
        else if (a < 4.0f) r = rintf(a);
        else r = fminf(rintf(a * 0.5f) * 2.0f, 6.0f);
        // 0, .5, 1, 1.5 -> 0..3;  2, 3 -> 4, 5;  4 -> 6;  6 -> 7
        const uint32_t mag = r < 2.0f ? (uint32_t)(r * 2.0f) : (r < 4.0f ? 2u + (uint32_t)r : (r < 5.0f ? 6u : 7u));
        out[i / 8] |= (((b >> 12) & 8u) | mag) << (4 * (i % 8));
    }
    cells[g * rows + row] = make_uint4(out[0], out[1], out[2], out[3]);
    const int64_t ks = g / 8;
    const int j = (int)(g % 8);
    scales[(((ks * 2 + (j & 1)) * rows + row) << 2) + (j >> 1)] = (uint8_t)(shared + 127);
}

int launch_mxfp4_pack(const void *x, int64_t rows, int64_t K, int64_t ldx, void *cells, void *scales, hipStream_t stream)
{
    const int64_t gpr = K / 32, n = rows * gpr;
    if (n == 0) return HIF4_OK;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(mxfp4_pack_kernel, grid, block, 0, stream, static_cast<const uint16_t *>(x), rows, gpr, ldx,
                       static_cast<uint4 *>(cells), static_cast<uint8_t *>(scales));
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_mxfp4_gemm(const void *a_cells, const void *a_scales, const void *w_cells, const void *w_scales, int64_t M, int64_t N,
                      int64_t K, void *c, int64_t ldc, int out_dtype, hipStream_t stream)
{
    PlaneGemmArgs g;
    g.a = static_cast<const uint4 *>(a_cells);
    g.w = static_cast<const uint4 *>(w_cells);
    g.a_scale = static_cast<const uint32_t *>(a_scales);
    g.w_scale = static_cast<const uint32_t *>(w_scales);
    g.c = c;
    g.c_meta = nullptr;
    g.ldc = ldc;
    return launch_planes<true>(g, M, N, K, out_dtype, stream);
}

} // namespace hif4
