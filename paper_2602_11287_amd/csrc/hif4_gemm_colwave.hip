// HiF4 GEMM for tiles with few rows and many weights per row of A: the grouped (per-expert)
// GEMM, where an expert's rows meet its whole weight matrix once, dense calls of at most 192
// rows, and small dense calls of a few m-tiles.  C = A * W^T per expert, A as
// exact BF16 values (decoded HiF4), W packed HiF4; each 64-wide K step of an output is the
// unit dot product of Eq. 4 of the HiF4 paper (Section III-B), accumulated in fp32 on
// v_mfma_f32_32x32x16_bf16.
//
// The work that counts here is expanding W (Eq. 2, Section II-A): every weight is used by the
// few rows of one expert only, so the expansion cannot be amortised over many tiles as in the
// dense kernels.  Hence the shape: a workgroup owns up to BM = 32 TMAX rows (a whole expert, if
// it fits) and 256 columns; each of its 8 waves owns 32 of those columns over the whole of K
// and expands their weights straight into the B operand registers of its MFMAs - every weight
// is expanded once per m-tile, by one lane, and never passes through LDS as BF16.  The rows of
// A are the same for all waves: a K step of them sits in LDS, [group of 8][row], brought in by
// direct global -> LDS loads from the decoded copy of A ("cell planes", see hif4_gemm_cells.hip:
// the 64 rows a wave moves at once are contiguous in memory) NB steps ahead.  The packed
// weights of a wave go through LDS as well, as bytes, lane-private: a ring of R steps filled by
// the same kind of load, 16 bytes of codes and the metadata word per lane and step.  So every
// global load of the loop is an LDS-writing one with a fixed count per wave and step, and one
// s_waitcnt vmcnt(N) per step covers exactly the loads that step needs.
// (Dense calls have one expert's worth of workgroups only; there the launcher takes 4 waves per
// workgroup and lets groups of waves split K, see the kernel's template arguments.)
//
// K order: sub-step s (of 4, a K slab of 16) takes group 4 h + s of a unit's 8 groups of 8
// from lane half h, for both operands, so a lane's 4 dwords of codes per unit are contiguous.
// A K step of a wave: for each sub-step, the LDS reads of the next sub-step's A operands, then up
// to TMAX MFMAs (one per 32-row block that has rows), each followed by one slice of the expansion
// of the next sub-step's weights.  The step boundary (wait, barrier, loads of the step NB ahead)
// lies before the last sub-step, whose slices already belong to the next unit.
//
// What bounds it on MI355X (measured with the instruction-issue probe of mfma_ceiling.hip): a wave
// issues one vector instruction per 7-8 cycles, a SIMD one per 4, and an MFMA costs about 8 cycles
// of that port next to its 32 in the matrix pipeline.  The expansion is 37 vector instructions per
// 8 weights, so with the two waves per SIMD that the accumulators leave room for, the loop is bound
// by vector instruction issue: everything that is not expansion is kept out of the vector ALUs
// (scalar address arithmetic, loads straight into LDS, one wait per sub-step).
#include <type_traits>

#include "hif4_emit.h"
#include "hif4_expand.h"
#include "hif4_grouped.h"
#include "hif4_store.h"

namespace hif4 {

// LDS-writing loads (see hif4_gemm_cells.hip for why they are inline assembly: the compiler's
// wait-count pass must not see them; the kernel counts them itself).  Address = 64-bit scalar base
// + 32-bit byte offset per lane; lane l lands at lds_byte + 16 l (or + 4 l); lds_byte is wave-uniform.
__device__ __forceinline__ uint64_t cw_uniform(uint64_t v) // a wave-uniform value, in scalar registers
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v), hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ void cw_load_to_lds_16(uint64_t base, uint32_t off, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_byte), "v"(off), "s"(base) : "memory");
}
__device__ __forceinline__ void cw_load_to_lds_4(uint64_t base, uint32_t off, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds_byte), "v"(off), "s"(base) : "memory");
}

struct ColwaveArgs {
    const uint4 *a_planes;   // decoded A: cell (row, group g of 8 along K) at g * M + row
    const uint32_t *w_codes; // [E][N][K/8] dwords
    const uint32_t *w_meta;  // [E][N][K/64]
    const int32_t *offs;     // device int32[E+1], or nullptr: one matrix W for all M rows
    void *c;
    uint32_t *c_meta; // HiF4 result: c is its codes plane [M][N/2], this its metadata plane [M][N/64]
    int64_t ldc;
    int M, N, K, E;
    int tiles_m, tiles_n;
};

// what the kernel writes: BF16, fp32, or the result as HiF4 with units along N (rounding mode OUT - COLWAVE_EMIT)
enum { COLWAVE_BF16 = 0, COLWAVE_F32 = 1, COLWAVE_EMIT = 2 };

// NW waves per workgroup in KS groups of NW / KS (a group takes one KS-th of K, a wave 32 columns of
// it), NB buffers of A, a ring of R steps of packed W.
template <int NW, int KS, int NB, int R>
struct ColwaveShape {
    // mblk: metadata in blocks of 8 units (two blocks of 32 rows per wave) instead of a word per lane and ring step;
    // wpair: codes in pairs of units (64-byte runs per row, see the kernel), (R + 2) / 2 pair slots of 2 KB per wave
    static constexpr size_t lds_bytes(int tmax, bool mblk, bool wpair = false)
    {
        const int rg = (32 * tmax + 63) / 64;
        return (size_t)NB * KS * 8 * 64 * rg * 16 + (wpair ? (size_t)((R + 2) / 2) * NW * 128 * 16 : (size_t)R * NW * 64 * 16) +
               (mblk ? (size_t)NW * 2048 : (size_t)R * NW * 64 * 4);
    }
};

// KS > 1 (dense calls only): the waves of a workgroup split K as well - wave group kw takes the
// units [kw K/64/KS, (kw + 1) K/64/KS) - and their partial sums meet in LDS after the loop.  With few
// rows and not many columns there are too few 32-column strips to give every SIMD its two waves,
// and a wave alone cannot issue faster than it does; K is the only other axis to cut.
// WPAIR: the packed codes come in pairs of units.  One load per step as before, but load j brings rows 16 (j % 2) ..
// + 15 of the wave's 32 weight rows for both units of pair j / 2: four adjacent lanes fetch the 64 contiguous bytes of a
// row, so a request covers half a 128-byte line instead of a quarter, and a line is fetched twice instead of four times
// by the time its four units are used.  The 16-byte chunks of a row are stored XOR-swizzled (chunk c of row n at
// position c ^ (n / 2 % 4) of the row's four), so that the operand reads of a wave are spread over the banks.
template <int TMAX, int NW, int KS, int NB, int R, int WPS, int OUT, bool MBLK, bool WPAIR = false>
__global__ __launch_bounds__(64 * NW, WPS) void gemm_colwave_kernel(ColwaveArgs g)
{
    constexpr bool OUT_F32 = OUT == COLWAVE_F32, EMIT = OUT >= COLWAVE_EMIT;
    constexpr int NWC = NW / KS;             // waves (32-column strips) across a tile
    constexpr int BM = 32 * TMAX, BN = 32 * NWC;
    constexpr int RG = (BM + 63) / 64;       // 64-row groups of a tile
    constexpr int BMP = 64 * RG;             // rows of a buffer
    constexpr int A_CELLS = 8 * BMP;         // cells of one K step of A
    constexpr int IA = (KS * 8 * RG + NW - 1) / NW; // A loads per wave and step
    constexpr int PER_STEP = IA + 2;         // LDS-writing loads per wave and step
    static_assert(R > NB && NB >= 2, "W(k + 1) must be older than A(k + 1)");
    static_assert(!WPAIR || R >= NB + 2, "both loads of the pair of unit k + 1 must be older than A(k + 1)");
    constexpr int RP = (R + 2) / 2;          // WPAIR: pair slots of the codes ring
    constexpr int WC_CELLS = WPAIR ? RP * NW * 128 : R * NW * 64;
    static_assert(NW % KS == 0, "whole wave groups");
    extern __shared__ uint4 lds[];
    uint4 *lds_a = lds;                                  // [NB][KS][8][BMP]
    uint4 *lds_wc = lds + NB * KS * A_CELLS;             // [R][NW][64], or WPAIR: [RP][NW][2 halves][16 rows][4 chunks]
    uint32_t *lds_wm = reinterpret_cast<uint32_t *>(lds_wc + WC_CELLS); // [R][NW][64], or MBLK: [NW][2 blocks][32 rows][8 units]

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int cw = wave % NWC, kw = wave / NWC; // column strip and K part of this wave
    const int half = lane / 32, l32 = lane % 32;

    // ---- which tile: m-tiles are dealt to the 8 XCDs round-robin (block b runs on XCD b % 8), all
    // n-tiles of an m-tile on one XCD, whose L2 then serves their common rows of A
    // (with fewer than 8 m-tiles the n-tiles of one are spread over the XCDs instead)
    const int bi = (int)(blockIdx.x / 8);
    const bool deal_m = g.tiles_m >= 8;
    const int tile_m = deal_m ? (bi / g.tiles_n) * 8 + (int)(blockIdx.x % 8) : (int)blockIdx.x / g.tiles_n;
    const int tile_n = deal_m ? bi % g.tiles_n : (int)blockIdx.x % g.tiles_n;
    if (tile_m >= g.tiles_m) return;
    int row0, rows_end;
    const uint32_t *w_codes = g.w_codes, *w_meta = g.w_meta;
    if (g.offs) {
        int e;
        if (!find_expert_tile<BM>(g.offs, g.E, g.M, tile_m, lane, e, row0, rows_end)) return;
        w_codes += (int64_t)e * g.N * (g.K / 8);
        w_meta += (int64_t)e * g.N * (g.K / 64);
    } else {
        row0 = tile_m * BM;
        rows_end = g.M;
    }
    const int col0 = tile_n * BN;
    const int nk = g.K / 64 / KS; // K steps of a wave (the host gives KS > 1 only a K it divides)
    const int u0 = kw * nk;       // its first unit
    // 32-row blocks of this tile that have rows
    int live = (rows_end - row0 + 31) / 32;
    live = __builtin_amdgcn_readfirstlane(live < TMAX ? live : TMAX);

    // ---- load plan.  W: lane (n, h) = (l32, half) takes the 16 bytes of codes [16 h, 16 h + 16)
    // of each unit of weight row col0 + 32 cw + n, and the unit's metadata word.  A: load
    // id = wave * IA + i moves, for wave group ks = id / (8 RG), cell j = id / RG % 8 of rows
    // rg * 64 .. + 63 (rg = id % RG); rows past the end of the matrix repeat its last row, loads past
    // 8 RG KS repeat the last one.
    // Every address is a scalar base that moves with the K step plus a fixed 32-bit offset per lane
    // (the host keeps the operands small enough for that).
    int wrow = col0 + cw * 32 + l32;
    wrow = wrow < g.N ? wrow : g.N - 1;
    const uint32_t wc_off = (uint32_t)wrow * (uint32_t)(g.K / 2) + 16u * half + (uint32_t)u0 * 32u;
    // WPAIR, load half t: lane -> weight row 16 t + lane / 4 of the wave's 32, position lane % 4 of the row's four 16-byte
    // chunks, which holds chunk position ^ swizzle(row); chunk c = half c % 2 of unit c / 2 of the pair.  The last pair
    // of an odd number of units has its first unit only: its chunks 2 and 3 repeat chunks 0 and 1 (never used, in bounds).
    // (plain values combined by masks, no arrays indexed by the load's parity: those would live in scratch memory)
    uint32_t wp_off0, wp_delta, wp_tail_adj;
    {
        const int r16 = lane / 4, c = (lane % 4) ^ ((r16 >> 1) & 3);
        int row0w = col0 + cw * 32 + r16, row1w = row0w + 16;
        row0w = row0w < g.N ? row0w : g.N - 1;
        row1w = row1w < g.N ? row1w : g.N - 1;
        wp_off0 = (uint32_t)row0w * (uint32_t)(g.K / 2) + 16u * c + (uint32_t)u0 * 32u;
        wp_delta = (uint32_t)(row1w - row0w) * (uint32_t)(g.K / 2); // half 1 of a load pair: 16 rows further on
        wp_tail_adj = 16u * (c & 2);                                // back to chunk c % 2
    }
    // Metadata.  MBLK: blocks of 8 units of the wave's 32 rows, one load of 8 rows x 8 units (32-byte runs) per step, see
    // issue_w; lane -> row lane / 8 of the load's 8, unit lane % 8 of the block (a K range of fewer than 8 units repeats
    // its last one).  Rows past N - 1 take row N - 1: the byte offset is capped at that row's (it grows with the row).
    // Otherwise the unit's word per lane and step.
    const int mj = lane % 8 < nk ? lane % 8 : nk - 1;
    const uint32_t wm_stride8 = (uint32_t)(g.K / 16) * 8u; // bytes between rows r and r + 8
    const uint32_t wm_off = MBLK ? (uint32_t)(col0 + cw * 32 + lane / 8) * (uint32_t)(g.K / 16) + (uint32_t)(u0 + mj) * 4u
                                 : (uint32_t)wrow * (uint32_t)(g.K / 16) + (uint32_t)u0 * 4u;
    const uint32_t wm_off_cap = (uint32_t)(g.N - 1) * (uint32_t)(g.K / 16) + (uint32_t)(u0 + mj) * 4u;
    // first unit of metadata block b of this wave's K range: the last block is moved back to end with the range
    auto mblk_start = [&](int b) { const int s8 = 8 * b; return nk >= 8 ? (s8 < nk - 8 ? s8 : nk - 8) : 0; };
    uint32_t a_off[IA], a_dst[IA];
#pragma unroll
    for (int i = 0; i < IA; ++i) {
        int id = wave * IA + i;
        id = id < KS * 8 * RG ? id : KS * 8 * RG - 1;
        const int ks = id / (8 * RG), j = id / RG % 8, rg = id % RG;
        int row = row0 + rg * 64 + lane;
        row = row < g.M ? row : g.M - 1;
        a_off[i] = ((uint32_t)(ks * nk * 8 + j) * (uint32_t)g.M + (uint32_t)row) * 16u;
        a_dst[i] = (uint32_t)__builtin_amdgcn_readfirstlane(((ks * 8 + j) * BMP + rg * 64) * 16);
    }
    auto lds_byte_of = [](const void *p) { return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)p; };
    const uint32_t a_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_byte_of(lds_a));
    const uint32_t wc_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_byte_of(lds_wc)) + (uint32_t)(wave * (WPAIR ? 128 : 64) * 16);
    const uint32_t wm_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_byte_of(lds_wm)) + (uint32_t)(wave * (MBLK ? 2048 : 64 * 4));
    const uint64_t a_step = (uint64_t)g.M * 128; // bytes of A planes per K step
    const uint64_t wc_ptr = cw_uniform((uint64_t)(uintptr_t)w_codes), wm_ptr = cw_uniform((uint64_t)(uintptr_t)w_meta);
    const uint64_t a_ptr = cw_uniform((uint64_t)(uintptr_t)g.a_planes);
    // the loads of unit u into ring slot / buffer number `at`: steps past the end of K repeat the last one (never used)
    // MBLK: the load of 8 rows x 8 units of metadata that goes with it belongs to block b = (u - R + 9) / 8, rows
    // 8 t .. 8 t + 7 with t = (u - R + 9) % 4: in step k = u - R of the main loop, block b is written during steps
    // 8 b - 9 .. 8 b - 2 (each quarter twice, the same bytes), after the last read of block b - 2 in the same slot
    // (unit 8 b - 9, read in step 8 b - 10) and complete with the load of step 8 b - 6, which every wait from step
    // 8 b - 6 + NB on covers (NB <= 3; the block's first unit is read in step 8 b - 1).  One load per step, so the
    // count of loads per step stays what the waits assume.
    auto issue_meta_block = [&](int b, int t) {
        uint32_t off = wm_off + (uint32_t)t * wm_stride8;
        off = off < wm_off_cap ? off : wm_off_cap;
        cw_load_to_lds_4(wm_ptr + (uint64_t)mblk_start(b) * 4, off, wm_base + (uint32_t)((b & 1) * 1024 + t * 256));
    };
    auto issue_w = [&](int u, int at) {
        const uint64_t uc = (uint64_t)(u < nk ? u : nk - 1);
        if constexpr (WPAIR) { // load number u: half u % 2 of pair u / 2 (`at` is not used: the pair slot follows from u)
            const int last = (nk - 1) / 2, p = u / 2 < last ? u / 2 : last, t = u & 1;
            const bool tail = 2 * p + 1 >= nk; // wave-uniform
            cw_load_to_lds_16(wc_ptr + (uint64_t)p * 64, wp_off0 + (wp_delta & (0u - (uint32_t)t)) - (wp_tail_adj & (0u - (uint32_t)tail)), wc_base + (uint32_t)(((u / 2) % RP * NW * 128 + t * 64) * 16));
        } else {
            cw_load_to_lds_16(wc_ptr + uc * 32, wc_off, wc_base + (uint32_t)(at * NW * 64 * 16));
        }
        if constexpr (MBLK) {
            const int x = u - R + 9; // >= 9 - R > 0
            issue_meta_block(x >> 3, x & 3);
        } else {
            cw_load_to_lds_4(wm_ptr + uc * 4, wm_off, wm_base + (uint32_t)(at * NW * 64 * 4));
        }
    };
    auto issue_a = [&](int u, int at) {
        const uint64_t base = a_ptr + (uint64_t)(u < nk ? u : nk - 1) * a_step;
#pragma unroll
        for (int i = 0; i < IA; ++i) cw_load_to_lds_16(base, a_off[i], a_base + (uint32_t)(at * KS * A_CELLS * 16) + a_dst[i]);
    };

    f32x16_t acc[TMAX];
#pragma unroll
    for (int i = 0; i < TMAX; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;

    // ---- the packed weights of the unit being expanded, as this lane needs them
    struct UnitW {
        uint32_t c[4];   // codes dwords 4 h .. 4 h + 3
        uint32_t m8, m16; // the unit's level-2 and level-3 bits, shifted so that bit 0 belongs to group 4 h
        uint32_t sbase;  // fp32 pattern of the unit scale
    };
    const uint32_t *lds_wm_lane = lds_wm + wave * 512 + l32 * 8; // MBLK: this lane's row in block slot 0
    // WPAIR: this lane's cell of a pair slot, for the first and the second unit of the pair
    const int wp_sw = (l32 >> 1) & 3;
    const int wp_cell0 = (l32 / 16) * 64 + 4 * (l32 % 16) + (half ^ wp_sw), wp_cell_delta = ((2 + half) ^ wp_sw) - (half ^ wp_sw);
    auto read_w = [&](UnitW &uw, int slot, int u) { // ring slot and number (in the wave's K range) of the unit
        uint4 cw;
        if constexpr (WPAIR) cw = lds_wc[((u / 2) % RP * NW + wave) * 128 + wp_cell0 + (wp_cell_delta & (0 - (u & 1)))];
        else cw = lds_wc[(slot * NW + wave) * 64 + lane];
        uint32_t m;
        if constexpr (MBLK) {
            const int uc = u < nk ? u : nk - 1, b = uc >> 3;
            m = lds_wm_lane[(b & 1) * 256 + uc - mblk_start(b)];
        } else {
            m = lds_wm[(slot * NW + wave) * 64 + lane];
        }
        uw.c[0] = cw.x, uw.c[1] = cw.y, uw.c[2] = cw.z, uw.c[3] = cw.w;
        uw.m8 = m >> (8 + 4 * half);
        uw.m16 = m >> (16 + 8 * half);
        uw.sbase = unit_scale_bits(m);
    };
    auto begin = [&](const UnitW &uw, int d) {
        ChunkState st;
        const uint32_t e8 = (uw.m8 >> d) & 1u, e16a = (uw.m16 >> (2 * d)) & 1u, e16b = (uw.m16 >> (2 * d + 1)) & 1u;
        st.sa = u2f(uw.sbase + ((e8 + e16a) << 23));
        st.sb = u2f(uw.sbase + ((e8 + e16b) << 23));
        st.c = uw.c[d];
        st.lo = st.c & 0x07070707u;
        st.hi = (st.c >> 4) & 0x07070707u;
        asm volatile("" : "+v"(st.lo), "+v"(st.hi));
        return st;
    };

    // ---- prologue.  After the barrier of step k the loop issues the group [A(k + NB), W(k + R)]; the
    // same groups for k < 0 start the pipeline, so that the loads in flight are always the same ones.
    if constexpr (MBLK) { // the first block of metadata, whole, before everything else
#pragma unroll
        for (int t = 0; t < 4; ++t) issue_meta_block(0, t);
    }
#pragma unroll
    for (int u = 0; u < R - NB; ++u) issue_w(u, u);
#pragma unroll
    for (int k = -NB; k < 0; ++k) {
        issue_a(k + NB, k + NB);
        issue_w(k + R, k + R);
    }
    // Why the wait counts below are exact.  (1) Loads land in the order they were issued, and from here to the end of
    // the main loop this wave issues no vector memory instruction but the LDS-writing loads of issue_a / issue_w, PER_STEP
    // per step in a fixed order: the reads of the row offsets in find_expert_tile were consumed above (the compiler waited
    // for them before the lane shuffles), the results are stored after the loop's final vmcnt(0), and the build fails if
    // this kernel uses scratch memory (paper_2602_11287_amd/build.py), so no spill code can sit between them.
    // (2) In the prologue the order is W(0) .. W(R - NB - 1), then [A(j), W(j + R - NB)] for j = 0 .. NB - 1: the loads
    // younger than A(0) are its own W (2) and NB - 1 later groups.  (3) In the loop, step k issues [A(k + NB), W(k + R)]
    // after its wait, so at the wait of step k the loads younger than A(k + 1) are W(k + 1 + R - NB) (2) and the groups
    // of steps k + 2 - NB .. k - 1, i.e. NB - 2 of them; W(k + 1) is older than A(k + 1) because R > NB.
    // A(0) and W(0) have landed once only the loads younger than A(0) are in flight
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 + (NB - 1) * PER_STEP) : "memory");
    __syncthreads();

    // The main loop, compiled once per number of row blocks that have rows (LIVE), so that its body
    // is one straight run of instructions: the slices of the expansion stay between the MFMAs where
    // they are put, and the waits for LDS reads count exactly.
    auto run = [&](auto live_c) {
        constexpr int LIVE = decltype(live_c)::value;
        constexpr int SP = (5 + LIVE - 1) / LIVE; // expansion slices after each MFMA (5 per sub-step)
        uint4 af[2][LIVE]; // A operands of two sub-steps, one per row block
        uint4 bcur, bnext;
        UnitW uw;
        ChunkState cs;
        auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
        // A operands of sub-step s from buffer `buf` into set `set`
        auto a_frags = [&](int set, int buf, int s) {
            const uint4 *src = lds_a + (buf * KS + kw) * A_CELLS + (4 * half + s) * BMP + l32;
#pragma unroll
            for (int i = 0; i < LIVE; ++i) af[set][i] = src[i * 32];
        };
        // One sub-step: request the A operands of the next one (sub-step ns of buffer nbuf), then the
        // MFMAs on (af[set], bcur), each followed by a slice of the expansion of dword d of `uw`.
        auto sub_step = [&](int set, int d, int nbuf, int ns) {
            a_frags(set ^ 1, nbuf, ns);
            fence();
#pragma unroll
            for (int i = 0; i < LIVE; ++i) {
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[set][i]), __builtin_bit_cast(bf16x8_t, bcur), acc[i], 0, 0, 0);
#pragma unroll
                for (int sl = i * SP; sl < (i + 1) * SP; ++sl) {
                    if (sl == 0) cs = begin(uw, d);
                    else if (sl == 1) bnext.x = chunk_pair<0>(cs);
                    else if (sl == 2) bnext.y = chunk_pair<1>(cs);
                    else if (sl == 3) bnext.z = chunk_pair<2>(cs);
                    else if (sl == 4) bnext.w = chunk_pair<3>(cs);
                }
                fence();
            }
            bcur = bnext;
        };

        read_w(uw, 0, 0);
        cs = begin(uw, 0);
        bcur.x = chunk_pair<0>(cs);
        bcur.y = chunk_pair<1>(cs);
        bcur.z = chunk_pair<2>(cs);
        bcur.w = chunk_pair<3>(cs);
        bnext = bcur;
        a_frags(0, 0, 0);

        int buf = 0, slot = 0; // buffer of A(k), ring slot of W(k)
        for (int k = 0; k < nk; ++k) {
            const int nbuf = buf + 1 == NB ? 0 : buf + 1, nslot = (slot + 1) % R;
            sub_step(0, 1, buf, 1);
            sub_step(1, 2, buf, 2);
            sub_step(0, 3, buf, 3);
            // A(k + 1) and W(k + 1) have landed once only the loads younger than A(k + 1) are in flight
            asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 + (NB - 2) * PER_STEP) : "memory");
            __syncthreads(); // every wave holds its last operands of buffer `buf`, which may now be refilled
            issue_a(k + NB, buf);
            issue_w(k + R, slot);
            read_w(uw, nslot, k + 1);
            sub_step(1, 0, nbuf, 0);
            buf = nbuf;
            slot = nslot;
        }
    };
    static_assert(TMAX <= 8, "dispatch below");
    switch (live) {
    case 1: run(std::integral_constant<int, 1>{}); break;
    case 2: run(std::integral_constant<int, 2>{}); break;
    case 3: if constexpr (TMAX >= 3) run(std::integral_constant<int, 3>{}); break;
    case 4: if constexpr (TMAX >= 4) run(std::integral_constant<int, 4>{}); break;
    case 5: if constexpr (TMAX >= 5) run(std::integral_constant<int, 5>{}); break;
    case 6: if constexpr (TMAX >= 6) run(std::integral_constant<int, 6>{}); break;
    case 7: if constexpr (TMAX >= 7) run(std::integral_constant<int, 7>{}); break;
    default: if constexpr (TMAX >= 8) run(std::integral_constant<int, 8>{}); break;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // no load may outlive the workgroup's LDS

    // ---- KS > 1: the partial sums of wave groups 1 .. KS - 1 go through LDS (all loads have landed and
    // all operands are read once every wave is past the barrier) to group 0, lane for lane
    if constexpr (KS > 1) {
        static_assert((size_t)(KS - 1) * NWC * TMAX * 4096 <= ColwaveShape<NW, KS, NB, R>::lds_bytes(TMAX, MBLK, WPAIR), "partial sums fit the buffers");
        float4 *red = reinterpret_cast<float4 *>(lds); // [kw - 1][cw][block][4][lane]
        __syncthreads();
        if (kw > 0) {
            float4 *dst = red + (size_t)((kw - 1) * NWC + cw) * TMAX * 256 + lane;
#pragma unroll
            for (int i = 0; i < TMAX; ++i) {
                if (i >= live) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) dst[(i * 4 + q) * 64] = make_float4(acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]);
            }
        }
        __syncthreads();
        if (!EMIT && kw > 0) return; // (a HiF4 result is encoded by all waves, see below)
        if (kw == 0) {
#pragma unroll
            for (int p = 0; p < KS - 1; ++p) {
                const float4 *src = red + (size_t)(p * NWC + cw) * TMAX * 256 + lane;
#pragma unroll
                for (int i = 0; i < TMAX; ++i) {
                    if (i >= live) continue;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 v = src[(i * 4 + q) * 64];
                        acc[i][4 * q] += v.x, acc[i][4 * q + 1] += v.y, acc[i][4 * q + 2] += v.z, acc[i][4 * q + 3] += v.w;
                    }
                }
            }
        }
    }

    // ---- result as HiF4 (hif4_emit.h): the tile, rounded to BF16 as the BF16 output would be, is parked in LDS
    // row-major by the waves that hold it, then every thread of the workgroup encodes units of 64 columns
    if constexpr (EMIT) {
        static_assert(BN % 64 == 0, "whole units across a tile");
        static_assert(emit_lds_bytes<BM, BN>() <= ColwaveShape<NW, KS, NB, R>::lds_bytes(TMAX, MBLK, WPAIR), "the parked tile fits the buffers");
        constexpr int RS = BN + 8; // row stride in BF16 elements
        uint16_t *tile = reinterpret_cast<uint16_t *>(lds);
        __syncthreads(); // all operand reads and loads are done (KS > 1: and group 0 has read the partial sums)
        if (kw == 0) {
#pragma unroll
            for (int i = 0; i < TMAX; ++i) {
                if (i >= live) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t u = f2u(acc[i][r]);
                    tile[(i * 32 + 8 * (r / 4) + 4 * half + (r % 4)) * RS + cw * 32 + l32] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
                }
            }
        }
        __syncthreads();
        emit_encode_parked<BM, BN, 64 * NW, OUT - COLWAVE_EMIT>(tile, row0, rows_end, col0, g.N, static_cast<uint32_t *>(g.c), g.c_meta);
        return;
    }

    // ---- epilogue: lane holds column l32 of each 32 x 32 block, rows 8 (r / 4) + 4 half + r % 4
    store_acc_32x32<OUT_F32>(acc, g.c, g.ldc, row0, col0 + cw * 32, rows_end, g.N);
}

#ifndef HIF4_COLWAVE_NW
#define HIF4_COLWAVE_NW 8
#define HIF4_COLWAVE_NB 3
#define HIF4_COLWAVE_R 4
#define HIF4_COLWAVE_WPS 2
#endif
// waves per workgroup of a dense call (one matrix W, few m-tiles) that does not split K: the grid is
// N / (32 NW) workgroups, and half as many columns per workgroup fill the chip better at every width measured
#ifndef HIF4_COLWAVE_NW_DENSE
#define HIF4_COLWAVE_NW_DENSE 4
#endif
#ifndef HIF4_COLWAVE_MBLK
#define HIF4_COLWAVE_MBLK 1
#endif
#ifndef HIF4_COLWAVE_WPAIR
#define HIF4_COLWAVE_WPAIR 1
#endif
// EMIT_OK: also instantiate the kernels that write the result as HiF4
template <int TMAX, int NW, int KS, bool EMIT_OK = false>
static int launch_colwave_t(ColwaveArgs g, int out_dtype, hipStream_t stream)
{
    // three buffers of A where LDS has room for them, else two; the codes of W in pairs of units (64-byte runs per row,
    // a ring of NB + 2 steps) where that fits as well, else one unit per step (a ring of NB + 1); metadata in blocks of 8
    // units (a quarter of the cache lines fetched per step) where that fits as well
    constexpr size_t LDS_MAX = 160 * 1024;
    constexpr bool PAIR3 = HIF4_COLWAVE_WPAIR && ColwaveShape<NW, KS, 3, 5>::lds_bytes(TMAX, false, true) <= LDS_MAX;
    constexpr bool PAIR2 = HIF4_COLWAVE_WPAIR && !PAIR3 && ColwaveShape<NW, KS, 2, 4>::lds_bytes(TMAX, false, true) <= LDS_MAX &&
                           ColwaveShape<NW, KS, HIF4_COLWAVE_NB, HIF4_COLWAVE_R>::lds_bytes(TMAX, false) > LDS_MAX;
    constexpr bool WPAIR = PAIR3 || PAIR2;
    constexpr bool DEEP = ColwaveShape<NW, KS, HIF4_COLWAVE_NB, HIF4_COLWAVE_R>::lds_bytes(TMAX, false) <= LDS_MAX;
    constexpr int NB = PAIR3 ? 3 : PAIR2 ? 2 : DEEP ? HIF4_COLWAVE_NB : 2, R = WPAIR ? NB + 2 : DEEP ? HIF4_COLWAVE_R : 3, WPS = HIF4_COLWAVE_WPS;
    constexpr bool MBLK = HIF4_COLWAVE_MBLK && ColwaveShape<NW, KS, NB, R>::lds_bytes(TMAX, true, WPAIR) <= LDS_MAX;
    constexpr int BM = 32 * TMAX, BN = 32 * NW / KS;
    constexpr size_t lds_bytes = ColwaveShape<NW, KS, NB, R>::lds_bytes(TMAX, MBLK, WPAIR);
    static_assert(lds_bytes <= 160 * 1024, "fits the LDS of one CU");
    g.tiles_n = (g.N + BN - 1) / BN;
    g.tiles_m = g.offs ? g.M / BM + g.E : (g.M + BM - 1) / BM; // grouped: upper bound of sum_e ceil(rows_e / BM)
    const int64_t blocks = (int64_t)(g.tiles_m >= 8 ? (g.tiles_m + 7) / 8 * 8 : g.tiles_m) * g.tiles_n;
    const dim3 grid((unsigned)blocks), block(64 * NW);
    auto launch = [&](auto k) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess) return false;
        hipLaunchKernelGGL(k, grid, block, lds_bytes, stream, g);
        return true;
    };
    bool ok;
    if (out_dtype == HIF4_OUT_F32) ok = launch(gemm_colwave_kernel<TMAX, NW, KS, NB, R, WPS, COLWAVE_F32, MBLK, WPAIR>);
    else if (out_dtype == HIF4_OUT_BF16) ok = launch(gemm_colwave_kernel<TMAX, NW, KS, NB, R, WPS, COLWAVE_BF16, MBLK, WPAIR>);
    else if constexpr (EMIT_OK && BN % 64 == 0) { // 16 + rounding mode: the result as HiF4 (the launcher below picks shapes that allow it)
        ok = out_dtype == 16 + HIF4_ROUND_RNE ? launch(gemm_colwave_kernel<TMAX, NW, KS, NB, R, WPS, COLWAVE_EMIT + HIF4_ROUND_RNE, MBLK, WPAIR>)
                                              : launch(gemm_colwave_kernel<TMAX, NW, KS, NB, R, WPS, COLWAVE_EMIT + HIF4_ROUND_RHA, MBLK, WPAIR>);
    } else return HIF4_ERR_UNSUPPORTED;
    if (!ok) return HIF4_ERR_DEVICE;
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// The kernel addresses each operand as a scalar base plus a 32-bit byte offset per lane.
bool colwave_fits(int64_t M, int64_t N, int64_t K)
{
    return M * 128 < ((int64_t)1 << 32) && N * (K / 2) < ((int64_t)1 << 32) && M * K * 2 < ((int64_t)1 << 32);
}

// a_planes: decoded A as cell planes (launch_decode_planes).  offs != nullptr: grouped, E experts;
// rows_per_tile: 64, 128, 192 or 256 rows of A per workgroup.
// out_dtype: HIF4_OUT_BF16, HIF4_OUT_F32, or (N a multiple of 64) 16 + rounding mode for a HiF4 result:
// c = codes plane, c_meta = its metadata plane, ldc unused.
int launch_gemm_colwave(const void *a_planes, const uint8_t *w_codes, const uint32_t *w_meta, const int32_t *offs, int E,
                        int64_t M, int64_t N, int64_t K, void *c, uint32_t *c_meta, int64_t ldc, int out_dtype, int rows_per_tile,
                        hipStream_t stream)
{
    ColwaveArgs g;
    g.a_planes = static_cast<const uint4 *>(a_planes);
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
    constexpr int NWG = HIF4_COLWAVE_NW, NWD = HIF4_COLWAVE_NW_DENSE;
    {
        // m-tiles: of a dense call, or what a grouped one is expected to have (between M / tile and M / tile + E; the
        // grid itself is sized for the upper bound, this number only picks the shape of the workgroups)
        const int tile_rows = rows_per_tile <= 64 ? 64 : rows_per_tile <= 128 ? 128 : rows_per_tile <= 192 ? 192 : 256;
        const int64_t m_tiles = offs ? M / tile_rows + (E + 1) / 2 : (M + rows_per_tile - 1) / rows_per_tile;
        const int64_t strips = (N + 31) / 32 * m_tiles, nk = K / 64;
        const bool emit = out_dtype >= 16;
        // K parts per workgroup (4, 2 or 1; tiles of more than 128 rows: LDS holds 2) and waves (4 or 8): the
        // most parts whose workgroups still run in one round (one workgroup per CU), with 4 waves rather than
        // 8 when both do - measured: twice the CUs beat twice the waves per CU.  Parts divide K's units and
        // keep at least 8 steps each.
        int ks = rows_per_tile > 128 ? 2 : 4, nw = NWD;
        for (; ks > 1; ks /= 2) {
            if (nk % ks != 0 || nk / ks < 8) continue;
            if (strips * ks <= 4 * 256 && !(emit && ks == 4)) { nw = 4; break; } // (a HiF4 result needs 64 columns per workgroup)
            if (strips * ks <= 8 * 256) { nw = 8; break; }
        }
        // no split: 4 waves per workgroup, unless their workgroups need a second round and are too big to share a
        // CU (tiles of more than 128 rows) - then 8 waves, half as many workgroups
        // (a grouped call keeps 8 waves once its strips make a full round of them: measured equal or better on 64
        // experts; below that 4 waves, 1.3 times faster on 8 to 16 experts whose K does not split)
        if (ks == 1) nw = offs ? (strips <= 8 * 256 ? NWD : NWG) : (strips <= 4 * 256 || rows_per_tile <= 128) ? NWD : NWG;
#define HIF4_CW_CASE(T, W, S) if (nw == W && ks == S) return launch_colwave_t<T, W, S, true>(g, out_dtype, stream)
        if (rows_per_tile <= 64) {
            HIF4_CW_CASE(2, 8, 4); HIF4_CW_CASE(2, 8, 2); HIF4_CW_CASE(2, 4, 4); HIF4_CW_CASE(2, 4, 2); HIF4_CW_CASE(2, NWG, 1);
            return launch_colwave_t<2, NWD, 1, true>(g, out_dtype, stream);
        }
        if (rows_per_tile <= 128) {
            HIF4_CW_CASE(4, 8, 4); HIF4_CW_CASE(4, 8, 2); HIF4_CW_CASE(4, 4, 4); HIF4_CW_CASE(4, 4, 2); HIF4_CW_CASE(4, NWG, 1);
            return launch_colwave_t<4, NWD, 1, true>(g, out_dtype, stream);
        }
        if (rows_per_tile <= 192) {
            HIF4_CW_CASE(6, 8, 2); HIF4_CW_CASE(6, 4, 2); HIF4_CW_CASE(6, NWG, 1);
            return launch_colwave_t<6, NWD, 1, true>(g, out_dtype, stream);
        }
        HIF4_CW_CASE(8, 8, 2); HIF4_CW_CASE(8, 4, 2); HIF4_CW_CASE(8, NWG, 1);
        return launch_colwave_t<8, NWD, 1, true>(g, out_dtype, stream);
#undef HIF4_CW_CASE
    }
}

} // namespace hif4
