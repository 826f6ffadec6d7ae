// HiF4 GEMM for at most 32 rows of A (token generation: the "decode" shape): C[M][N] = A[M][K] * W[N][K]^T
// with W packed HiF4 and A BF16 rows (plain activations, or the exact BF16 values of HiF4 activations).
// The work is streaming W from HBM once, 0.5625 bytes per weight, and turning it into matrix operands;
// every 64-wide K step of an output is the unit dot product of Eq. 4 of the HiF4 paper (Section III-B),
// in the factored form that equation prints: the sum over the unit's 64 products of S1P2 integers and
// micro-exponent powers of two first, one multiplication by the unit scale E6M2 after it.
//
// How a weight becomes an operand (Eq. 2, Section II-A, without its E6M2 factor): the 3-bit magnitude of
// four codes goes through one v_perm_b32 with the FP8 (E4M3) patterns of 0..7 as its byte table, the
// sign bits are OR-ed in, and v_cvt_scalef32_pk_bf16_fp8 turns two such bytes into two BF16 values times
// 2^(E1_8 + E1_16), the power of two riding in the exponent of its scale operand (zero stays zero, which
// a table of BF16 patterns with the exponent added afterwards would not give).  That is about 2.3 vector
// instructions per weight instead of 4.6 for the expansion that carries the E6M2 factor in every weight.
// The factor (4 + M) 2^(E - 50) of the unit, which no 8-bit format can carry next to the code (six
// significant bits), is applied to the unit's partial sums instead: every unit starts from a zero
// accumulator, and 8 fused multiply-adds per lane and 16 rows add its scaled sums to the running result.  With few rows that is cheap; from about 128 rows
// on it would cost what it saves, which is why the kernels for more rows keep the full expansion.
//
// Shape: a wave owns a strip of CG column groups of 16 output columns (v_mfma_f32_16x16x32_bf16, whose K of
// 32 is half a unit: lane (n, q) = (lane % 16, lane / 16) supplies group 4 hs + q of the unit's 8 groups of 8
// from both operands in half step hs) over one of KS parts of K; a workgroup is NWC such column strips
// times KS parts.  With CG = 2 an operand of A serves two MFMAs; with CG = 1 there are twice as many strips to
// spread over the compute units and over K, which is what counts on all but the widest matrices.
// Everything comes in through LDS by direct global -> LDS loads, D steps of two units deep, so that the
// bytes in flight per CU (what hides HBM latency) are bounded by LDS, not by registers:
//   W codes  per wave and step: 16 CG rows x 64 bytes, four adjacent lanes per row, so every request
//            covers whole 64-byte runs of a row (two steps use up a 128-byte line); the 16-byte chunks
//            of a row are stored XOR-swizzled so that the operand reads are spread over the banks;
//   W meta   per wave and 8 steps: 16 CG rows x 16 words (64-byte runs again: a request per row and step for
//            8 bytes would double the number of requests, and requests in flight are what a CU runs out of);
//   A        per K part and step: 16 cells of 8 values x RM rows, [cell][row], shared by the part's
//            NWC waves (plain 16-byte pieces of the rows of A: the K order inside a cell is natural here).
// One barrier per step (two units).  The partial sums of the K parts meet in LDS at the end, in a
// fixed order.  All global loads of the loop are LDS-writing loads in inline assembly, PER per wave and step
// plus CG of metadata every eighth step, issued at least eight steps before their use; loads land in
// the order they were issued, so s_waitcnt vmcnt((D - 2) PER) before step i leaves only loads younger than
// those of step i in flight (the compiler never sees them, and the loop contains no other vector memory
// instruction).  K must be a multiple of 256 (metadata rows then start on 16-byte boundaries).
#include <type_traits>

#include "hif4_expand_fp8.h"

namespace hif4 {

__device__ __forceinline__ void fr_load_to_lds_16(uint64_t base, uint32_t off, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_byte), "v"(off), "s"(base) : "memory");
}
__device__ __forceinline__ void fr_load_to_lds_4(uint64_t base, uint32_t off, uint32_t lds_byte)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds_byte), "v"(off), "s"(base) : "memory");
}
__device__ __forceinline__ uint64_t fr_uniform(uint64_t v) // a wave-uniform value, in scalar registers
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v), hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

struct FewRowsArgs {
    const void *a; // BF16 [M][lda], natural element order
    int64_t lda;
    const uint8_t *w_codes; // [N][K/2]
    const uint32_t *w_meta; // [N][K/64]
    void *c;
    int64_t ldc;
    int M, N, K;
    int out_f32;
};

template <int RM, int NWC, int KS, int CG>
struct FewRowsShape {
    static constexpr int NW = NWC * KS;
    static constexpr size_t slot_bytes = (size_t)KS * 16 * RM * 16 + (size_t)NW * CG * 1024; // A of every K part, codes of every wave
    static constexpr size_t meta_bytes = (size_t)NW * 2 * CG * 1024;                          // two blocks of 16 units x 16 CG rows per wave
    // workgroups of 4 waves leave room for a second one on the CU where three steps fit half the LDS
    static constexpr size_t budget = ((NW == 4 && 3 * slot_bytes + meta_bytes <= 80 * 1024) ? 80 * 1024 : 160 * 1024) - meta_bytes;
    static constexpr int D = budget / slot_bytes >= 6 ? 6 : (int)(budget / slot_bytes);
    static constexpr bool fits = D >= 3;
    static constexpr size_t lds_bytes = D * slot_bytes + meta_bytes;
};

template <int RM, int NWC, int KS, int CG>
__global__ __launch_bounds__(64 * NWC * KS) void gemm_fewrows_kernel(FewRowsArgs g)
{
    using Shape = FewRowsShape<RM, NWC, KS, CG>;
    constexpr int NW = Shape::NW, D = Shape::D;
    constexpr int RB = RM / 16;                   // 16-row blocks
    constexpr int A_INSTR = RM / 4;               // 64-cell loads of A per K part and step (16 cells x RM rows)
    constexpr int IA = (KS * A_INSTR + NW - 1) / NW; // of them per wave
    constexpr int PER = IA + CG;                  // LDS-writing loads per wave and step: A, one of codes per column group
    constexpr int A_PART = 16 * RM;               // cells of A per K part and slot
    constexpr int CODES0 = KS * A_PART;           // first cell of the codes of a slot
    constexpr int WCELLS = 64 * CG;               // cells of codes per wave and step (16 CG rows x 64 bytes), and of a metadata block
    constexpr int SLOT = CODES0 + NW * WCELLS;    // cells per slot
    constexpr int META0 = D * SLOT;               // first cell of the metadata ring: [wave][2 blocks][16 CG rows][4 cells]
    static_assert(Shape::fits && SLOT * 16 == Shape::slot_bytes, "LDS plan");
    static_assert((D - 2) * PER <= 63, "the wait count is a 6-bit field");
    static_assert(RM == 16 || RM == 32, "rows of a tile");
    static_assert(CG == 1 || CG == 2, "column groups of a wave");
    extern __shared__ uint4 lds[];

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int cw = wave % NWC, kw = wave / NWC; // column strip and K part of this wave
    const int col0 = ((int)blockIdx.x * NWC + cw) * 16 * CG;
    const int upr = g.K / 64, np = (upr + 1) / 2; // units per row, pairs of units (steps) in K
    const int ppp = (np + KS - 1) / KS;           // steps per K part; part kw takes pairs [kw ppp, (kw + 1) ppp)
    const int p0 = kw * ppp;
    const bool odd_tail = (upr & 1) != 0;         // the last pair has one unit only

    // ---- load plan.  Every address is a 64-bit scalar base that moves with the step plus a 32-bit byte
    // offset per lane (the host keeps the operands below 4 GiB).  Loads past the end of K repeat the
    // last pair, and the missing second unit of an odd last pair repeats its first: never used, in bounds.
    // W codes, load t of CG: lane -> weight row 16 t + lane / 4, position lane % 4 of the row's four
    // 16-byte chunks, which holds chunk (position ^ swizzle(row)); chunk c = half c % 2 of unit c / 2.
    uint32_t wc_off[CG], wc_off_tail[CG];
#pragma unroll
    for (int t = 0; t < CG; ++t) {
        const int row = 16 * t + lane / 4, c = (lane % 4) ^ ((row >> 2) & 3);
        int col = col0 + row;
        col = col < g.N ? col : g.N - 1;
        wc_off[t] = (uint32_t)col * (uint32_t)(g.K / 2) + 16u * c;
        wc_off_tail[t] = (uint32_t)col * (uint32_t)(g.K / 2) + 16u * (c & 1);
    }
    // W metadata, a block of 16 units at a time (blocks aligned to multiples of 16 units of the row), load t of CG:
    // lane -> weight row 16 t + lane / 4, units 4 (lane % 4) .. + 3 of the block; chunks past the end of the
    // row repeat its last four units
    uint32_t wm_row_off[CG];
#pragma unroll
    for (int t = 0; t < CG; ++t) {
        int col = col0 + 16 * t + lane / 4;
        col = col < g.N ? col : g.N - 1;
        wm_row_off[t] = (uint32_t)col * (uint32_t)upr * 4u;
    }
    // A: load id = wave IA + i covers, for K part id / A_INSTR, the 64 cells (j, row) with
    // j = (id % A_INSTR) (64 / RM) + lane / RM, row = lane % RM; rows past M repeat the last row
    uint32_t a_row_off[IA], a_pair0[IA], a_tail_adj[IA], a_dst[IA];
#pragma unroll
    for (int i = 0; i < IA; ++i) {
        int id = wave * IA + i;
        id = id < KS * A_INSTR ? id : KS * A_INSTR - 1;
        const int part = id / A_INSTR, ai = id % A_INSTR;
        const int j = ai * (64 / RM) + lane / RM;
        int row = lane % RM;
        row = row < g.M ? row : g.M - 1;
        a_row_off[i] = (uint32_t)row * (uint32_t)g.lda * 2u + 16u * j;
        a_pair0[i] = (uint32_t)(part * ppp);
        a_tail_adj[i] = j >= 8 ? 128u : 0u;
        a_dst[i] = (uint32_t)__builtin_amdgcn_readfirstlane((part * A_PART + ai * 64) * 16);
    }
    auto lds_byte_of = [](const void *p) { return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)p; };
    const uint32_t lds0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_byte_of(lds));
    const uint64_t wc_ptr = fr_uniform((uint64_t)(uintptr_t)g.w_codes), wm_ptr = fr_uniform((uint64_t)(uintptr_t)g.w_meta);
    const uint64_t a_ptr = fr_uniform((uint64_t)(uintptr_t)g.a);

    // the loads of step `it` (of every K part, this wave's share of A; of this wave's part, its W) into slot `slot`
    auto issue = [&](int it, int slot) {
        const uint32_t sbase = lds0 + (uint32_t)(slot * SLOT * 16);
#pragma unroll
        for (int i = 0; i < IA; ++i) {
            uint32_t p = a_pair0[i] + (uint32_t)it;
            p = p < (uint32_t)np ? p : (uint32_t)(np - 1);
            uint32_t off = a_row_off[i] + p * 256u;
            if (odd_tail) off -= (2 * p + 1 >= (uint32_t)upr) ? a_tail_adj[i] : 0u;
            fr_load_to_lds_16(a_ptr, off, sbase + a_dst[i]);
        }
        int pw = p0 + it;
        pw = pw < np ? pw : np - 1;
        const bool tail = 2 * pw + 1 >= upr; // wave-uniform
        const uint32_t cdst = sbase + (uint32_t)((CODES0 + wave * WCELLS) * 16);
#pragma unroll
        for (int t = 0; t < CG; ++t) fr_load_to_lds_16(wc_ptr + (uint64_t)pw * 64, tail ? wc_off_tail[t] : wc_off[t], cdst + 1024u * t);
    };
    // the metadata of block `blk` (units 16 blk .. 16 blk + 15 of this wave's rows) into its ring slot blk % 2
    auto issue_meta = [&](int blk) {
        int u4 = 16 * blk + 4 * (lane % 4);
        u4 = u4 < upr - 4 ? u4 : upr - 4;
        const uint32_t dst = lds0 + (uint32_t)((META0 + (wave * 2 + (blk & 1)) * WCELLS) * 16);
#pragma unroll
        for (int t = 0; t < CG; ++t) fr_load_to_lds_16(wm_ptr, wm_row_off[t] + 4u * (uint32_t)u4, dst + 1024u * t);
    };

    // results: acc[cg][rb] is the 16 x 16 tile of column group cg (columns 16 cg .. + 15 of the strip) and row
    // block rb; lane (n, q) = (lane % 16, lane / 16) holds its column n, rows 4 q .. 4 q + 3
    f32x4_t acc[CG][RB];
#pragma unroll
    for (int cg = 0; cg < CG; ++cg)
#pragma unroll
        for (int i = 0; i < RB; ++i) acc[cg][i] = f32x4_t{ 0.f, 0.f, 0.f, 0.f };

    // ---- expansion (hif4_expand_fp8.h): lane (n, q) expands groups of 8 number q (half step 0) and 4 + q (half
    // step 1) of a unit
    const MicroExpShifts mes = micro_exp_shifts(lane / 16);
    auto micro_exponents = [&](uint32_t m) { return micro_exponent_bytes(m, mes); };
    auto expand_dword = [](uint32_t c, uint32_t xb, int hs) { return expand_dword_fp8(c, xb, hs); };
    auto unit_scale = [](uint32_t m) { return unit_scale_f32(m); };

    // Matrix instruction: v_mfma_f32_16x16x32_bf16, half a unit of K each.  Lane (n, q) = (lane % 16, lane / 16)
    // supplies, for half step hs of a unit, group of 8 number 4 hs + q of both operands: of row n of a 16-row
    // block of A, and of weight rows n and 16 + n of the strip (two column groups).  Codes live in LDS as
    // cell(row, chunk) = 4 row + (chunk ^ swizzle(row)) (see the load plan): the 64 dword reads of a wave
    // fall on 64 different banks.
    const int n16 = lane % 16, q = lane / 16;
    const int wswz = (n16 >> 2) & 3; // swizzle of rows n and 16 + n alike
    const f32x4_t zero4 = { 0.f, 0.f, 0.f, 0.f };

    // matrix work of the pair in slot `slot` (a compile-time number: every LDS address of the step is then a lane
    // constant plus an immediate offset).  Every LDS read of the step is requested up front, so that the read latency
    // is covered by arithmetic the wave has anyway.  TWO: the pair has both units (all pairs but the last of an odd K/64).
    auto compute = [&](auto slot_c, int pair, auto two_c) {
        constexpr int slot = decltype(slot_c)::value;
        constexpr bool TWO = decltype(two_c)::value;
        constexpr int NU = TWO ? 2 : 1;
        const uint4 *sl = lds + slot * SLOT;
        const int u0 = 2 * pair; // the pair's first unit; both units lie in metadata block u0 / 16
        const uint32_t *mring = reinterpret_cast<const uint32_t *>(lds + META0 + (wave * 2 + ((u0 >> 4) & 1)) * WCELLS) + (u0 & 15);
        uint2 mm[CG];       // metadata of the pair's units, per column group
        uint32_t cd[CG][2][2]; // codes dword [column group][unit][half step]
        const uint32_t *cbase = reinterpret_cast<const uint32_t *>(sl + CODES0 + wave * WCELLS) + q;
#pragma unroll
        for (int cg = 0; cg < CG; ++cg) {
            mm[cg] = *reinterpret_cast<const uint2 *>(mring + (16 * cg + n16) * 16);
#pragma unroll
            for (int uu = 0; uu < NU; ++uu)
#pragma unroll
                for (int hs = 0; hs < 2; ++hs) cd[cg][uu][hs] = cbase[(64 * cg + 4 * n16 + ((2 * uu + hs) ^ wswz)) * 4];
        }
        uint4 av[2][2][RB]; // A operands [unit][half step][row block]
#pragma unroll
        for (int uu = 0; uu < NU; ++uu)
#pragma unroll
            for (int hs = 0; hs < 2; ++hs)
#pragma unroll
                for (int i = 0; i < RB; ++i) av[uu][hs][i] = sl[kw * A_PART + (uu * 8 + 4 * hs + q) * RM + i * 16 + n16];
        __builtin_amdgcn_sched_barrier(0);
        f32x4_t part[2][CG][RB]; // the units' own sums [unit][column group][row block]
#pragma unroll
        for (int uu = 0; uu < NU; ++uu) {
            uint32_t xb[CG];
#pragma unroll
            for (int cg = 0; cg < CG; ++cg) xb[cg] = micro_exponents(uu == 0 ? mm[cg].x : mm[cg].y);
#pragma unroll
            for (int hs = 0; hs < 2; ++hs)
#pragma unroll
                for (int cg = 0; cg < CG; ++cg) {
                    const uint4 b = expand_dword(cd[cg][uu][hs], xb[cg], hs);
#pragma unroll
                    for (int i = 0; i < RB; ++i)
                        part[uu][cg][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[uu][hs][i]), __builtin_bit_cast(bf16x8_t, b),
                                                                                   hs == 0 ? zero4 : part[uu][cg][i], 0, 0, 0);
                }
        }
        // the units' sums times their E6M2 factors (the first unit's have long left the matrix pipeline)
#pragma unroll
        for (int uu = 0; uu < NU; ++uu) {
#pragma unroll
            for (int cg = 0; cg < CG; ++cg) {
                const float sc = unit_scale(uu == 0 ? mm[cg].x : mm[cg].y);
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[cg][i][r] = __builtin_fmaf(part[uu][cg][i][r], sc, acc[cg][i][r]);
            }
        }
    };

    // ---- pipeline: step `it` is issued D - 1 steps ahead of its matrix work; the two metadata blocks the part
    // starts in come first, block b + 1 follows when the part enters block b.  The loop is unrolled over the D slots
    // of the ring, so that a step's slot is a compile-time number.
    int blk = (2 * p0) >> 4;
    issue_meta(blk);
    issue_meta(blk + 1);
#pragma unroll
    for (int it = 0; it < D - 1; ++it) issue(it, it);
    auto step = [&](int it, auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
        // the loads of step `it` have landed once only younger ones (those of D - 2 steps, at least) are in flight
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"((D - 2) * PER) : "memory");
        __syncthreads(); // every wave's share of A(it) is there, and every wave is through with the slot refilled next
        const int nblk = (2 * (p0 + it)) >> 4;
        if (nblk != blk) { // wave-uniform: block nblk - 1 is used up, its ring slot takes block nblk + 1
            blk = nblk;
            issue_meta(blk + 1);
        }
        issue(it + D - 1, slot == 0 ? D - 1 : slot - 1);
        const int pair = p0 + it;
        if (pair >= np) return;                       // wave-uniform: a K part past the end of K
        if (2 * pair + 1 < upr) compute(slot_c, pair, std::true_type{}); // wave-uniform
        else compute(slot_c, pair, std::false_type{});
    };
    for (int it0 = 0; it0 < ppp; it0 += D) {
        step(it0, std::integral_constant<int, 0>{});
        if (it0 + 1 < ppp) step(it0 + 1, std::integral_constant<int, 1>{});
        if (it0 + 2 < ppp) step(it0 + 2, std::integral_constant<int, 2>{});
        if constexpr (D > 3) { if (it0 + 3 < ppp) step(it0 + 3, std::integral_constant<int, 3>{}); }
        if constexpr (D > 4) { if (it0 + 4 < ppp) step(it0 + 4, std::integral_constant<int, 4>{}); }
        if constexpr (D > 5) { if (it0 + 5 < ppp) step(it0 + 5, std::integral_constant<int, 5>{}); }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // no load may outlive the workgroup's LDS

    // ---- the partial sums of K parts 1 .. KS - 1 go through LDS to part 0, lane for lane, in a fixed order
    if constexpr (KS > 1) {
        static_assert((size_t)(KS - 1) * NWC * CG * RB * 1024 <= Shape::lds_bytes, "partial sums fit the buffers");
        f32x4_t *red = reinterpret_cast<f32x4_t *>(lds); // [kw - 1][cw][column group][row block][lane]
        __syncthreads();
        if (kw > 0) {
            f32x4_t *dst = red + (size_t)((kw - 1) * NWC + cw) * CG * RB * 64 + lane;
#pragma unroll
            for (int cg = 0; cg < CG; ++cg)
#pragma unroll
                for (int i = 0; i < RB; ++i) dst[(cg * RB + i) * 64] = acc[cg][i];
        }
        __syncthreads();
        if (kw > 0) return;
#pragma unroll
        for (int p = 0; p < KS - 1; ++p) {
            const f32x4_t *src = red + (size_t)(p * NWC + cw) * CG * RB * 64 + lane;
#pragma unroll
            for (int cg = 0; cg < CG; ++cg)
#pragma unroll
                for (int i = 0; i < RB; ++i) acc[cg][i] += src[(cg * RB + i) * 64];
        }
    }

    // ---- epilogue: lane (n, q) holds column n of each 16 x 16 tile, rows 4 q + r
#pragma unroll
    for (int cg = 0; cg < CG; ++cg) {
        const int col = col0 + 16 * cg + n16;
        if (col >= g.N) continue;
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = i * 16 + 4 * q + r;
                if (row < g.M) {
                    const float v = acc[cg][i][r];
                    if (g.out_f32) static_cast<float *>(g.c)[(int64_t)row * g.ldc + col] = v;
                    else static_cast<uint16_t *>(g.c)[(int64_t)row * g.ldc + col] = (uint16_t)((f2u(v) + 0x7FFFu + ((f2u(v) >> 16) & 1u)) >> 16);
                }
            }
    }
}

// ------------------------------------------------------------------ launch

namespace {

struct FewRowsChoice {
    int nwc, ks, cg;
};

// The shapes a workgroup can take: (column strips, K parts, column groups of 16 per strip).  Strips of 16 columns
// give twice as many strips to spread over the chip and over K; strips of 32 share each A operand between two MFMAs.
#ifndef HIF4_FR_SHAPES
#define HIF4_FR_SHAPES(X) X(7, 2, 1) X(3, 4, 1) X(2, 4, 1) X(4, 2, 1) X(4, 2, 2)
#endif

// Which of them a call takes.  The kernel is bound by the vector instructions of the expansion, which a SIMD
// issues for its waves in turn, so time is modelled as rounds of workgroups over the chip's 256 CUs times the
// waves a SIMD holds times the weights of a wave: its column groups times its steps of K, plus 8 steps for
// starting a workgroup, filling its pipeline and the final reduction (fitted to measurements of thirteen shapes,
// those of the list among them, on ten weight matrices from 2048 x 7168 to 28672 x 8192: the choice is the fastest
// or within 6 % of it; the shapes the model never picks from 6144 columns on are no longer compiled);
// among equals, the earlier entry of the list.  Only shapes whose LDS plan fits are offered (the arithmetic mirrors
// FewRowsShape).
template <int RM>
FewRowsChoice fewrows_choose(int64_t N, int64_t K)
{
    const int64_t np = (K / 64 + 1) / 2;
#define HIF4_FR_ENTRY(W, S, G) { W, S, G },
    const FewRowsChoice cand[] = { HIF4_FR_SHAPES(HIF4_FR_ENTRY) };
#undef HIF4_FR_ENTRY
    FewRowsChoice best = cand[0];
    double best_t = 1e300;
    for (const FewRowsChoice &c : cand) {
        const int nw = c.nwc * c.ks;
        const size_t slot = (size_t)c.ks * 16 * RM * 16 + (size_t)nw * c.cg * 1024, meta = (size_t)nw * 2 * c.cg * 1024;
        const bool half_lds = nw == 4 && 3 * slot + meta <= 80 * 1024;
        const size_t budget = (half_lds ? 80 * 1024 : 160 * 1024) - meta;
        if (budget / slot < 3) continue;
        const int64_t per_cu = half_lds ? 2 : 1;
        const int64_t strips = (N + 16 * c.cg - 1) / (16 * c.cg);
        const int64_t wgs = (strips + c.nwc - 1) / c.nwc;
        const int64_t rounds = (wgs + 256 * per_cu - 1) / (256 * per_cu);
        const int64_t steps = (np + c.ks - 1) / c.ks;
        // (a second round costs more than its share: the tail of the first leaves compute units idle)
        const double t = (double)rounds * (1.0 + 0.05 * (double)(rounds - 1)) * (double)(per_cu * nw) / 4.0 * c.cg * (double)(steps + 8);
        if (t < best_t) best = c, best_t = t;
    }
    return best;
}

template <int RM, int NWC, int KS, int CG>
int launch_fewrows_t(const FewRowsArgs &g, hipStream_t stream)
{
    using Shape = FewRowsShape<RM, NWC, KS, CG>;
    if constexpr (!Shape::fits) {
        return HIF4_ERR_UNSUPPORTED;
    } else {
        auto k = gemm_fewrows_kernel<RM, NWC, KS, CG>;
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)Shape::lds_bytes) != hipSuccess)
            return HIF4_ERR_DEVICE;
        const dim3 grid((unsigned)((g.N + 16 * CG * NWC - 1) / (16 * CG * NWC))), block(64 * NWC * KS);
        hipLaunchKernelGGL(k, grid, block, Shape::lds_bytes, stream, g);
        return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
    }
}

template <int RM>
int launch_fewrows_rm(const FewRowsArgs &g, hipStream_t stream)
{
    const FewRowsChoice c = fewrows_choose<RM>(g.N, g.K);
#define HIF4_FR_CASE(W, S, G) if (c.nwc == W && c.ks == S && c.cg == G) return launch_fewrows_t<RM, W, S, G>(g, stream);
    HIF4_FR_SHAPES(HIF4_FR_CASE)
#undef HIF4_FR_CASE
    return HIF4_ERR_UNSUPPORTED;
}

} // namespace

// The kernel addresses each operand as a scalar base plus a 32-bit byte offset per lane.
bool fewrows_fits(int64_t M, int64_t N, int64_t K, int64_t lda)
{
    return M >= 1 && M <= 32 && K >= 256 && K % 256 == 0 && N * (K / 2) < ((int64_t)1 << 32) && M * lda * 2 < ((int64_t)1 << 32);
}

// a: BF16 rows in natural element order (row stride lda elements, 16-byte aligned rows).
int launch_gemm_fewrows(const void *a, int64_t lda, const uint8_t *w_codes, const uint32_t *w_meta, int64_t M, int64_t N, int64_t K,
                        void *c, int64_t ldc, int out_dtype, hipStream_t stream)
{
    FewRowsArgs g;
    g.a = a;
    g.lda = lda;
    g.w_codes = w_codes;
    g.w_meta = w_meta;
    g.c = c;
    g.ldc = ldc;
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    g.out_f32 = out_dtype == HIF4_OUT_F32;
    if (M <= 16) return launch_fewrows_rm<16>(g, stream);
    return launch_fewrows_rm<32>(g, stream);
}

} // namespace hif4
