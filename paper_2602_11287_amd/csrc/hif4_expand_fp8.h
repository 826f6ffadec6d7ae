// Expansion of packed HiF4 weights for the kernels that meet few rows (token generation): Eq. 2 of the HiF4 paper
// (Section II-A) without its E6M2 factor, which those kernels apply to the partial sums of a unit instead, as the
// factored form of Eq. 4 (Section III-B) has it.
//
// The 3-bit magnitude of four codes goes through one v_perm_b32 with the FP8 (E4M3) patterns of 0..7 as its byte
// table, the sign bits are OR-ed in, and v_cvt_scalef32_pk_bf16_fp8 turns two such bytes into two BF16 values times
// 2^(E1_8 + E1_16), the power of two riding in the exponent of its scale operand (zero stays zero, which a table of
// BF16 patterns with the exponent added afterwards would not give).
#pragma once
#include "hif4_common.h"

namespace hif4 {

// E4M3 patterns of the integers 0..7 (bias 7: 1 = 0x38, 2 = 0x40, 3 = 0x44, ...), the byte table of v_perm_b32
constexpr uint32_t FP8_OF_0123 = 0x44403800u, FP8_OF_4567 = 0x4E4C4A48u;

// byte B of x, shifted into the exponent field of an fp32 pattern: one instruction (the operand's byte select does the
// extraction; the shift amount has to sit in a register for this encoding)
template <int B>
__device__ __forceinline__ uint32_t byte_shl23(uint32_t x)
{
    static_assert(B == 1 || B == 2, "bytes 0 and 3 need no extraction");
    uint32_t r;
    if (B == 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(23u), "v"(x));
    else asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(23u), "v"(x));
    return r;
}

// The powers of two of a unit's micro-exponents, as a lane needs them that expands groups of 8 number q (half step 0)
// and 4 + q (half step 1): E1_8 bits q and 4 + q and E1_16 bits 2 q, 2 q + 1, 8 + 2 q, 9 + 2 q of the metadata word m.
// Result: the biased exponents 127 + E1_8 + E1_16 of 2^(E1_8 + E1_16) as four bytes - byte 0: half step 0, elements
// 0..3 of the group; byte 1: half step 1, elements 0..3; byte 2: half step 0, elements 4..7; byte 3: half step 1,
// elements 4..7 - by arithmetic on all four at once (a multiplication spreads the bits).
struct MicroExpShifts {
    uint32_t sh16, sh8, sh8b;
};
__device__ __forceinline__ MicroExpShifts micro_exp_shifts(int q) { return { 16u + 2u * (uint32_t)q, 8u + (uint32_t)q, 12u + (uint32_t)q }; }

__device__ __forceinline__ uint32_t micro_exponent_bytes(uint32_t m, const MicroExpShifts &s)
{
    const uint32_t t = __builtin_amdgcn_ubfe(m, s.sh16, 10);          // bits 0, 1, 8, 9 are the four E1_16 bits
    const uint32_t s16 = __umul24(t, 0x8001u) & 0x01010101u;          // bit 0 -> 0, 1 -> 16, 8 -> 8, 9 -> 24
    const uint32_t e = __builtin_amdgcn_ubfe(m, s.sh8, 1) | (__builtin_amdgcn_ubfe(m, s.sh8b, 1) << 8); // E1_8 of the two groups
    return s16 + __umul24(e, 0x10001u) + 0x7F7F7F7Fu;                 // no carries: every byte is 127 .. 129
}

// One dword of codes (group of 8 number j = 4 hs + q of its unit) -> one MFMA operand of 8 BF16: S1P2 magnitude times
// sign times 2^(E1_8 + E1_16), natural element order.  xb: micro_exponent_bytes() of the unit.  The conversion
// instruction reads the exponent field of its scale operand only, so whatever a shift leaves in the low 23 bits does
// not matter; the sign bit stays clear.
__device__ __forceinline__ uint4 expand_dword_fp8(uint32_t c, uint32_t xb, int hs)
{
    const float sa = u2f(hs == 0 ? xb << 23 : byte_shl23<1>(xb));    // elements 0..3
    const float sb = u2f(hs == 0 ? byte_shl23<2>(xb) : xb >> 1);     // elements 4..7
    const uint32_t lo = c & 0x07070707u, hi = (c >> 4) & 0x07070707u; // magnitudes, one per byte
    const uint32_t f8lo = or_and(__builtin_amdgcn_perm(FP8_OF_4567, FP8_OF_0123, lo), c << 4, 0x80808080u);
    const uint32_t f8hi = or_and(__builtin_amdgcn_perm(FP8_OF_4567, FP8_OF_0123, hi), c, 0x80808080u);
    uint4 b;
    b.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(f8lo, sa, false));
    b.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(f8lo, sa, true));
    b.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(f8hi, sb, false));
    b.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(f8hi, sb, true));
    return b;
}

// fp32 value of the unit scale (4 + M) 2^(E - 48 - 4) (codes count quarters, E6M2 = (1 + M / 4) 2^(E - 48)); NaN unit: NaN
__device__ __forceinline__ float unit_scale_f32(uint32_t m)
{
    const uint32_t s = ((((m >> 2) & 0x3Fu) + (127u - 50u)) << 23) | ((m & 3u) << 21);
    return u2f((m & 0xFFu) == 0xFFu ? 0x7FC00000u : s);
}

} // namespace hif4
