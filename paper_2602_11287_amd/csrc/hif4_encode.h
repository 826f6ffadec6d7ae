// Algorithm 1 of the HiF4 paper (Section II-B) for the share of a unit that one lane holds:
// the arithmetic of the encoder, shared by the streaming encoder kernel and by the GEMM
// epilogue that writes its result as HiF4.
#pragma once
#include "hif4_common.h"

namespace hif4 {

// ------------------------------------------------------------------ rounding steps

// fp32 -> BF16 pattern, for a product that is exact in fp32.
template <int MODE>
__device__ __forceinline__ uint32_t round_bf16(float f)
{
    uint32_t u = f2u(f);
    if (MODE == HIF4_ROUND_RNE) return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return (u + 0x8000u) >> 16; // half away from zero acts on the magnitude bits
}

// Two exact fp32 products -> packed BF16 pair (first in the low half).
template <int MODE>
__device__ __forceinline__ uint32_t round_bf16_pair(float lo, float hi)
{
    if (MODE == HIF4_ROUND_RNE) {
        f32x2_t v = { lo, hi };
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t)); // v_cvt_pk_bf16_f32
    }
    return ((f2u(lo) + 0x8000u) >> 16) | ((f2u(hi) + 0x8000u) & 0xFFFF0000u);
}

// BF16_to_E6M2: keep two mantissa bits, carry into the exponent, rebias 127 -> 48,
// saturate to [0x00, 0xFE].
template <int MODE>
__device__ __forceinline__ uint32_t bf16_to_e6m2(uint32_t sfb)
{
    uint32_t q = (sfb + (MODE == HIF4_ROUND_RNE ? 0xFu + ((sfb >> 5) & 1u) : 0x10u)) >> 5;
    int e = (int)q - ((127 - 48) << 2);
    e = e < 0 ? 0 : e;
    return (uint32_t)(e > 0xFE ? 0xFE : e);
}

// E6M2_REC_to_BF16 as an fp32 pattern: table on the mantissa, exponent subtraction.
__device__ __forceinline__ float e6m2_reciprocal(uint32_t e6)
{
    uint32_t M = e6 & 3u;
    uint32_t expf = 175u - (e6 >> 2) - (M ? 1u : 0u);
    uint32_t mant = (0x122B4D00u >> (8u * M)) & 0xFFu; // 1/1, 1/1.25, 1/1.5, 1/1.75 to 7 bits
    return u2f((expf << 23) | (mant << 16));
}

// Algorithm 1 for the share of one unit that this lane holds (NCH chunks of 8 elements,
// chunk c being group-of-8 number c*LPU + l of the unit).  Returns the packed codes of
// the lane's chunks and the complete metadata word.
template <int LPU, int MODE>
__device__ __forceinline__ uint32_t encode_share(const uint4 (&w)[8 / LPU], int l, uint32_t (&out)[8 / LPU])
{
    constexpr int NCH = 8 / LPU; // chunks of 8 elements per lane

    // Stage 1: peak magnitudes as BF16 patterns (they order like unsigned integers).
    uint32_t am[NCH][4]; // |x| pairs, reused by stage 3
    uint32_t v16a[NCH], v16b[NCH], v8[NCH];
    uint32_t vmax = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        am[c][0] = w[c].x & 0x7FFF7FFFu;
        am[c][1] = w[c].y & 0x7FFF7FFFu;
        am[c][2] = w[c].z & 0x7FFF7FFFu;
        am[c][3] = w[c].w & 0x7FFF7FFFu;
#pragma unroll
        for (int t = 0; t < 4; ++t) asm volatile("" : "+v"(am[c][t])); // keep the masked value, do not re-derive it
        const uint32_t m01 = pk_max_u16(am[c][0], am[c][1]);
        const uint32_t m23 = pk_max_u16(am[c][2], am[c][3]);
        v16a[c] = umax(m01 & 0xFFFFu, m01 >> 16);
        v16b[c] = umax(m23 & 0xFFFFu, m23 >> 16);
        v8[c] = umax(v16a[c], v16b[c]);
        vmax = umax(vmax, v8[c]);
    }
    vmax = umax(vmax, dpp<DPP_XOR1>(vmax));
    if (LPU >= 4) vmax = umax(vmax, dpp<DPP_XOR2>(vmax));
    if (LPU >= 8) vmax = umax(vmax, dpp<DPP_HALF_MIRROR>(vmax));
    const bool special = vmax >= 0x7F80u; // an Inf or NaN somewhere in the unit

    // Stage 2: level-1 scale and its reciprocal.
    const uint32_t sfb = round_bf16<MODE>(u2f(vmax << 16) * u2f(0x3E120000u)); // Vmax * (1/7)_BF16
    const uint32_t e6 = bf16_to_e6m2<MODE>(sfb);
    const float rec = e6m2_reciprocal(e6);

    // BF16(V * REC) >= 4 holds exactly when V >= 4 * E6M2 (the product 4 * E6M2 * REC is at or
    // above the rounding boundary 4 - 2^-7 for each of the four table entries, the BF16 just
    // below 4 * E6M2 falls under it, and rounding is monotone), likewise for 2: the
    // multiply-compare steps become integer compares of BF16 patterns.
    const uint32_t S = (e6 << 5) + (79u << 7); // BF16 pattern of the E6M2 value
    const uint32_t thr2 = S + 0x80u, thr4 = S + 0x100u;

    // Rebias constants for the three possible divisors 2^0, 2^1, 2^2 (see stage 3 below).
    constexpr uint32_t RB0 = 0x38003800u, RBSTEP = 0x00800080u;

    uint32_t mbits = 0; // this lane's share of E1_8 (bits 8..15) and E1_16 (bits 16..31)
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int j = c * LPU + l; // index of this group of 8 inside the unit
        const bool b8 = v8[c] >= thr4;
        const uint32_t thr16 = b8 ? thr4 : thr2; // V16 * REC * 2^-E1_8 >= 2
        const bool ba = v16a[c] >= thr16, bb = v16b[c] >= thr16;
        mbits |= ((b8 ? 1u : 0u) << (8 + j)) | (((ba ? 1u : 0u) | (bb ? 2u : 0u)) << (16 + 2 * j));

        // Stage 3: scale, round to BF16, divide by 2^(E1_8+E1_16), clamp, round to S1P2.
        // Magnitudes only: the sign bits are copied from the inputs further down.
        uint32_t mag0, mag1; // byte t of mag0 = magnitude of element t, of mag1 = element 4 + t
        if (MODE == HIF4_ROUND_RNE) {
            // Packed fp16 arithmetic, two elements per instruction.  A BF16 magnitude p (8
            // significant bits) divided by 2^sh and clamped to 1.75 is exact in fp16: subtract
            // (112 + sh) << 7 from the pattern with saturation (exponent rebias 127 -> 15 and the
            // division; patterns below 2^(sh-14) become 0 or tiny, far under the first rounding
            // boundary 0.125), clamp to the rebiased 1.75, move the 7 mantissa bits up by 3.
            // 384 = 1.5 * 2^8 has an fp16 ulp of 0.25: adding it rounds to the S1P2 grid with
            // ties to even and leaves the count of quarter steps in the low mantissa bits.
            const uint32_t rb_lo = b8 ? RB0 + RBSTEP : RB0, rb_hi = b8 ? RB0 + 2 * RBSTEP : RB0 + RBSTEP;
            const uint32_t rba = ba ? rb_hi : rb_lo, rbb = bb ? rb_hi : rb_lo;
            uint32_t r[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t a = am[c][t];
                const uint32_t P = round_bf16_pair<MODE>(u2f(a << 16) * rec, u2f(a & 0xFFFF0000u) * rec);
                const uint32_t H = pk_shl3_u16(pk_min_u16(pk_sub_sat_u16(P, t < 2 ? rba : rbb), 0x07E007E0u));
                r[t] = pk_add_f16(H, 0x5E005E00u);
            }
            mag0 = __builtin_amdgcn_perm(r[1], r[0], 0x06040200u);
            mag1 = __builtin_amdgcn_perm(r[3], r[2], 0x06040200u);
        } else {
            const uint32_t sha = (b8 ? 1u : 0u) + (ba ? 1u : 0u), shb = (b8 ? 1u : 0u) + (bb ? 1u : 0u);
            const uint32_t ca = (0x3FE0u + (sha << 7)) * 0x00010001u; // BF16 pair of 1.75 * 2^sh
            const uint32_t cb = (0x3FE0u + (shb << 7)) * 0x00010001u;
            const float sa = u2f(0x40800000u - (sha << 23)), sb = u2f(0x40800000u - (shb << 23)); // 2^(2-sh)
            uint32_t r[8];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t a = am[c][t];
                const uint32_t P = round_bf16_pair<MODE>(u2f(a << 16) * rec, u2f(a & 0xFFFF0000u) * rec);
                const uint32_t Pc = pk_min_u16(P, t < 2 ? ca : cb); // patterns order like integers
                // truncation of t * 4 + 0.5 rounds half away from zero
                r[2 * t] = (uint32_t)__builtin_fmaf(u2f(Pc << 16), t < 2 ? sa : sb, 0.5f);
                r[2 * t + 1] = (uint32_t)__builtin_fmaf(u2f(Pc & 0xFFFF0000u), t < 2 ? sa : sb, 0.5f);
            }
            mag0 = __builtin_amdgcn_perm(r[1], r[0], 0x0C0C0400u) | __builtin_amdgcn_perm(r[3], r[2], 0x04000C0Cu);
            mag1 = __builtin_amdgcn_perm(r[5], r[4], 0x0C0C0400u) | __builtin_amdgcn_perm(r[7], r[6], 0x04000C0Cu);
        }
        const uint32_t ww[4] = { w[c].x, w[c].y, w[c].z, w[c].w };
        // sign bits: top bit of each BF16 -> bit 3 of the element's byte
        const uint32_t b0 = or_and(mag0, __builtin_amdgcn_perm(ww[1], ww[0], 0x07050301u) >> 4, 0x08080808u);
        const uint32_t b1 = or_and(mag1, __builtin_amdgcn_perm(ww[3], ww[2], 0x07050301u) >> 4, 0x08080808u);
        // byte t of the chunk: element t in the low nibble, element 4 + t in the high nibble
        out[c] = special ? 0u : (b0 | (b1 << 4));
    }

    // Collect the metadata bits of the LPU lanes; every lane ends up with all of them.
    mbits |= dpp<DPP_XOR1>(mbits);
    if (LPU >= 4) mbits |= dpp<DPP_XOR2>(mbits);
    if (LPU >= 8) mbits |= dpp<DPP_HALF_MIRROR>(mbits);

    return special ? 0x000000FFu : (mbits | e6);
}

} // namespace hif4
