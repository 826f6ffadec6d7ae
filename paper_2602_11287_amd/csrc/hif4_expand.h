// Expansion of packed HiF4 code words to BF16 (Eq. 2 of the HiF4 paper, Section II-A),
// shared by the decoder and the GEMM kernels.
#pragma once
#include "hif4_common.h"

namespace hif4 {

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

// Eq. 2 for 8 consecutive elements: group-of-8 number j of a unit with metadata m,
// codes dword c (byte t: element t low nibble, element 4+t high nibble) -> 16 bytes of BF16.
__device__ __forceinline__ uint4 decode_chunk(uint32_t c, uint32_t m, int j)
{
    if ((m & 0xFFu) == 0xFFu) return make_uint4(0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u);
    // value = (4 + M) * mag * 2^(E - 48 - 4 + E1_8 + E1_16): at most 6 significant bits, exact.
    // (4 + M) * 2^x as an fp32 pattern: exponent x + 2, mantissa M in the top two bits.
    const uint32_t e8 = (m >> (8 + j)) & 1u;
    const uint32_t e16a = (m >> (16 + 2 * j)) & 1u, e16b = (m >> (17 + 2 * j)) & 1u;
    const uint32_t sbase = ((((m >> 2) & 0x3Fu) + (127u - 50u) + e8) << 23) | ((m & 3u) << 21);
    const float sa = u2f(sbase + (e16a << 23)), sb = u2f(sbase + (e16b << 23));
    const uint32_t lo = c & 0x07070707u, hi = (c >> 4) & 0x07070707u; // magnitudes of elements 0..3 / 4..7
    const uint32_t sl = (c << 4) & 0x80808080u, sh = c & 0x80808080u; // their signs, bit 7 of each byte
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
        // exact values: their BF16 form is the top half of the fp32 pattern
        const uint32_t pair = __builtin_amdgcn_perm(f2u(f[2 * t + 1]), f2u(f[2 * t]), 0x07060302u);
        // sign bytes of elements 2t, 2t+1 -> bits 15 and 31
        const uint32_t sg = __builtin_amdgcn_perm(0u, t < 2 ? sl : sh, (t & 1) ? 0x030C020Cu : 0x010C000Cu);
        r[t] = pair | sg;
    }
    return make_uint4(r[0], r[1], r[2], r[3]);
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

} // namespace hif4
