// HiF4 encoder (Algorithm 1, Section II-B of the HiF4 paper) and decoder (Eq. 2,
// Section II-A) for gfx950.  Both are HBM-bound streaming kernels: 128 B of BF16
// against 36 B of packed unit.
//
// Work split: a unit of 64 elements is shared by LPU adjacent lanes; every lane owns
// 8/LPU "chunks" of 8 consecutive elements (one 128-bit load each, one level-2
// micro-exponent domain, two level-3 domains).  The peak magnitude of the unit and
// the metadata bits are exchanged across the LPU lanes with DPP moves; nothing goes
// through LDS.
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

// Scaled magnitude (BF16 value held in the top half of an fp32 pattern, sign
// cleared) -> S1P2 magnitude 0..7 after division by 2^sh.
//   clampc = pattern of 1.75 * 2^sh, scale = 2^-sh (RNE) or 2^(2-sh) (RHA).
template <int MODE>
__device__ __forceinline__ uint32_t s1p2_magnitude(uint32_t abits, uint32_t clampc, float scale)
{
    float t = u2f(umin(abits, clampc)); // positive patterns order like integers
    if (MODE == HIF4_ROUND_RNE) {
        // 1.5 * 2^21 has an ulp of 0.25: the add rounds to the S1P2 grid, ties to even
        return f2u(__builtin_fmaf(t, scale, 3145728.0f)) & 7u;
    }
    return (uint32_t)__builtin_fmaf(t, scale, 0.5f); // truncation of x*4 + 0.5
}

// ------------------------------------------------------------------ encoder

template <int LPU, int MODE, bool CONTIG>
__global__ __launch_bounds__(256) void encode_kernel(const uint16_t *__restrict__ x, int64_t units, int64_t upr,
                                                     int64_t ldx, uint32_t *__restrict__ codes,
                                                     uint32_t *__restrict__ meta)
{
    constexpr int NCH = 8 / LPU; // chunks of 8 elements per lane
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t unit_raw = tid / LPU;
    const int l = (int)(tid % LPU);
    const bool live = unit_raw < units;
    const int64_t unit = live ? unit_raw : units - 1; // dead lanes redo the last unit, store nothing

    const uint16_t *src;
    if (CONTIG) {
        src = x + unit * 64;
    } else {
        const int64_t row = unit / upr;
        src = x + row * ldx + (unit - row * upr) * 64;
    }

    uint4 w[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) w[c] = *reinterpret_cast<const uint4 *>(src + 8 * (c * LPU + l));

    // Stage 1: peak magnitudes as BF16 patterns (they order like unsigned integers).
    uint32_t v16a[NCH], v16b[NCH], v8[NCH];
    uint32_t vmax = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const uint32_t m01 = pk_max_u16(w[c].x & 0x7FFF7FFFu, w[c].y & 0x7FFF7FFFu);
        const uint32_t m23 = pk_max_u16(w[c].z & 0x7FFF7FFFu, w[c].w & 0x7FFF7FFFu);
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

    uint32_t mbits = 0; // this lane's share of E1_8 (bits 8..15) and E1_16 (bits 16..31)
    uint32_t out[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int j = c * LPU + l; // index of this group of 8 inside the unit
        const uint32_t p8 = round_bf16<MODE>(u2f(v8[c] << 16) * rec);
        const uint32_t pa = round_bf16<MODE>(u2f(v16a[c] << 16) * rec);
        const uint32_t pb = round_bf16<MODE>(u2f(v16b[c] << 16) * rec);
        const uint32_t e8 = p8 >= 0x4080u ? 1u : 0u;                         // >= 4
        const uint32_t e16a = (int)pa - (int)(e8 << 7) >= 0x4000 ? 1u : 0u;  // * 2^-E1_8 >= 2
        const uint32_t e16b = (int)pb - (int)(e8 << 7) >= 0x4000 ? 1u : 0u;
        mbits |= (e8 << (8 + j)) | (e16a << (16 + 2 * j)) | (e16b << (17 + 2 * j));

        // Stage 3: scale, round to BF16, divide by 2^(E1_8+E1_16), round to S1P2.
        const uint32_t sha = e8 + e16a, shb = e8 + e16b;
        const uint32_t base = MODE == HIF4_ROUND_RNE ? 0x3F800000u : 0x40800000u; // 1 or 4
        const uint32_t ca = 0x3FE00000u + (sha << 23), cb = 0x3FE00000u + (shb << 23);
        const float sa = u2f(base - (sha << 23)), sb = u2f(base - (shb << 23));
        const uint32_t ww[4] = { w[c].x, w[c].y, w[c].z, w[c].w };
        uint32_t mag[2]; // byte t of mag[h] = magnitude of element 4h + t
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t cc = h ? cb : ca;
            const float ss = h ? sb : sa;
            uint32_t acc = 0;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t d = ww[2 * h + t];
                const uint32_t P = round_bf16_pair<MODE>(u2f(d << 16) * rec, u2f(d & 0xFFFF0000u) * rec);
                const uint32_t m_lo = s1p2_magnitude<MODE>((P << 16) & 0x7FFFFFFFu, cc, ss);
                const uint32_t m_hi = s1p2_magnitude<MODE>(P & 0x7FFF0000u, cc, ss);
                acc |= (m_lo | (m_hi << 8)) << (16 * t);
            }
            mag[h] = acc;
        }
        // sign bits: top bit of each BF16 -> bit 3 of the element's byte
        const uint32_t s0 = (__builtin_amdgcn_perm(ww[1], ww[0], 0x07050301u) >> 4) & 0x08080808u;
        const uint32_t s1 = (__builtin_amdgcn_perm(ww[3], ww[2], 0x07050301u) >> 4) & 0x08080808u;
        const uint32_t b0 = mag[0] | s0, b1 = mag[1] | s1;
        // bytes -> nibbles: byte0|byte1<<4 lands in byte 0, byte2|byte3<<4 in byte 2
        const uint32_t n0 = b0 | (b0 >> 4), n1 = b1 | (b1 >> 4);
        out[c] = special ? 0u : __builtin_amdgcn_perm(n1, n0, 0x06040200u);
    }

    // Collect the metadata bits of the LPU lanes; every lane ends up with all of them.
    mbits |= dpp<DPP_XOR1>(mbits);
    if (LPU >= 4) mbits |= dpp<DPP_XOR2>(mbits);
    if (LPU >= 8) mbits |= dpp<DPP_HALF_MIRROR>(mbits);

    if (live) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) codes[unit * 8 + c * LPU + l] = out[c];
        if (l == 0) meta[unit] = special ? 0x000000FFu : (mbits | e6);
    }
}

// ------------------------------------------------------------------ decoder

// One lane decodes 8 consecutive elements: a dword of codes -> 16 bytes of BF16.
template <bool CONTIG>
__global__ __launch_bounds__(256) void decode_kernel(const uint32_t *__restrict__ codes,
                                                     const uint32_t *__restrict__ meta, int64_t chunks, int64_t upr,
                                                     int64_t ldy, uint16_t *__restrict__ y)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= chunks) return;
    const int64_t unit = tid >> 3;
    const int j = (int)(tid & 7);
    const uint32_t c = codes[tid];
    const uint32_t m = meta[unit];

    uint16_t *dst;
    if (CONTIG) {
        dst = y + tid * 8;
    } else {
        const int64_t row = unit / upr;
        dst = y + row * ldy + (unit - row * upr) * 64 + j * 8;
    }

    uint4 o;
    if ((m & 0xFFu) == 0xFFu) {
        o = make_uint4(0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u);
    } else {
        // value = (4 + M) * m * 2^(E - 48 - 4 + E1_8 + E1_16): at most 6 significant bits, exact
        const uint32_t e8 = (m >> (8 + j)) & 1u;
        const uint32_t e16a = (m >> (16 + 2 * j)) & 1u, e16b = (m >> (17 + 2 * j)) & 1u;
        const uint32_t ebase = ((m >> 2) & 0x3Fu) + (127u - 52u) + e8;
        const float sig = (float)(4u + (m & 3u));
        const float sa = sig * u2f((ebase + e16a) << 23), sb = sig * u2f((ebase + e16b) << 23);
        const uint32_t lo = c & 0x07070707u, hi = (c >> 4) & 0x07070707u; // magnitudes of even / odd elements
        float f[8];
        f[0] = (float)(lo & 0xFFu) * sa;
        f[1] = (float)(hi & 0xFFu) * sa;
        f[2] = (float)((lo >> 8) & 0xFFu) * sa;
        f[3] = (float)((hi >> 8) & 0xFFu) * sa;
        f[4] = (float)((lo >> 16) & 0xFFu) * sb;
        f[5] = (float)((hi >> 16) & 0xFFu) * sb;
        f[6] = (float)(lo >> 24) * sb;
        f[7] = (float)(hi >> 24) * sb;
        uint32_t r[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            // exact values: their BF16 form is the top half of the fp32 pattern
            const uint32_t pair = __builtin_amdgcn_perm(f2u(f[2 * t + 1]), f2u(f[2 * t]), 0x07060302u);
            // sign of element 2t sits at bit 8t+3, of element 2t+1 at bit 8t+7
            const uint32_t cs = c >> (8 * t);
            const uint32_t sg = ((cs << 12) & 0x8000u) | ((cs << 24) & 0x80000000u);
            r[t] = pair | sg;
        }
        o = make_uint4(r[0], r[1], r[2], r[3]);
    }
    *reinterpret_cast<uint4 *>(dst) = o;
}

// ------------------------------------------------------------------ launchers

int launch_encode(const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode,
                  hipStream_t stream)
{
    const int64_t upr = K / 64, units = rows * upr;
    if (units == 0) return HIF4_OK;
    constexpr int LPU = 8;
    const int64_t threads = units * LPU;
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    const uint16_t *xs = static_cast<const uint16_t *>(x);
    uint32_t *cd = reinterpret_cast<uint32_t *>(codes);
    const bool contig = ldx == K;
    if (mode == HIF4_ROUND_RNE) {
        if (contig) hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RNE, true>), grid, block, 0, stream, xs, units, upr, ldx, cd, meta);
        else hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RNE, false>), grid, block, 0, stream, xs, units, upr, ldx, cd, meta);
    } else {
        if (contig) hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RHA, true>), grid, block, 0, stream, xs, units, upr, ldx, cd, meta);
        else hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RHA, false>), grid, block, 0, stream, xs, units, upr, ldx, cd, meta);
    }
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_decode(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, int64_t ldy,
                  hipStream_t stream)
{
    const int64_t upr = K / 64, chunks = rows * upr * 8;
    if (chunks == 0) return HIF4_OK;
    const dim3 grid((unsigned)((chunks + 255) / 256)), block(256);
    const uint32_t *cd = reinterpret_cast<const uint32_t *>(codes);
    uint16_t *ys = static_cast<uint16_t *>(y);
    if (ldy == K) hipLaunchKernelGGL((decode_kernel<true>), grid, block, 0, stream, cd, meta, chunks, upr, ldy, ys);
    else hipLaunchKernelGGL((decode_kernel<false>), grid, block, 0, stream, cd, meta, chunks, upr, ldy, ys);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

} // namespace hif4
