// HiF4 encoder (Algorithm 1, Section II-B of the HiF4 paper) and decoder (Eq. 2,
// Section II-A) for gfx950.  Both are HBM-bound streaming kernels: 128 B of BF16
// against 36 B of packed unit.
//
// Work split: a unit of 64 elements is shared by LPU adjacent lanes; every lane owns
// 8/LPU "chunks" of 8 consecutive elements (one 128-bit load each, one level-2
// micro-exponent domain, two level-3 domains).  The peak magnitude of the unit and
// the metadata bits are exchanged across the LPU lanes with DPP moves; nothing goes
// through LDS.
#include "hif4_expand.h"

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

// ------------------------------------------------------------------ encoder

template <bool NT>
__device__ __forceinline__ uint4 load16(const void *p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *q = static_cast<const u32x4 *>(p);
    u32x4 v = NT ? __builtin_nontemporal_load(q) : *q;
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <bool NT>
__device__ __forceinline__ void store16(void *p, uint4 v)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 t = { v.x, v.y, v.z, v.w };
    if (NT) __builtin_nontemporal_store(t, static_cast<u32x4 *>(p));
    else *static_cast<u32x4 *>(p) = t;
}

template <bool NT>
__device__ __forceinline__ void store4(uint32_t *p, uint32_t v)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
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
        const uint32_t b0 = ((__builtin_amdgcn_perm(ww[1], ww[0], 0x07050301u) >> 4) & 0x08080808u) | mag0;
        const uint32_t b1 = ((__builtin_amdgcn_perm(ww[3], ww[2], 0x07050301u) >> 4) & 0x08080808u) | mag1;
        // byte t of the chunk: element t in the low nibble, element 4 + t in the high nibble
        out[c] = special ? 0u : (b0 | (b1 << 4));
    }

    // Collect the metadata bits of the LPU lanes; every lane ends up with all of them.
    mbits |= dpp<DPP_XOR1>(mbits);
    if (LPU >= 4) mbits |= dpp<DPP_XOR2>(mbits);
    if (LPU >= 8) mbits |= dpp<DPP_HALF_MIRROR>(mbits);

    return special ? 0x000000FFu : (mbits | e6);
}

// Input element types of the encoder.  FP16 and FP32 inputs are first rounded to BF16 by the
// rounding mode of the conversion (Section II-B: other high-precision formats follow the same
// procedure; Algorithm 1 itself is written on BF16), then take the same path.
enum { IN_BF16 = 0, IN_F16 = 1, IN_F32 = 2 };

// One exact fp32 value -> BF16 pattern under MODE; NaNs stay NaNs, overflow gives infinity.
template <int MODE>
__device__ __forceinline__ uint32_t input_pair_to_bf16(float lo, float hi)
{
    if (MODE == HIF4_ROUND_RNE) return round_bf16_pair<MODE>(lo, hi); // v_cvt_pk_bf16_f32 keeps NaN and Inf
    uint32_t r[2];
    const uint32_t u[2] = { f2u(lo), f2u(hi) };
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t a = u[i] & 0x7FFFFFFFu;
        const uint32_t m = a > 0x7F800000u ? 0x7FC0u : (a + 0x8000u) >> 16; // magnitude, half away from zero
        r[i] = m | ((u[i] >> 16) & 0x8000u);
    }
    return r[0] | (r[1] << 16);
}

// 8 consecutive input elements starting at element index e of x -> 8 BF16 in a uint4.
template <int IN, int MODE, bool NT>
__device__ __forceinline__ uint4 load_chunk(const void *x, int64_t e)
{
    if (IN == IN_BF16) return load16<NT>(static_cast<const uint16_t *>(x) + e);
    if (IN == IN_F16) {
        const uint4 h = load16<NT>(static_cast<const uint16_t *>(x) + e);
        const uint32_t hw[4] = { h.x, h.y, h.z, h.w };
        uint32_t r[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            typedef _Float16 h2 __attribute__((ext_vector_type(2)));
            const h2 v = __builtin_bit_cast(h2, hw[t]);
            r[t] = input_pair_to_bf16<MODE>((float)v.x, (float)v.y); // FP16 -> fp32 is exact
        }
        return make_uint4(r[0], r[1], r[2], r[3]);
    }
    const float *f = static_cast<const float *>(x) + e;
    const uint4 a = load16<NT>(f), b = load16<NT>(f + 4);
    return make_uint4(input_pair_to_bf16<MODE>(u2f(a.x), u2f(a.y)), input_pair_to_bf16<MODE>(u2f(a.z), u2f(a.w)),
                      input_pair_to_bf16<MODE>(u2f(b.x), u2f(b.y)), input_pair_to_bf16<MODE>(u2f(b.z), u2f(b.w)));
}

// Thread block b encodes units [b * UPB, (b+1) * UPB), UPB = UPT * 256 / LPU; a thread's
// t-th unit is UPB*b + t*(256/LPU) + threadIdx/LPU, so that every load and store
// instruction of a wave touches one contiguous range.
template <int LPU, int MODE, bool CONTIG, int UPT, bool NT, int IN = IN_BF16>
__global__ __launch_bounds__(256) void encode_kernel(const void *__restrict__ x, int64_t units, int64_t upr,
                                                     int64_t ldx, uint32_t *__restrict__ codes,
                                                     uint32_t *__restrict__ meta)
{
    constexpr int NCH = 8 / LPU;
    constexpr int UPS = 256 / LPU; // units per block per slice
    const int l = (int)(threadIdx.x % LPU);
    const int64_t first = (int64_t)blockIdx.x * (UPS * UPT) + threadIdx.x / LPU;

    uint4 w[UPT][NCH];
    int64_t unit[UPT];
    bool live[UPT];
#pragma unroll
    for (int t = 0; t < UPT; ++t) {
        const int64_t u = first + (int64_t)t * UPS;
        live[t] = u < units;
        unit[t] = live[t] ? u : units - 1; // dead lanes redo the last unit and store nothing
        int64_t e0; // index of the unit's first element in x
        if (CONTIG) {
            e0 = unit[t] * 64;
        } else {
            const int64_t row = unit[t] / upr;
            e0 = row * ldx + (unit[t] - row * upr) * 64;
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c) w[t][c] = load_chunk<IN, MODE, NT>(x, e0 + 8 * (c * LPU + l));
    }
#pragma unroll
    for (int t = 0; t < UPT; ++t) {
        uint32_t out[NCH];
        const uint32_t m = encode_share<LPU, MODE>(w[t], l, out);
        if (live[t]) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) store4<NT>(codes + unit[t] * 8 + c * LPU + l, out[c]);
            if (l == 0) store4<NT>(meta + unit[t], m);
        }
    }
}

// ------------------------------------------------------------------ decoder

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

// One lane decodes CPT chunks of 8 elements; block b owns chunks [b*256*CPT, (b+1)*256*CPT).
// CELL: write each group of 8 in the GEMM's cell order (an internal staging format) instead
// of element order.
template <bool CONTIG, int CPT, bool NT, bool CELL = false>
__global__ __launch_bounds__(256) void decode_kernel(const uint32_t *__restrict__ codes,
                                                     const uint32_t *__restrict__ meta, int64_t chunks, int64_t upr,
                                                     int64_t ldy, uint16_t *__restrict__ y)
{
    const int64_t first = (int64_t)blockIdx.x * (256 * CPT) + threadIdx.x;
    uint32_t c[CPT], m[CPT];
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
        const int64_t id = first + t * 256;
        const int64_t idc = id < chunks ? id : chunks - 1;
        c[t] = NT ? __builtin_nontemporal_load(codes + idc) : codes[idc];
        m[t] = meta[idc >> 3];
    }
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
        const int64_t id = first + t * 256;
        if (id >= chunks) continue;
        const int64_t unit = id >> 3;
        const int j = (int)(id & 7);
        uint16_t *dst;
        if (CONTIG) {
            dst = y + id * 8;
        } else {
            const int64_t row = unit / upr;
            dst = y + row * ldy + (unit - row * upr) * 64 + j * 8;
        }
        if (CELL) store16<NT>(dst, expand_chunk(c[t], m[t], unit_scale_bits(m[t]), j));
        else store16<NT>(dst, decode_chunk(c[t], m[t], j));
    }
}

// ------------------------------------------------------------------ launchers

// Launch shapes measured on MI355X at 512 MiB of BF16: 4 lanes per unit and one unit
// slice per thread for the encoder (the kernel is VALU-limited, fewer lanes per unit
// amortise the per-unit scalar work); 4 chunks per thread and streaming stores for the
// decoder (write-dominated).
#ifndef HIF4_ENC_LPU
#define HIF4_ENC_LPU 4
#endif
#ifndef HIF4_ENC_UPT
#define HIF4_ENC_UPT 1
#endif
#ifndef HIF4_ENC_NT
#define HIF4_ENC_NT false
#endif
#ifndef HIF4_DEC_CPT
#define HIF4_DEC_CPT 4
#endif
#ifndef HIF4_DEC_NT
#define HIF4_DEC_NT true
#endif

template <int IN>
static int launch_encode_in(const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode,
                            hipStream_t stream)
{
    const int64_t upr = K / 64, units = rows * upr;
    if (units == 0) return HIF4_OK;
    constexpr int LPU = HIF4_ENC_LPU, UPT = HIF4_ENC_UPT;
    constexpr bool NT = HIF4_ENC_NT;
    constexpr int64_t UPB = (256 / LPU) * UPT; // units per block
    const dim3 grid((unsigned)((units + UPB - 1) / UPB)), block(256);
    uint32_t *cd = reinterpret_cast<uint32_t *>(codes);
    const bool contig = ldx == K;
    if (mode == HIF4_ROUND_RNE) {
        if (contig) hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RNE, true, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
        else hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RNE, false, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
    } else {
        if (contig) hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RHA, true, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
        else hipLaunchKernelGGL((encode_kernel<LPU, HIF4_ROUND_RHA, false, UPT, NT, IN>), grid, block, 0, stream, x, units, upr, ldx, cd, meta);
    }
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

int launch_encode(const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode,
                  hipStream_t stream)
{
    return launch_encode_in<IN_BF16>(x, rows, K, ldx, codes, meta, mode, stream);
}

// in_dtype: HIF4_IN_BF16 / HIF4_IN_F16 / HIF4_IN_F32 of the C interface (same numbering as above).
int launch_encode_from(int in_dtype, const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta,
                       int mode, hipStream_t stream)
{
    if (in_dtype == IN_F16) return launch_encode_in<IN_F16>(x, rows, K, ldx, codes, meta, mode, stream);
    if (in_dtype == IN_F32) return launch_encode_in<IN_F32>(x, rows, K, ldx, codes, meta, mode, stream);
    return launch_encode_in<IN_BF16>(x, rows, K, ldx, codes, meta, mode, stream);
}

int launch_decode(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, int64_t ldy,
                  hipStream_t stream)
{
    const int64_t upr = K / 64, chunks = rows * upr * 8;
    if (chunks == 0) return HIF4_OK;
    constexpr int CPT = HIF4_DEC_CPT;
    constexpr bool NT = HIF4_DEC_NT;
    const dim3 grid((unsigned)((chunks + 256 * CPT - 1) / (256 * CPT))), block(256);
    const uint32_t *cd = reinterpret_cast<const uint32_t *>(codes);
    uint16_t *ys = static_cast<uint16_t *>(y);
    if (ldy == K) hipLaunchKernelGGL((decode_kernel<true, CPT, NT>), grid, block, 0, stream, cd, meta, chunks, upr, ldy, ys);
    else hipLaunchKernelGGL((decode_kernel<false, CPT, NT>), grid, block, 0, stream, cd, meta, chunks, upr, ldy, ys);
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

// HiF4 -> BF16 copy in cell order, dense rows (row stride K): the activation operand of the
// tile GEMM.  Regular stores: the GEMM reads the copy right away.
int launch_decode_cells(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, hipStream_t stream)
{
    const int64_t upr = K / 64, chunks = rows * upr * 8;
    if (chunks == 0) return HIF4_OK;
    constexpr int CPT = HIF4_DEC_CPT;
    const dim3 grid((unsigned)((chunks + 256 * CPT - 1) / (256 * CPT))), block(256);
    hipLaunchKernelGGL((decode_kernel<true, CPT, false, true>), grid, block, 0, stream,
                       reinterpret_cast<const uint32_t *>(codes), meta, chunks, upr, K, static_cast<uint16_t *>(y));
    return hipGetLastError() == hipSuccess ? HIF4_OK : HIF4_ERR_DEVICE;
}

} // namespace hif4
