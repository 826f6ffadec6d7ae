/*
 * HiF4 CPU oracle — TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow, scalar implementation of what the HiFloat4 hot path computes,
 * written from the paper (HiFloat4 Format for Language Model Inference):
 *   - decode      : the value equation of Section II-A (Eq. 2) with the E6M2 /
 *                   S1P2 code points of Table 1;
 *   - encode      : Algorithm 1 (Section II-B): its three stages in the paper's order and
 *                   under the paper's names, every multiply producing a BF16, every
 *                   intermediate kept in a record that the tests can read;
 *   - GEMM        : the plain definition C = dec(A) * dec(W)^T in fp64, which per
 *                   pair of units equals the dot product of Eq. 4 (Section III-B).
 * Nothing here is blocked, fused or reordered.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call into this file; the GPU library
 * shares no code with it.
 *
 * Pins (see tests/test_oracle_*.py): Table 1 / Table 2 code points and extremes,
 * exhaustive decode in rational arithmetic, brute-force nearest-code search,
 * scaling / negation / permutation invariants, canonical round trips, units
 * worked by hand under both roundings (final planes and, through the record of
 * intermediates, every rounding step on an exact tie), and the MSE ratios of
 * Section III-A.  Under round-half-away only the rounding to E6M2 can change a
 * packed unit; the BF16 roundings of SF and of the scaled values (and of FP16 /
 * FP32 inputs) are still pinned, on the intermediates themselves.
 * Parity unpinned (the paper is silent; these are documented readings): the bit
 * layout of the packed unit, RNE as the default of the two roundings the paper
 * allows, Inf inputs producing the NaN unit, the reciprocal table being rounded
 * to nearest, the sign of zero copying the input sign, FP16 / FP32 inputs being
 * rounded to BF16 before Algorithm 1 (hif4o_quantize_from).
 *
 * Packed layout used on both sides of the boundary:
 *   codes[row][K/2] : 32 bytes per unit, 4 bytes per group of 8 elements; inside
 *                     group j, byte 4j+t (t = 0..3) holds element 8j+t in its low
 *                     nibble and element 8j+4+t in its high nibble, so the low
 *                     nibbles of the 4 bytes are one level-3 group and the high
 *                     nibbles the next.  nibble = sign(bit3) | integer bit(bit2) |
 *                     2 fraction bits (S1P2, sign-magnitude).
 *   meta[row][K/64] : u32, bits 7:0 E6M2 byte (eeeeee_mm), bits 15:8 E1_8 (bit j
 *                     <-> elements 8j..8j+7), bits 31:16 E1_16 (bit k <-> elements
 *                     4k..4k+3).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Where element i (0..63) of a unit lives in its 32 code bytes. */
static int code_byte(int i) { return 4 * (i >> 3) + (i & 3); }
static int code_shift(int i) { return ((i >> 2) & 1) * 4; }

#define HIF4O_ROUND_RNE 0 /* round half to even            (Section II-B, last paragraph) */
#define HIF4O_ROUND_RHA 1 /* round half away from zero     (same paragraph)               */

/* ---------------------------------------------------------------- BF16 scalar */

/* BF16 bit pattern -> its exact value (BF16 is the top half of an IEEE fp32). */
double hif4o_bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round a non-negative, exactly-held quotient to an integer in the chosen mode. */
static double round_int(double q, int mode)
{
    if (mode == HIF4O_ROUND_RHA) return floor(q + 0.5); /* q has few bits: q+0.5 is exact */
    return nearbyint(q); /* default FP environment: ties to even */
}

/* Round an exactly-held real to BF16 (8-bit significand, exponent range of fp32,
 * gradual underflow), returning the bit pattern. */
uint16_t hif4o_f64_to_bf16(double v, int mode)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    if (isnan(v)) return 0x7FC0u;
    double a = fabs(v);
    if (isinf(a)) return sign | 0x7F80u;
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e); /* a = f * 2^e, f in [0.5,1)  ->  a = 1.xxx * 2^(e-1) */
    int E = e - 1;
    if (E < -126) { /* subnormal range: spacing 2^-133 */
        double r = round_int(ldexp(a, 133), mode); /* 0..128; 128 is the least normal */
        return sign | (uint16_t)r;
    }
    double r = round_int(ldexp(a, 7 - E), mode); /* in [128,256] */
    if (r == 256.0) { r = 128.0; E += 1; }
    if (E > 127) return sign | 0x7F80u; /* overflow -> inf */
    return sign | (uint16_t)(((E + 127) << 7) | ((int)r - 128));
}

/* BF16 x BF16 -> BF16.  The exact product has at most 16 significant bits, so it
 * is exact in fp64; one rounding follows. */
uint16_t hif4o_bf16_mul(uint16_t a, uint16_t b, int mode)
{
    return hif4o_f64_to_bf16(hif4o_bf16_to_f64(a) * hif4o_bf16_to_f64(b), mode);
}

/* ------------------------------------------------------------ E6M2 (Table 1) */

/* Value of an E6M2 byte: 2^E * 1.M, bias 48, normals only; 0xFF is NaN (Eq. 1). */
double hif4o_e6m2_to_f64(uint8_t byte)
{
    if (byte == 0xFF) return NAN;
    int E = (int)(byte >> 2) - 48;
    int M = byte & 3;
    return ldexp(1.0 + 0.25 * M, E);
}

/* BF16_to_E6M2 (Algorithm 1, level-1 scale factor): round the BF16 scale to a
 * 3-bit significand.  E6M2 has neither zero nor subnormals nor infinity, and its
 * top code is NaN, so results below 2^-48 become the least code 0x00 and results
 * of 2^15*1.75 or more become the greatest finite code 0xFE. */
uint8_t hif4o_bf16_to_e6m2(uint16_t sf, int mode)
{
    double v = hif4o_bf16_to_f64(sf & 0x7FFFu);
    if (v == 0.0) return 0x00;
    int e;
    (void)frexp(v, &e);
    int E = e - 1;
    double q = round_int(ldexp(v, 2 - E), mode); /* significand in quarter steps: 4..8 */
    if (q == 8.0) { q = 4.0; E += 1; }
    if (E < -48) return 0x00;
    if (E > 15 || (E == 15 && q == 7.0)) return 0xFE;
    return (uint8_t)(((E + 48) << 2) | ((int)q - 4));
}

/* E6M2_REC_to_BF16 (Algorithm 1, reciprocal of E6M2): four-entry table on the
 * 2-bit mantissa plus an exponent subtraction.  Entries are 1/1.00, 1/1.25, 1/1.50
 * and 1/1.75 rounded to nearest BF16: 1.0, 1.6015625/2, 1.3359375/2, 1.140625/2. */
uint16_t hif4o_e6m2_rec_to_bf16(uint8_t byte)
{
    static const uint16_t rec_mant[4] = { 0x00, 0x4D, 0x2B, 0x12 };
    int E = (int)(byte >> 2) - 48;
    int M = byte & 3;
    int exp_field = 127 - E - (M ? 1 : 0);
    return (uint16_t)((exp_field << 7) | rec_mant[M]);
}

/* BF16_to_S1P2 (Algorithm 1, last step) on an exactly-held scaled value: round the
 * magnitude to a multiple of 0.25, clamp to 1.75, keep the sign given. */
uint8_t hif4o_to_s1p2(double scaled, int negative, int mode)
{
    double a = fabs(scaled);
    double m = round_int(a * 4.0, mode); /* a*4 is exact */
    if (m > 7.0) m = 7.0;                /* nearest representable bound */
    return (uint8_t)((negative ? 8 : 0) | (int)m);
}

/* ------------------------------------------------------------ one unit: encode */

#define INV7_BF16 0x3E12u /* (1/7) rounded to BF16 = 73/512 */

/* Every intermediate of one conversion, under the paper's names (Algorithm 1), so that each
 * rounding step can be pinned on its own by the tests.  BF16 values are bit patterns. */
typedef struct {
    uint16_t V16[16], V8[8], Vmax; /* stage 1: peak magnitudes 64 -> 16 -> 8 -> 1                     */
    uint16_t SF;                   /* stage 2: Vmax * (1/7)_BF16, a BF16                               */
    uint8_t E6M2;                  /*          BF16_to_E6M2(SF)                                        */
    uint16_t REC;                  /*          E6M2_REC_to_BF16(E6M2)                                  */
    uint16_t P8[8], P16[16];       /*          V8[j] * REC and V16[k] * REC, each a BF16               */
    uint32_t E1_8, E1_16;          /*          the micro-exponent bits                                 */
    uint16_t scaled[64];           /* stage 3: V64[i] * REC, a BF16 (before the exact 2^-E1 factors)   */
    uint8_t S1P2[64];              /*          the 4-bit codes                                         */
    int special;                   /* a NaN or an infinity among the inputs: the unit is the NaN unit  */
} hif4o_steps;

static double mag_of(uint16_t b) { return hif4o_bf16_to_f64(b & 0x7FFFu); }

/* Stage 1: the tree of peak magnitudes.  Each level takes the larger of its children. */
static void peak_tree(const uint16_t x[64], hif4o_steps *t)
{
    for (int k = 0; k < 16; ++k) {
        t->V16[k] = 0;
        for (int i = 4 * k; i < 4 * k + 4; ++i)
            if (mag_of(x[i]) > mag_of(t->V16[k])) t->V16[k] = x[i] & 0x7FFFu;
    }
    for (int j = 0; j < 8; ++j) t->V8[j] = mag_of(t->V16[2 * j + 1]) > mag_of(t->V16[2 * j]) ? t->V16[2 * j + 1] : t->V16[2 * j];
    t->Vmax = 0;
    for (int j = 0; j < 8; ++j)
        if (mag_of(t->V8[j]) > mag_of(t->Vmax)) t->Vmax = t->V8[j];
}

/* Stage 2: the unit scale from the overall peak, its reciprocal, and one micro-exponent bit per
 * group of 8 (scaled peak at least 4) and per group of 4 (scaled peak, halved where its group of 8
 * has its bit set, at least 2).  Every product is a BF16 before it is compared. */
static void scaling_metadata(hif4o_steps *t, int mode)
{
    t->SF = hif4o_bf16_mul(t->Vmax, INV7_BF16, mode);
    t->E6M2 = hif4o_bf16_to_e6m2(t->SF, mode);
    t->REC = hif4o_e6m2_rec_to_bf16(t->E6M2);
    t->E1_8 = t->E1_16 = 0;
    for (int j = 0; j < 8; ++j) {
        t->P8[j] = hif4o_bf16_mul(t->V8[j], t->REC, mode);
        if (hif4o_bf16_to_f64(t->P8[j]) >= 4.0) t->E1_8 |= 1u << j;
    }
    for (int k = 0; k < 16; ++k) {
        t->P16[k] = hif4o_bf16_mul(t->V16[k], t->REC, mode);
        int above = (int)((t->E1_8 >> (k / 2)) & 1u);             /* the bit of the enclosing group of 8 */
        if (ldexp(hif4o_bf16_to_f64(t->P16[k]), -above) >= 2.0) t->E1_16 |= 1u << k; /* times 2^-E1_8: exact */
    }
}

/* Stage 3: every element times the reciprocal (a BF16), divided by the two powers of two that its
 * groups carry (exact), rounded to S1P2 with the input's sign. */
static void element_codes(const uint16_t x[64], hif4o_steps *t, int mode)
{
    for (int i = 0; i < 64; ++i) {
        t->scaled[i] = hif4o_bf16_mul(x[i], t->REC, mode);
        int halvings = (int)((t->E1_8 >> (i / 8)) & 1u) + (int)((t->E1_16 >> (i / 4)) & 1u);
        double s = ldexp(hif4o_bf16_to_f64(t->scaled[i]), -halvings);
        t->S1P2[i] = hif4o_to_s1p2(s, (x[i] & 0x8000u) != 0, mode);
    }
}

/* Algorithm 1 for one vector of 64 BF16 values, all intermediates kept. */
void hif4o_encode_unit_steps(const uint16_t x[64], int mode, hif4o_steps *t)
{
    memset(t, 0, sizeof *t);
    for (int i = 0; i < 64; ++i)
        if ((x[i] & 0x7FFFu) >= 0x7F80u) t->special = 1; /* Inf or NaN among the inputs */
    if (t->special) { /* the unit as a whole becomes NaN (Eq. 2, first case) */
        t->E6M2 = 0xFF;
        return;
    }
    peak_tree(x, t);
    scaling_metadata(t, mode);
    element_codes(x, t, mode);
}

/* Algorithm 1 for one vector of 64 BF16 values.  codes: 32 bytes, meta: one u32. */
void hif4o_encode_unit(const uint16_t x[64], uint8_t codes[32], uint32_t *meta, int mode)
{
    hif4o_steps t;
    hif4o_encode_unit_steps(x, mode, &t);
    memset(codes, 0, 32);
    for (int i = 0; i < 64; ++i) codes[code_byte(i)] |= (uint8_t)(t.S1P2[i] << code_shift(i));
    *meta = (t.E1_16 << 16) | (t.E1_8 << 8) | t.E6M2;
}

/* ------------------------------------------------------------ one unit: decode */

/* Eq. 2 for element i (0-based) of a unit, as an exact real. */
double hif4o_decode_elem_f64(const uint8_t codes[32], uint32_t meta, int i)
{
    uint8_t e6m2 = (uint8_t)(meta & 0xFFu);
    if (e6m2 == 0xFF) return NAN;
    int e8 = (int)((meta >> (8 + (i >> 3))) & 1u);
    int e16 = (int)((meta >> (16 + (i >> 2))) & 1u);
    uint8_t c = (uint8_t)((codes[code_byte(i)] >> code_shift(i)) & 0xFu);
    double s1p2 = 0.25 * (double)(c & 7u);
    if (c & 8u) s1p2 = -s1p2; /* keeps -0.0 */
    return hif4o_e6m2_to_f64(e6m2) * ldexp(1.0, e8 + e16) * s1p2;
}

/* Eq. 2 for a whole unit, as BF16 patterns.  Every finite HiF4 value has at most
 * six significant bits and lies in [2^-50, 2^18*1.3125], so this conversion never
 * rounds; *inexact is set if it ever would. */
void hif4o_decode_unit(const uint8_t codes[32], uint32_t meta, uint16_t y[64], int *inexact)
{
    for (int i = 0; i < 64; ++i) {
        double v = hif4o_decode_elem_f64(codes, meta, i);
        y[i] = hif4o_f64_to_bf16(v, HIF4O_ROUND_RNE);
        if (inexact && !isnan(v) && hif4o_bf16_to_f64(y[i]) != v) *inexact = 1;
    }
}

/* ------------------------------------------------------------ matrices of units */

/* rows x K BF16 matrix (row stride ldx elements, K a multiple of 64) -> planes. */
int hif4o_quantize(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx,
                   uint8_t *codes, uint32_t *meta, int mode)
{
    if (K % 64 != 0 || rows < 0 || K < 0 || ldx < K) return -2;
    int64_t upr = K / 64;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t u = 0; u < upr; ++u)
            hif4o_encode_unit(x + r * ldx + 64 * u, codes + (r * upr + u) * 32, meta + r * upr + u, mode);
    return 0;
}

/* IEEE binary16 pattern -> its exact value, by the definition of the format. */
double hif4o_f16_to_f64(uint16_t h)
{
    int sign = h >> 15, e = (h >> 10) & 0x1F, m = h & 0x3FF;
    double v;
    if (e == 0x1F) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -24);          /* subnormal: m * 2^-10 * 2^-14 */
    else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

/* FP32 / FP16 matrices (Section II-B, first paragraph: other high-precision formats take
 * the same procedure).  The paper prints no algorithm for them; the reading taken here is
 * that every input is first rounded to BF16 with the conversion's rounding mode, after
 * which Algorithm 1 runs as written.  in_dtype: 1 = FP16 patterns (uint16), 2 = FP32.
 * as_bf16 (may be NULL): receives the rounded inputs, rows x K dense, so that the conversion step
 * can be pinned on its own. */
int hif4o_quantize_from(int in_dtype, const void *x, int64_t rows, int64_t K, int64_t ldx,
                        uint8_t *codes, uint32_t *meta, int mode, uint16_t *as_bf16)
{
    if (in_dtype == 0) {
        if (as_bf16 && K % 64 == 0 && rows >= 0 && K >= 0 && ldx >= K)
            for (int64_t r = 0; r < rows; ++r) memcpy(as_bf16 + r * K, (const uint16_t *)x + r * ldx, (size_t)K * 2);
        return hif4o_quantize((const uint16_t *)x, rows, K, ldx, codes, meta, mode);
    }
    if (in_dtype != 1 && in_dtype != 2) return -4;
    if (K % 64 != 0 || rows < 0 || K < 0 || ldx < K) return -2;
    int64_t upr = K / 64;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t u = 0; u < upr; ++u) {
            uint16_t v64[64];
            for (int i = 0; i < 64; ++i) {
                int64_t at = r * ldx + 64 * u + i;
                double v = in_dtype == 1 ? hif4o_f16_to_f64(((const uint16_t *)x)[at]) : (double)((const float *)x)[at];
                v64[i] = hif4o_f64_to_bf16(v, mode);
            }
            if (as_bf16) memcpy(as_bf16 + r * K + 64 * u, v64, sizeof v64);
            hif4o_encode_unit(v64, codes + (r * upr + u) * 32, meta + r * upr + u, mode);
        }
    return 0;
}

int hif4o_dequantize(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K,
                     uint16_t *y, int64_t ldy)
{
    if (K % 64 != 0 || rows < 0 || K < 0 || ldy < K) return -2;
    int64_t upr = K / 64;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t u = 0; u < upr; ++u) {
            int inexact = 0;
            hif4o_decode_unit(codes + (r * upr + u) * 32, meta[r * upr + u], y + r * ldy + 64 * u, &inexact);
            bad |= inexact;
        }
    return bad ? -100 : 0;
}

/* ------------------------------------------------------------ GEMM, fp64 */

/* C[i][j] = sum_k a[rows[i]][k] * w[cols[j]][k], operands given as BF16 patterns
 * (already decoded, or plain BF16 activations), accumulated in fp64 in index order.
 * rows == NULL means rows 0..nr-1, likewise cols.  c is nr x nc, row-major. */
int hif4o_gemm_f64(const uint16_t *a, int64_t lda, const uint16_t *w, int64_t ldw,
                   const int64_t *rows, int64_t nr, const int64_t *cols, int64_t nc,
                   int64_t K, double *c)
{
    if (nr < 0 || nc < 0 || K < 0 || lda < K || ldw < K) return -2;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nr; ++i) {
        const uint16_t *ar = a + (rows ? rows[i] : i) * lda;
        for (int64_t j = 0; j < nc; ++j) {
            const uint16_t *wr = w + (cols ? cols[j] : j) * ldw;
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += hif4o_bf16_to_f64(ar[k]) * hif4o_bf16_to_f64(wr[k]);
            c[i * nc + j] = acc;
        }
    }
    return 0;
}

/* Eq. 4 for one pair of units, in the paper's nesting: integer sums of S1P2
 * products (in sixteenths), shifted by the level-3 then level-2 micro-exponents,
 * one floating-point scale at the end. */
double hif4o_unit_dot(const uint8_t ca[32], uint32_t ma, const uint8_t cb[32], uint32_t mb)
{
    if ((ma & 0xFFu) == 0xFF || (mb & 0xFFu) == 0xFF) return NAN;
    int64_t outer = 0;
    for (int i = 0; i < 8; ++i) {
        int64_t mid = 0;
        for (int j = 2 * i; j < 2 * i + 2; ++j) {
            int64_t inner = 0;
            for (int k = 4 * j; k < 4 * j + 4; ++k) {
                int a = (ca[code_byte(k)] >> code_shift(k)) & 0xF, b = (cb[code_byte(k)] >> code_shift(k)) & 0xF;
                int sa = (a & 8) ? -(a & 7) : (a & 7), sb = (b & 8) ? -(b & 7) : (b & 7);
                inner += sa * sb; /* in units of 1/16 */
            }
            mid += inner * ((int64_t)1 << (((ma >> (16 + j)) & 1u) + ((mb >> (16 + j)) & 1u)));
        }
        outer += mid * ((int64_t)1 << (((ma >> (8 + i)) & 1u) + ((mb >> (8 + i)) & 1u)));
    }
    return hif4o_e6m2_to_f64((uint8_t)(ma & 0xFF)) * hif4o_e6m2_to_f64((uint8_t)(mb & 0xFF)) * ((double)outer / 16.0);
}

int hif4o_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void hif4o_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
