/*
 * libhif4 — HiFloat4 (HiF4) block floating point on AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer below is a DEVICE pointer owned by the caller unless it
 * says "host".  The library allocates nothing and keeps no state between calls;
 * each call validates its arguments on the host, enqueues its kernels on the
 * caller's stream (a hipStream_t passed as void*, NULL = the default stream) and
 * returns without synchronising.  Return value: HIF4_OK or a negative error code;
 * nothing is enqueued when an error is returned, except HIF4_ERR_DEVICE, which
 * reports a launch failure.
 *
 * The format (paper: "HiFloat4 Format for Language Model Inference", Section II-A):
 * one unit = 64 consecutive values along the reduction axis K, stored as 64 4-bit
 * S1P2 elements plus 32 bits of scaling metadata (E6M2, E1_8, E1_16) = 36 bytes,
 * 4.5 bits per value.  Element i (0-based) of a unit has the value (Eq. 2)
 *     E6M2 * 2^(E1_8[i/8] + E1_16[i/4]) * S1P2[i],      all 64 NaN if E6M2 is NaN.
 *
 * Packed layout (version 1; the paper's figure fixing the bit order is not part of
 * its text, so this is the library's own, documented choice) — two planes:
 *   codes : uint8  [rows][K/2]   32 bytes per unit, 4 bytes per group of 8 elements (one
 *                                level-2 domain).  Inside group j, byte 4j+t (t = 0..3)
 *                                holds element 8j+t in its low nibble and element 8j+4+t
 *                                in its high nibble: the four low nibbles are one level-3
 *                                group, the four high nibbles the next, so that one mask
 *                                separates the two groups of a 32-bit word.
 *                                nibble = sign<<3 | integer bit<<2 | two fraction bits
 *                                (sign-magnitude, +-0 both exist).
 *   meta  : uint32 [rows][K/64]  bits  7:0  E6M2 byte, exponent field (bias 48) in bits
 *                                           7:2, mantissa in bits 1:0, 0xFF = NaN;
 *                                bits 15:8  E1_8,  bit j  scales elements 8j..8j+7 by 2;
 *                                bits 31:16 E1_16, bit k  scales elements 4k..4k+3 by 2.
 * Rows of both planes are dense (no padding).  BF16 matrices are row-major with K
 * contiguous and a row stride (ldx, ldy, lda) given in elements.
 */
#ifndef HIF4_H
#define HIF4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HIF4_VERSION 1
#define HIF4_UNIT 64 /* group size (Table 2) */

enum {
    HIF4_OK = 0,
    HIF4_ERR_NULL = -1,        /* a required pointer is NULL */
    HIF4_ERR_SHAPE = -2,       /* negative size, K not a multiple of 64, leading dimension < K, sizes over 2^31 units per row */
    HIF4_ERR_ALIGN = -3,       /* BF16 matrices: base and row stride 16-byte aligned; codes 16-byte; meta 4-byte */
    HIF4_ERR_UNSUPPORTED = -4, /* an enum value this build does not implement */
    HIF4_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than hif4_gemm_workspace_bytes() */
    HIF4_ERR_DEVICE = -6,      /* the HIP runtime reported an error at launch */
    HIF4_ERR_SCRATCH = -7      /* hif4_gemm_noalloc: the call needs more than HIF4_NOALLOC_SCRATCH_BYTES of scratch */
};

/* Rounding used by every rounding step of the conversion (Section II-B, last
 * paragraph: round-half-to-even or round-half-away-from-zero). */
enum { HIF4_ROUND_RNE = 0, HIF4_ROUND_RHA = 1 };

/* What the A operand of a GEMM is. */
enum {
    HIF4_A_BF16_QUANTIZE = 0, /* BF16 activations, converted to HiF4 inside the call (W4A4)     */
    HIF4_A_HIF4 = 1,          /* already packed: a = codes plane, a_meta = meta plane (W4A4)      */
    HIF4_A_BF16_KEEP = 2      /* BF16 activations used as they are (HiF4-weight-only GEMM)        */
};

enum { HIF4_OUT_BF16 = 0, HIF4_OUT_F32 = 1 };

/* Element type of the matrix hif4_quantize_from converts. */
enum { HIF4_IN_BF16 = 0, HIF4_IN_F16 = 1 /* IEEE binary16 */, HIF4_IN_F32 = 2 };

/*
 * BF16 -> HiF4: Algorithm 1 (Section II-B) on every unit of a rows x K matrix.
 *   stage 1  peak magnitudes 64 -> 16 -> 8 -> 1;
 *   stage 2  SF = Vmax * (1/7)_BF16, E6M2 = BF16_to_E6M2(SF), its reciprocal by table,
 *            E1_8[j]  = (V8[j]  * REC >= 4),  E1_16[k] = (V16[k] * REC * 2^-E1_8[k/2] >= 2);
 *   stage 3  each element * REC * 2^-(E1_8 + E1_16), rounded to a multiple of 0.25 and
 *            clamped to +-1.75 with its sign kept.
 * Every product is rounded to BF16 before it is compared or converted.  E6M2 saturates
 * at its least (0x00) and greatest finite (0xFE) codes.  A unit holding a NaN or an
 * infinity becomes the NaN unit (meta 0x000000FF, codes 0).  The sign bit of every
 * element, zero included, is the sign bit of its input.
 *   x      in   BF16 [rows][ldx], ldx >= K, read only
 *   codes  out  uint8 [rows][K/2]
 *   meta   out  uint32 [rows][K/64]
 * rows == 0 or K == 0 is a no-op.  x must not overlap the outputs.
 */
int hif4_quantize(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx,
                  uint8_t *codes, uint32_t *meta, int round_mode, void *stream);

/*
 * The same conversion from a BF16, FP16 or FP32 matrix (Section II-B, first paragraph: other
 * high-precision formats follow the same procedure).  The paper gives no separate algorithm
 * for them; here every FP16 / FP32 input is first rounded to BF16 with round_mode (FP32 values
 * beyond the BF16 range become infinities, so their unit becomes the NaN unit), then Algorithm 1
 * runs as written.  in_dtype == HIF4_IN_BF16 is hif4_quantize.  x and ldx as there, with ldx in
 * elements and rows starting on 16-byte boundaries (ldx a multiple of 8, or of 4 for FP32).
 */
int hif4_quantize_from(int in_dtype, const void *x, int64_t rows, int64_t K, int64_t ldx,
                       uint8_t *codes, uint32_t *meta, int round_mode, void *stream);

/*
 * HiF4 -> BF16: Eq. 2 (Section II-A) on every unit.  Every finite HiF4 value has at
 * most six significant bits and lies in [2^-50, 2^18 * 1.3125], so the result is
 * exact.  NaN units give the quiet NaN 0x7FC0 in all 64 places; zero elements keep
 * their sign.
 *   y  out  BF16 [rows][ldy], ldy >= K
 */
int hif4_dequantize(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K,
                    void *y_bf16, int64_t ldy, void *stream);

/*
 * C[M][N] = A[M][K] * W[N][K]^T with W in HiF4 (units along K) and fp32 accumulation.
 * Between two HiF4 operands each 64-wide K step is the unit dot product of Eq. 4
 * (Section III-B); with a_kind == HIF4_A_BF16_KEEP, A enters the products as BF16.
 *   a          in   BF16 [M][lda] (kinds 0 and 2) or codes uint8 [M][K/2] (kind 1; lda ignored)
 *   a_meta     in   uint32 [M][K/64] for kind 1, NULL otherwise
 *   w_codes    in   uint8 [N][K/2];  w_meta in uint32 [N][K/64]
 *   c          out  BF16 or fp32 [M][ldc] per out_dtype, ldc >= N
 *   workspace       device scratch of at least hif4_gemm_workspace_bytes(a_kind, M, K)
 *                   bytes, 16-byte aligned.  Kinds 0 and 1 use it for the exact BF16 values
 *                   of the HiF4 activations (2 bytes per element; when the call quantises A
 *                   itself, always with HIF4_ROUND_RNE, the packed planes never reach memory);
 *                   kind 2 needs none and it may be NULL.  Its contents after the call are
 *                   unspecified.
 * M == 0 or N == 0 is a no-op; K == 0 writes zeros.
 * Which kernel runs depends on a_kind, M, N, K and the workspace size only, and every kernel adds
 * its products in a fixed order (no atomics): equal calls give equal bits; calls that differ in
 * those agree to fp32 summation accuracy.
 */
int hif4_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda,
              const uint8_t *w_codes, const uint32_t *w_meta,
              int64_t M, int64_t N, int64_t K,
              void *c, int64_t ldc, int out_dtype,
              void *workspace, size_t workspace_bytes, void *stream);

/*
 * hif4_gemm whose result leaves as HiF4: C = A * W^T is rounded to BF16 as HIF4_OUT_BF16 would
 * round it, and every row of C is then converted by Algorithm 1 (Section II-B) with units of 64
 * consecutive columns, i.e. along the axis the next linear layer reduces over (the paper converts
 * every linear layer's input before its matrix product, Section IV).  The planes equal
 * hif4_quantize(result of hif4_gemm with HIF4_OUT_BF16) bit for bit where hif4_gemm runs the same
 * main loop with the same split of K, which it does from 65 rows on given the same workspace size;
 * up to 64 rows hif4_gemm may take another kernel, whose fp32 additions are grouped differently, so
 * that a BF16 value may now and then round the other way.  C never crosses HBM as BF16.
 *   c_codes  out  uint8 [M][N/2], c_meta out uint32 [M][N/64];  N a multiple of 64
 * Other arguments, workspace and errors as hif4_gemm.
 */
int hif4_gemm_to_hif4(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda,
                      const uint8_t *w_codes, const uint32_t *w_meta,
                      int64_t M, int64_t N, int64_t K,
                      uint8_t *c_codes, uint32_t *c_meta, int round_mode,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Grouped (mixture-of-experts) GEMM: the rows of A are sorted by expert; expert e owns
 * rows offs[e] .. offs[e+1]-1 and multiplies them by its own weights
 * W[e] (w_codes [E][N][K/2], w_meta [E][N][K/64]).  offs is a DEVICE int32[E+1] array,
 * non-decreasing, offs[0] == 0, offs[E] == total_rows; it is read by the kernels only,
 * so no host synchronisation happens.  Experts with no rows are skipped.  Other
 * arguments as hif4_gemm with M = total_rows.  For a_kind 2 no workspace is needed; given
 * one of at least total_rows * K * 2 bytes (16-byte aligned) the call keeps a reordered copy
 * of A there and runs the faster kernel of the other two kinds.
 */
int hif4_grouped_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda,
                      const uint8_t *w_codes, const uint32_t *w_meta,
                      const int32_t *offs, int E, int64_t total_rows, int64_t N, int64_t K,
                      void *c, int64_t ldc, int out_dtype,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * hif4_grouped_gemm whose result leaves as HiF4 (mixture-of-experts layers feed the next linear layer, whose input
 * the paper converts before its matrix product, Section IV): every row of C that an expert owns, rounded to BF16 as
 * HIF4_OUT_BF16 would round it, is converted by Algorithm 1 (Section II-B) with units of 64 consecutive columns.
 * The planes equal hif4_quantize(result of hif4_grouped_gemm with HIF4_OUT_BF16 and the same workspace size) bit
 * for bit.  Rows that no expert owns are not written.
 *   c_codes  out  uint8 [total_rows][N/2], c_meta out uint32 [total_rows][N/64];  N a multiple of 64
 * Other arguments, workspace and errors as hif4_grouped_gemm.
 */
int hif4_grouped_gemm_to_hif4(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda,
                              const uint8_t *w_codes, const uint32_t *w_meta,
                              const int32_t *offs, int E, int64_t total_rows, int64_t N, int64_t K,
                              uint8_t *c_codes, uint32_t *c_meta, int round_mode,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Scratch bytes hif4_gemm / hif4_grouped_gemm need for M (or total_rows) rows of A. Host function. */
size_t hif4_gemm_workspace_bytes(int a_kind, int64_t M_or_total_rows, int64_t K);

/*
 * Optional larger workspace for hif4_gemm / hif4_gemm_to_hif4 (not the grouped calls): the size below which the
 * library cannot take its fastest path for the shape.  Host function.  hif4_gemm_plan() tells which path a given
 * size selects; a workspace between two sizes of the table is used as the smaller one.
 *
 *   shape                                                what the extra room holds             returned size
 *   ---------------------------------------------------  ------------------------------------  -----------------------------
 *   M >= 3328; or M >= 1536 with N*K <= 128 Mi and       a decoded copy of W (exact BF16       kinds 0, 1: mandatory size (16-byte
 *   ceil(N/32)*ceil(M/128) > 2048 (or M > 2048)          values, 2 bytes per weight); kind 2    rounded) + N*K*2;  kind 2: M*K*2
 *                                                        also a reordered copy of A             (16-byte rounded) + N*K*2
 *   kind 2 only, 17 <= M <= 64 with N*K above 48 Mi      a reordered copy of A (it selects     M*K*2
 *   (M <= 32) or 24 Mi; 65 <= M <= 192; 193 <= M <=      the kernel of the HiF4 x HiF4 calls
 *   2048 with ceil(N/32)*ceil(M/128) <= 2048             of those shapes)
 *   anything else                                        nothing                               hif4_gemm_workspace_bytes()
 *
 * With the decoded copy of W the products are the same and exact and the fp32 additions are grouped differently,
 * so results agree to fp32 summation accuracy, not always bit for bit.
 */
size_t hif4_gemm_workspace_bytes_decoded_w(int a_kind, int64_t M, int64_t N, int64_t K);

/*
 * hif4_gemm for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The call takes the
 * scratch that hif4_gemm takes from its workspace argument (the exact BF16 values of HiF4
 * activations, hif4_gemm_workspace_bytes(a_kind, M, K) bytes) from a static device array of
 * HIF4_NOALLOC_SCRATCH_BYTES bytes inside the library instead; it allocates and frees nothing.  Every
 * GPU the library runs on holds its own copy of that array from the first such call on it until the
 * process ends.  Result: bit for bit that of hif4_gemm given a workspace of exactly
 * hif4_gemm_workspace_bytes(a_kind, M, K) bytes (the same kernels run).  a_kind HIF4_A_BF16_KEEP needs no
 * scratch and is hif4_gemm with a NULL workspace.
 * A call that needs more scratch returns HIF4_ERR_SCRATCH and enqueues nothing; other arguments and
 * errors as hif4_gemm.  All calls on one GPU share the one array, which keeps the last call's contents
 * (every call overwrites the part it reads before reading it, nothing needs to start at zero): calls
 * whose kernels may overlap on one GPU (different streams, or threads) race and must be ordered by the
 * caller.
 */
#define HIF4_NOALLOC_SCRATCH_BYTES (64 << 20)
int hif4_gemm_noalloc(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda,
                      const uint8_t *w_codes, const uint32_t *w_meta,
                      int64_t M, int64_t N, int64_t K,
                      void *c, int64_t ldc, int out_dtype, void *stream);

/* HIF4_NOALLOC_SCRATCH_BYTES of the built library.  Host function. */
size_t hif4_gemm_noalloc_max_bytes(void);

/*
 * Which main loop a GEMM call runs: a pure host function of the call's kind, shape, output form and workspace size,
 * the same one the library itself dispatches by (for tests, benchmarks and bug reports; nothing is launched).
 *   experts          0 for hif4_gemm / hif4_gemm_to_hif4 / hif4_gemm_noalloc, E for the grouped calls
 *   result_as_hif4   non-zero for the ..._to_hif4 calls
 *   workspace_bytes  as passed to the call (taken to be non-NULL and 16-byte aligned when non-zero); lda is taken as K
 * Returns a HIF4_PLAN_* value, or a negative status for arguments the calls would reject.
 */
enum {
    HIF4_PLAN_ZERO_FILL = 0, /* K == 0: the result is zero                                                        */
    HIF4_PLAN_FEWROWS = 1,   /* up to 32 rows against a wide W: W streamed once, E6M2 applied to unit sums      */
    HIF4_PLAN_SKINNY = 2,    /* up to 64 rows: K split over the waves of 16-column workgroups                     */
    HIF4_PLAN_STREAM = 3,    /* 33..64 BF16 rows against many columns: columns split only                         */
    HIF4_PLAN_COLWAVE = 4,   /* few rows per weight (grouped, small dense): W expanded into MFMA operands         */
    HIF4_PLAN_PLANES = 5,    /* many rows, large workspace: both operands decoded once, plain BF16 main loop      */
    HIF4_PLAN_TILES = 6      /* 256 x 256 tiles, W expanded inside the main loop                                  */
};
int hif4_gemm_plan(int a_kind, int experts, int64_t M_or_total_rows, int64_t N, int64_t K, int result_as_hif4,
                   size_t workspace_bytes);

/* Static host string naming a HIF4_PLAN_* value (the kernel's name in the sources). */
const char *hif4_gemm_plan_name(int plan);

/*
 * How a HIF4_PLAN_PLANES call of M rows and N columns is cut into launches (host function, nothing is launched).  One
 * workgroup per 256-row tile holds a compute unit, so a last round of tiles that is mostly empty costs a full one; the
 * library then runs whole rounds of 256-column tiles first and the remaining columns in narrower tiles that fill one
 * more round.  Every output keeps the order of its additions over K, so results do not depend on the cut.
 *   main_tile_columns  out: tile columns of 256 in the first launch (0: there is only one launch)
 *   tail_tile_width    out: tile width of the launch that takes the remaining columns: 256, 192 or 128
 * Returns HIF4_OK, HIF4_ERR_NULL or HIF4_ERR_SHAPE.
 */
int hif4_gemm_plan_planes_split(int64_t M, int64_t N, int *main_tile_columns, int *tail_tile_width);

/* Static host string naming a status code. */
const char *hif4_status_string(int status);

/* HIF4_VERSION of the built library (also the version of the packed layout). */
int hif4_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HIF4_H */
