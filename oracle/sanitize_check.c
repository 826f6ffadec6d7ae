/*
 * Driver for the sanitizer build of the HiF4 CPU oracle — TEST INFRASTRUCTURE.
 *
 * Linked with hif4_oracle.c, both compiled with -fsanitize=address,undefined.  Reads a file of
 * inputs written by tests/test_oracle_sanitizers.py, runs every entry point of the oracle on
 * them and writes the results to a second file, which the test compares byte for byte with what
 * the ordinary build of the oracle returns for the same inputs.  Any report of a sanitizer ends
 * the run with a non-zero status.
 *
 * Input file:  int64 rows, int64 K, then rows*K BF16 patterns (uint16), rows*K floats,
 *              rows*K FP16 patterns (uint16).
 * Output file: for mode in {0, 1}: codes, meta of the BF16 matrix; decoded BF16; codes, meta
 *              of the FP32 and of the FP16 matrix; then the fp64 GEMM of the decoded matrix with
 *              itself (rows x rows doubles) and unit_dot of every unit of row 0 with row 1.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int hif4o_quantize(const uint16_t *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode);
int hif4o_quantize_from(int in_dtype, const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta,
                        int mode, uint16_t *as_bf16);
int hif4o_dequantize(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, uint16_t *y, int64_t ldy);
int hif4o_gemm_f64(const uint16_t *a, int64_t lda, const uint16_t *w, int64_t ldw, const int64_t *rows, int64_t nr,
                   const int64_t *cols, int64_t nc, int64_t K, double *c);
double hif4o_unit_dot(const uint8_t ca[32], uint32_t ma, const uint8_t cb[32], uint32_t mb);

static void *must(void *p)
{
    if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s inputs outputs\n", argv[0]); return 2; }
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) { fprintf(stderr, "cannot open files\n"); return 2; }
    int64_t rows, K;
    if (fread(&rows, 8, 1, in) != 1 || fread(&K, 8, 1, in) != 1 || rows < 2 || K < 64 || K % 64) return 2;
    const size_t n = (size_t)(rows * K), units = (size_t)(rows * (K / 64));
    uint16_t *xb = must(malloc(n * 2)), *xh = must(malloc(n * 2)), *y = must(malloc(n * 2)), *asb = must(malloc(n * 2));
    float *xf = must(malloc(n * 4));
    uint8_t *codes = must(malloc(n / 2));
    uint32_t *meta = must(malloc(units * 4));
    double *c = must(malloc((size_t)(rows * rows) * 8));
    if (fread(xb, 2, n, in) != n || fread(xf, 4, n, in) != n || fread(xh, 2, n, in) != n) return 2;
    for (int mode = 0; mode < 2; ++mode) {
        if (hif4o_quantize(xb, rows, K, K, codes, meta, mode)) return 4;
        fwrite(codes, 1, n / 2, out);
        fwrite(meta, 4, units, out);
        int rc = hif4o_dequantize(codes, meta, rows, K, y, K);
        if (rc != 0) return 4;
        fwrite(y, 2, n, out);
        if (hif4o_quantize_from(2, xf, rows, K, K, codes, meta, mode, asb)) return 4;
        fwrite(codes, 1, n / 2, out);
        fwrite(meta, 4, units, out);
        if (hif4o_quantize_from(1, xh, rows, K, K, codes, meta, mode, NULL)) return 4;
        fwrite(codes, 1, n / 2, out);
        fwrite(meta, 4, units, out);
    }
    if (hif4o_quantize(xb, rows, K, K, codes, meta, 0) || hif4o_dequantize(codes, meta, rows, K, y, K)) return 4;
    if (hif4o_gemm_f64(y, K, y, K, NULL, rows, NULL, rows, K, c)) return 4;
    fwrite(c, 8, (size_t)(rows * rows), out);
    for (int64_t u = 0; u < K / 64; ++u) {
        double d = hif4o_unit_dot(codes + u * 32, meta[u], codes + (K / 2) + u * 32, meta[K / 64 + u]);
        fwrite(&d, 8, 1, out);
    }
    fclose(in);
    if (fclose(out)) return 2;
    free(xb); free(xh); free(y); free(asb); free(xf); free(codes); free(meta); free(c);
    return 0;
}
