// C ABI of libhif4: host-side argument validation, then kernel launches on the
// caller's stream.  See include/hif4.h for the contract of every entry point.
#include <mutex>

#include "hif4_common.h"

#include "../../include/hif4_compare.h"

namespace hif4 {
int launch_encode(const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta, int mode,
                  hipStream_t stream);
int launch_encode_from(int in_dtype, const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta,
                       int mode, hipStream_t stream);
int launch_decode(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y, int64_t ldy,
                  hipStream_t stream);
int launch_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
                const uint32_t *w_meta, const int32_t *offs, int E, int64_t M, int64_t N, int64_t K, void *c,
                uint32_t *c_meta, int64_t ldc, int out_dtype, void *workspace, size_t workspace_bytes, hipStream_t stream);
int launch_fake_quant(int format, const void *x, int64_t rows, int64_t K, int64_t ldx, const uint32_t *tensor_peak, double *y,
                      double *sq_err, hipStream_t stream);
int launch_abs_max(const void *x, int64_t rows, int64_t K, int64_t ldx, uint32_t *peak, hipStream_t stream);
int launch_sq_err(const void *x, const void *y, int64_t rows, int64_t K, int64_t ldx, int64_t ldy, double *sq_err,
                  hipStream_t stream);
int launch_mxfp4_pack(const void *x, int64_t rows, int64_t K, int64_t ldx, void *cells, void *scales, hipStream_t stream);
int launch_mxfp4_gemm(const void *a_cells, const void *a_scales, const void *w_cells, const void *w_scales, int64_t M, int64_t N,
                      int64_t K, void *c, int64_t ldc, int out_dtype, hipStream_t stream);
int launch_mfma_loop(int kind, int iters, float *out, hipStream_t stream);
int gemm_plan(int a_kind, bool grouped, int E, int64_t M, int64_t N, int64_t K, int64_t lda, bool emit, bool ws_ok, size_t ws_bytes);
struct PlanesSplit {
    int main_tile_cols, tail_bn;
};
PlanesSplit planes_split(int64_t M, int64_t N);
size_t gemm_workspace_bytes(int a_kind, int64_t M, int64_t K);
size_t gemm_workspace_bytes_decoded_w(int a_kind, int64_t M, int64_t N, int64_t K);
} // namespace hif4

// Scratch of hif4_gemm_noalloc: device memory that belongs to the loaded library, one copy per GPU,
// held until the process ends.  In host code the name below stands for the symbol, not for a device
// address; the address on each device comes from hipGetSymbolAddress (noalloc_scratch()).
static __device__ __align__(256) unsigned char scratch[HIF4_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex scratch_lock;
void *scratch_ptr[MAX_DEVICES]; // device address of `scratch` on each GPU, once known

// Address of this library's scratch array on the current device; nullptr (and *status set) on failure.
void *noalloc_scratch(int *status)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        *status = HIF4_ERR_DEVICE;
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            *status = HIF4_ERR_DEVICE;
            return nullptr;
        }
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Limits that keep every index computation inside the kernels in range.
constexpr int64_t MAX_DIM = (int64_t)1 << 31;

int check_matrix_shape(int64_t rows, int64_t K, int64_t ld)
{
    if (rows < 0 || K < 0 || K % HIF4_UNIT != 0 || ld < K) return HIF4_ERR_SHAPE;
    if (rows >= MAX_DIM || K >= MAX_DIM || ld >= MAX_DIM) return HIF4_ERR_SHAPE;
    return HIF4_OK;
}

int check_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
               const uint32_t *w_meta, int64_t M, int64_t N, int64_t K, const void *c, int64_t ldc, int out_dtype,
               const void *workspace, size_t workspace_bytes)
{
    if (a_kind != HIF4_A_BF16_QUANTIZE && a_kind != HIF4_A_HIF4 && a_kind != HIF4_A_BF16_KEEP) return HIF4_ERR_UNSUPPORTED;
    if (out_dtype != HIF4_OUT_BF16 && out_dtype != HIF4_OUT_F32) return HIF4_ERR_UNSUPPORTED;
    if (M < 0 || N < 0 || K < 0 || K % HIF4_UNIT != 0 || ldc < N) return HIF4_ERR_SHAPE;
    if (M >= MAX_DIM || N >= MAX_DIM || K >= MAX_DIM || ldc >= MAX_DIM) return HIF4_ERR_SHAPE;
    if (a_kind != HIF4_A_HIF4 && (lda < K || lda >= MAX_DIM)) return HIF4_ERR_SHAPE;
    if (M == 0 || N == 0) return HIF4_OK;
    if (!c) return HIF4_ERR_NULL;
    if (K > 0) {
        if (!a || !w_codes || !w_meta) return HIF4_ERR_NULL;
        if (a_kind == HIF4_A_HIF4 && !a_meta) return HIF4_ERR_NULL;
    }
    if (!aligned(a, 16) || !aligned(w_codes, 16) || !aligned(w_meta, 4) || !aligned(a_meta, 4)) return HIF4_ERR_ALIGN;
    if (a_kind != HIF4_A_HIF4 && (lda % 8) != 0) return HIF4_ERR_ALIGN;
    if (!aligned(c, out_dtype == HIF4_OUT_BF16 ? 2 : 4)) return HIF4_ERR_ALIGN;
    const size_t need = hif4_gemm_workspace_bytes(a_kind, M, K);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return HIF4_ERR_WORKSPACE;
        if (!aligned(workspace, 16)) return HIF4_ERR_ALIGN;
    }
    return HIF4_OK;
}

} // namespace

extern "C" {

int hif4_quantize(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta,
                  int round_mode, void *stream)
{
    if (round_mode != HIF4_ROUND_RNE && round_mode != HIF4_ROUND_RHA) return HIF4_ERR_UNSUPPORTED;
    if (int rc = check_matrix_shape(rows, K, ldx)) return rc;
    if (rows == 0 || K == 0) return HIF4_OK;
    if (!x_bf16 || !codes || !meta) return HIF4_ERR_NULL;
    if (!aligned(x_bf16, 16) || (ldx % 8) != 0 || !aligned(codes, 16) || !aligned(meta, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_encode(x_bf16, rows, K, ldx, codes, meta, round_mode, static_cast<hipStream_t>(stream));
}

int hif4_quantize_from(int in_dtype, const void *x, int64_t rows, int64_t K, int64_t ldx, uint8_t *codes, uint32_t *meta,
                       int round_mode, void *stream)
{
    if (in_dtype != HIF4_IN_BF16 && in_dtype != HIF4_IN_F16 && in_dtype != HIF4_IN_F32) return HIF4_ERR_UNSUPPORTED;
    if (round_mode != HIF4_ROUND_RNE && round_mode != HIF4_ROUND_RHA) return HIF4_ERR_UNSUPPORTED;
    if (int rc = check_matrix_shape(rows, K, ldx)) return rc;
    if (rows == 0 || K == 0) return HIF4_OK;
    if (!x || !codes || !meta) return HIF4_ERR_NULL;
    const int64_t elems16 = in_dtype == HIF4_IN_F32 ? 4 : 8; // elements per 16 bytes
    if (!aligned(x, 16) || (ldx % elems16) != 0 || !aligned(codes, 16) || !aligned(meta, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_encode_from(in_dtype, x, rows, K, ldx, codes, meta, round_mode, static_cast<hipStream_t>(stream));
}

int hif4_dequantize(const uint8_t *codes, const uint32_t *meta, int64_t rows, int64_t K, void *y_bf16, int64_t ldy,
                    void *stream)
{
    if (int rc = check_matrix_shape(rows, K, ldy)) return rc;
    if (rows == 0 || K == 0) return HIF4_OK;
    if (!y_bf16 || !codes || !meta) return HIF4_ERR_NULL;
    if (!aligned(y_bf16, 16) || (ldy % 8) != 0 || !aligned(codes, 16) || !aligned(meta, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_decode(codes, meta, rows, K, y_bf16, ldy, static_cast<hipStream_t>(stream));
}

size_t hif4_gemm_workspace_bytes(int a_kind, int64_t M_or_total_rows, int64_t K)
{
    if (K % HIF4_UNIT != 0) return 0;
    return hif4::gemm_workspace_bytes(a_kind, M_or_total_rows, K);
}

size_t hif4_gemm_workspace_bytes_decoded_w(int a_kind, int64_t M, int64_t N, int64_t K)
{
    if (K % HIF4_UNIT != 0) return 0;
    return hif4::gemm_workspace_bytes_decoded_w(a_kind, M, N, K);
}

int hif4_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
              const uint32_t *w_meta, int64_t M, int64_t N, int64_t K, void *c, int64_t ldc, int out_dtype,
              void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, workspace, workspace_bytes))
        return rc;
    if (M == 0 || N == 0) return HIF4_OK;
    return hif4::launch_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, nullptr, 1, M, N, K, c, nullptr, ldc, out_dtype, workspace,
                             workspace_bytes, static_cast<hipStream_t>(stream));
}

int hif4_gemm_noalloc(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
                      const uint32_t *w_meta, int64_t M, int64_t N, int64_t K, void *c, int64_t ldc, int out_dtype, void *stream)
{
    // the scratch stands in for a workspace of exactly hif4_gemm_workspace_bytes() bytes: same checks, same kernels
    const size_t need = (K % HIF4_UNIT == 0) ? hif4::gemm_workspace_bytes(a_kind, M, K) : 0;
    if (need > (size_t)HIF4_NOALLOC_SCRATCH_BYTES) return HIF4_ERR_SCRATCH;
    // any non-null, aligned pointer passes the argument checks; the real one is fetched only if there is work
    alignas(16) static const unsigned char probe[16] = { 0 };
    if (int rc = check_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, M, N, K, c, ldc, out_dtype, need ? probe : nullptr, need))
        return rc;
    if (M == 0 || N == 0) return HIF4_OK;
    void *ws = nullptr;
    if (need) {
        int status = HIF4_OK;
        ws = noalloc_scratch(&status);
        if (!ws) return status;
    }
    return hif4::launch_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, nullptr, 1, M, N, K, c, nullptr, ldc, out_dtype, ws, need,
                             static_cast<hipStream_t>(stream));
}

size_t hif4_gemm_noalloc_max_bytes(void) { return (size_t)HIF4_NOALLOC_SCRATCH_BYTES; }

int hif4_gemm_to_hif4(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
                      const uint32_t *w_meta, int64_t M, int64_t N, int64_t K, uint8_t *c_codes, uint32_t *c_meta,
                      int round_mode, void *workspace, size_t workspace_bytes, void *stream)
{
    if (round_mode != HIF4_ROUND_RNE && round_mode != HIF4_ROUND_RHA) return HIF4_ERR_UNSUPPORTED;
    if (N % HIF4_UNIT != 0) return HIF4_ERR_SHAPE; // units of the result run along N
    // the other checks are those of hif4_gemm with a BF16 result of row stride N in place of the planes
    if (int rc = check_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, M, N, K, c_codes, N, HIF4_OUT_BF16, workspace, workspace_bytes))
        return rc;
    if (M == 0 || N == 0) return HIF4_OK;
    if (!c_meta) return HIF4_ERR_NULL;
    if (!aligned(c_codes, 16) || !aligned(c_meta, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, nullptr, 1, M, N, K, c_codes, c_meta, N, 16 + round_mode,
                             workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

int hif4_grouped_gemm(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
                      const uint32_t *w_meta, const int32_t *offs, int E, int64_t total_rows, int64_t N, int64_t K,
                      void *c, int64_t ldc, int out_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    if (E < 0) return HIF4_ERR_SHAPE;
    if (int rc = check_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, total_rows, N, K, c, ldc, out_dtype, workspace, workspace_bytes))
        return rc;
    if (total_rows == 0 || N == 0 || E == 0) return HIF4_OK;
    if (!offs) return HIF4_ERR_NULL;
    if (!aligned(offs, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, offs, E, total_rows, N, K, c, nullptr, ldc, out_dtype,
                             workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

int hif4_grouped_gemm_to_hif4(int a_kind, const void *a, const uint32_t *a_meta, int64_t lda, const uint8_t *w_codes,
                              const uint32_t *w_meta, const int32_t *offs, int E, int64_t total_rows, int64_t N, int64_t K,
                              uint8_t *c_codes, uint32_t *c_meta, int round_mode, void *workspace, size_t workspace_bytes, void *stream)
{
    if (round_mode != HIF4_ROUND_RNE && round_mode != HIF4_ROUND_RHA) return HIF4_ERR_UNSUPPORTED;
    if (E < 0 || N % HIF4_UNIT != 0) return HIF4_ERR_SHAPE; // units of the result run along N
    if (int rc = check_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, total_rows, N, K, c_codes, N, HIF4_OUT_BF16, workspace, workspace_bytes))
        return rc;
    if (total_rows == 0 || N == 0 || E == 0) return HIF4_OK;
    if (!c_meta || !offs) return HIF4_ERR_NULL;
    if (!aligned(c_codes, 16) || !aligned(c_meta, 4) || !aligned(offs, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_gemm(a_kind, a, a_meta, lda, w_codes, w_meta, offs, E, total_rows, N, K, c_codes, c_meta, N, 16 + round_mode,
                             workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

// ---- comparison tools (include/hif4_compare.h)

static int check_compare_matrix(const void *x, int64_t rows, int64_t K, int64_t ldx, int64_t group)
{
    if (rows < 0 || K < 0 || K % group != 0 || ldx < K || rows >= MAX_DIM || K >= MAX_DIM || ldx >= MAX_DIM) return HIF4_ERR_SHAPE;
    if (rows == 0 || K == 0) return HIF4_OK;
    if (!x) return HIF4_ERR_NULL;
    if (!aligned(x, 16) || (ldx % 8) != 0) return HIF4_ERR_ALIGN;
    return HIF4_OK;
}

int hif4cmp_mxfp4_fake_quant(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, double *y, double *sq_err, void *stream)
{
    if (int rc = check_compare_matrix(x_bf16, rows, K, ldx, 32)) return rc;
    if (!aligned(y, 8) || !aligned(sq_err, 8)) return HIF4_ERR_ALIGN;
    if (rows == 0 || K == 0) return HIF4_OK;
    return hif4::launch_fake_quant(0, x_bf16, rows, K, ldx, nullptr, y, sq_err, static_cast<hipStream_t>(stream));
}

int hif4cmp_nvfp4_fake_quant(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, const uint32_t *tensor_peak, double *y,
                             double *sq_err, void *stream)
{
    if (int rc = check_compare_matrix(x_bf16, rows, K, ldx, 16)) return rc;
    if (!aligned(y, 8) || !aligned(sq_err, 8) || !aligned(tensor_peak, 4)) return HIF4_ERR_ALIGN;
    if (rows == 0 || K == 0) return HIF4_OK;
    return hif4::launch_fake_quant(1, x_bf16, rows, K, ldx, tensor_peak, y, sq_err, static_cast<hipStream_t>(stream));
}

int hif4cmp_abs_max(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, uint32_t *peak, void *stream)
{
    if (int rc = check_compare_matrix(x_bf16, rows, K, ldx, 8)) return rc;
    if (rows == 0 || K == 0) return HIF4_OK;
    if (!peak) return HIF4_ERR_NULL;
    if (!aligned(peak, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_abs_max(x_bf16, rows, K, ldx, peak, static_cast<hipStream_t>(stream));
}

int hif4cmp_sq_err_bf16(const void *x_bf16, const void *y_bf16, int64_t rows, int64_t K, int64_t ldx, int64_t ldy,
                        double *sq_err, void *stream)
{
    if (int rc = check_compare_matrix(x_bf16, rows, K, ldx, 8)) return rc;
    if (int rc = check_compare_matrix(y_bf16, rows, K, ldy, 8)) return rc;
    if (rows == 0 || K == 0) return HIF4_OK;
    if (!sq_err) return HIF4_ERR_NULL;
    if (!aligned(sq_err, 8)) return HIF4_ERR_ALIGN;
    return hif4::launch_sq_err(x_bf16, y_bf16, rows, K, ldx, ldy, sq_err, static_cast<hipStream_t>(stream));
}

int hif4ref_mxfp4_pack(const void *x_bf16, int64_t rows, int64_t K, int64_t ldx, void *cells, void *scales, void *stream)
{
    if (int rc = check_compare_matrix(x_bf16, rows, K, ldx, 256)) return rc;
    if (rows == 0 || K == 0) return HIF4_OK;
    if (!cells || !scales) return HIF4_ERR_NULL;
    if (!aligned(cells, 16) || !aligned(scales, 16)) return HIF4_ERR_ALIGN;
    return hif4::launch_mxfp4_pack(x_bf16, rows, K, ldx, cells, scales, static_cast<hipStream_t>(stream));
}

int hif4ref_mxfp4_gemm(const void *a_cells, const void *a_scales, const void *w_cells, const void *w_scales, int64_t M,
                       int64_t N, int64_t K, void *c, int64_t ldc, int out_dtype, void *stream)
{
    if (out_dtype != HIF4_OUT_BF16 && out_dtype != HIF4_OUT_F32) return HIF4_ERR_UNSUPPORTED;
    if (M < 0 || N < 0 || K <= 0 || K % 256 != 0 || ldc < N) return HIF4_ERR_SHAPE;
    if (M >= MAX_DIM || N >= MAX_DIM || K >= MAX_DIM || ldc >= MAX_DIM) return HIF4_ERR_SHAPE;
    if (M == 0 || N == 0) return HIF4_OK;
    if (!a_cells || !a_scales || !w_cells || !w_scales || !c) return HIF4_ERR_NULL;
    if (!aligned(a_cells, 16) || !aligned(w_cells, 16) || !aligned(a_scales, 4) || !aligned(w_scales, 4)) return HIF4_ERR_ALIGN;
    if (!aligned(c, out_dtype == HIF4_OUT_BF16 ? 2 : 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_mxfp4_gemm(a_cells, a_scales, w_cells, w_scales, M, N, K, c, ldc, out_dtype, static_cast<hipStream_t>(stream));
}

int hif4ref_mfma_loop(int kind, int iters, float *out, void *stream)
{
    if (kind != 0 && kind != 1 && kind != 2) return HIF4_ERR_UNSUPPORTED;
    if (iters < 0 || iters > (1 << 24)) return HIF4_ERR_SHAPE;
    if (!out) return HIF4_ERR_NULL;
    if (!aligned(out, 4)) return HIF4_ERR_ALIGN;
    return hif4::launch_mfma_loop(kind, iters, out, static_cast<hipStream_t>(stream));
}

int hif4_gemm_plan(int a_kind, int experts, int64_t M, int64_t N, int64_t K, int result_as_hif4, size_t workspace_bytes)
{
    if (a_kind != HIF4_A_BF16_QUANTIZE && a_kind != HIF4_A_HIF4 && a_kind != HIF4_A_BF16_KEEP) return HIF4_ERR_UNSUPPORTED;
    if (experts < 0 || M < 0 || N < 0 || K < 0 || K % HIF4_UNIT != 0 || M >= MAX_DIM || N >= MAX_DIM || K >= MAX_DIM) return HIF4_ERR_SHAPE;
    if (result_as_hif4 && N % HIF4_UNIT != 0) return HIF4_ERR_SHAPE;
    if (workspace_bytes < hif4_gemm_workspace_bytes(a_kind, M, K)) return HIF4_ERR_WORKSPACE;
    return hif4::gemm_plan(a_kind, experts > 0, experts, M, N, K, K, result_as_hif4 != 0, workspace_bytes > 0, workspace_bytes);
}

int hif4_gemm_plan_planes_split(int64_t M, int64_t N, int *main_tile_columns, int *tail_tile_width)
{
    if (!main_tile_columns || !tail_tile_width) return HIF4_ERR_NULL;
    if (M < 0 || N < 0 || M >= MAX_DIM || N >= MAX_DIM) return HIF4_ERR_SHAPE;
    const hif4::PlanesSplit sp = hif4::planes_split(M, N);
    *main_tile_columns = sp.main_tile_cols;
    *tail_tile_width = sp.tail_bn;
    return HIF4_OK;
}

const char *hif4_gemm_plan_name(int plan)
{
    switch (plan) {
    case HIF4_PLAN_ZERO_FILL: return "hif4::zero_kernel";
    case HIF4_PLAN_FEWROWS: return "hif4::gemm_fewrows_kernel";
    case HIF4_PLAN_SKINNY: return "hif4::gemm_skinny_kernel";
    case HIF4_PLAN_STREAM: return "hif4::gemm_stream_kernel";
    case HIF4_PLAN_COLWAVE: return "hif4::gemm_colwave_kernel";
    case HIF4_PLAN_PLANES: return "hif4::gemm_planes16_kernel";
    case HIF4_PLAN_TILES: return "hif4::gemm_kernel";
    default: return "unknown plan";
    }
}

const char *hif4_status_string(int status)
{
    switch (status) {
    case HIF4_OK: return "ok";
    case HIF4_ERR_NULL: return "null pointer";
    case HIF4_ERR_SHAPE: return "bad shape (negative, K not a multiple of 64, leading dimension too small, or too large)";
    case HIF4_ERR_ALIGN: return "misaligned pointer or leading dimension";
    case HIF4_ERR_UNSUPPORTED: return "unsupported enum value";
    case HIF4_ERR_WORKSPACE: return "workspace missing or too small";
    case HIF4_ERR_DEVICE: return "HIP launch error";
    case HIF4_ERR_SCRATCH: return "call needs more scratch than the library's static buffer holds (hif4_gemm_noalloc_max_bytes)";
    default: return "unknown status";
    }
}

int hif4_version(void) { return HIF4_VERSION; }

} // extern "C"
