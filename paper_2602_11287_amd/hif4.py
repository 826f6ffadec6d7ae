"""Thin Python binding of the libhif4 C ABI (see include/hif4.h).

Argument marshalling only: every step of the HiF4 path runs in the HIP kernels of
``libhif4.so``.  PyTorch supplies device memory and the current stream.  There is
no CPU fallback: if the shared library is missing, loading raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhif4.so")

HIF4_OK = 0
HIF4_ERR_NULL, HIF4_ERR_SHAPE, HIF4_ERR_ALIGN = -1, -2, -3
HIF4_ERR_UNSUPPORTED, HIF4_ERR_WORKSPACE, HIF4_ERR_DEVICE, HIF4_ERR_SCRATCH = -4, -5, -6, -7
HIF4_ROUND_RNE, HIF4_ROUND_RHA = 0, 1
HIF4_A_BF16_QUANTIZE, HIF4_A_HIF4, HIF4_A_BF16_KEEP = 0, 1, 2
HIF4_OUT_BF16, HIF4_OUT_F32 = 0, 1
HIF4_PLAN_ZERO_FILL = 0

EXPORTS = ["hif4_quantize", "hif4_quantize_from", "hif4_dequantize", "hif4_gemm", "hif4_gemm_to_hif4", "hif4_grouped_gemm",
           "hif4_gemm_noalloc", "hif4_gemm_noalloc_max_bytes", "hif4_grouped_gemm_to_hif4", "hif4_gemm_plan", "hif4_gemm_plan_name", "hif4_gemm_plan_planes_split",
           "hif4_gemm_workspace_bytes", "hif4_gemm_workspace_bytes_decoded_w", "hif4_status_string", "hif4_version",
           "hif4cmp_mxfp4_fake_quant", "hif4cmp_nvfp4_fake_quant", "hif4cmp_abs_max", "hif4cmp_sq_err_bf16",
           "hif4ref_mxfp4_pack", "hif4ref_mxfp4_gemm", "hif4ref_mfma_loop"]


class Hif4Error(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {hif4_status_string(status)} ({status})")


_lib = None


def load():
    """Load libhif4.so (built in-tree by paper_2602_11287_amd/build.py); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
        L.hif4_quantize.restype = i32
        L.hif4_quantize.argtypes = [vp, i64, i64, i64, vp, vp, i32, vp]
        L.hif4_quantize_from.restype = i32
        L.hif4_quantize_from.argtypes = [i32, vp, i64, i64, i64, vp, vp, i32, vp]
        L.hif4_dequantize.restype = i32
        L.hif4_dequantize.argtypes = [vp, vp, i64, i64, vp, i64, vp]
        L.hif4_gemm.restype = i32
        L.hif4_gemm.argtypes = [i32, vp, vp, i64, vp, vp, i64, i64, i64, vp, i64, i32, vp, sz, vp]
        L.hif4_gemm_to_hif4.restype = i32
        L.hif4_gemm_to_hif4.argtypes = [i32, vp, vp, i64, vp, vp, i64, i64, i64, vp, vp, i32, vp, sz, vp]
        L.hif4_grouped_gemm.restype = i32
        L.hif4_grouped_gemm.argtypes = [i32, vp, vp, i64, vp, vp, vp, i32, i64, i64, i64, vp, i64, i32, vp, sz, vp]
        L.hif4_grouped_gemm_to_hif4.restype = i32
        L.hif4_grouped_gemm_to_hif4.argtypes = [i32, vp, vp, i64, vp, vp, vp, i32, i64, i64, i64, vp, vp, i32, vp, sz, vp]
        L.hif4_gemm_plan.restype = i32
        L.hif4_gemm_plan.argtypes = [i32, i32, i64, i64, i64, i32, sz]
        L.hif4_gemm_plan_name.restype = C.c_char_p
        L.hif4_gemm_plan_name.argtypes = [i32]
        L.hif4_gemm_plan_planes_split.restype = i32
        L.hif4_gemm_plan_planes_split.argtypes = [i64, i64, C.POINTER(i32), C.POINTER(i32)]
        L.hif4_gemm_noalloc.restype = i32
        L.hif4_gemm_noalloc.argtypes = [i32, vp, vp, i64, vp, vp, i64, i64, i64, vp, i64, i32, vp]
        L.hif4_gemm_noalloc_max_bytes.restype = sz
        L.hif4_gemm_noalloc_max_bytes.argtypes = []
        L.hif4_gemm_workspace_bytes.restype = sz
        L.hif4_gemm_workspace_bytes.argtypes = [i32, i64, i64]
        L.hif4_gemm_workspace_bytes_decoded_w.restype = sz
        L.hif4_gemm_workspace_bytes_decoded_w.argtypes = [i32, i64, i64, i64]
        L.hif4cmp_mxfp4_fake_quant.restype = i32
        L.hif4cmp_mxfp4_fake_quant.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        L.hif4cmp_nvfp4_fake_quant.restype = i32
        L.hif4cmp_nvfp4_fake_quant.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
        L.hif4cmp_abs_max.restype = i32
        L.hif4cmp_abs_max.argtypes = [vp, i64, i64, i64, vp, vp]
        L.hif4cmp_sq_err_bf16.restype = i32
        L.hif4cmp_sq_err_bf16.argtypes = [vp, vp, i64, i64, i64, i64, vp, vp]
        L.hif4ref_mxfp4_pack.restype = i32
        L.hif4ref_mxfp4_pack.argtypes = [vp, i64, i64, i64, vp, vp, vp]
        L.hif4ref_mxfp4_gemm.restype = i32
        L.hif4ref_mxfp4_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, i64, i32, vp]
        L.hif4ref_mfma_loop.restype = i32
        L.hif4ref_mfma_loop.argtypes = [i32, i32, vp, vp]
        L.hif4_status_string.restype = C.c_char_p
        L.hif4_status_string.argtypes = [i32]
        L.hif4_version.restype = i32
        L.hif4_version.argtypes = []
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status, where):
    if status != HIF4_OK:
        raise Hif4Error(status, where)


def hif4_version():
    return load().hif4_version()


def hif4_status_string(status):
    return load().hif4_status_string(int(status)).decode()


def hif4_gemm_workspace_bytes(a_kind, rows, K):
    return int(load().hif4_gemm_workspace_bytes(int(a_kind), int(rows), int(K)))


def hif4_gemm_plan(a_kind, M, N, K, experts=0, result_as_hif4=False, workspace_bytes=None):
    """HIF4_PLAN_* value of the main loop a call with these arguments runs (workspace_bytes None: the mandatory size)."""
    if workspace_bytes is None:
        workspace_bytes = hif4_gemm_workspace_bytes(a_kind, M, K)
    plan = load().hif4_gemm_plan(int(a_kind), int(experts), int(M), int(N), int(K), int(bool(result_as_hif4)), int(workspace_bytes))
    _check(min(plan, 0), "hif4_gemm_plan")
    return plan


def hif4_gemm_plan_name(plan):
    return load().hif4_gemm_plan_name(int(plan)).decode()


def hif4_gemm_plan_planes_split(M, N):
    """(tile columns of 256 in the first launch, tile width of the launch for the remaining columns) of a HIF4_PLAN_PLANES call."""
    main, width = C.c_int(0), C.c_int(0)
    _check(load().hif4_gemm_plan_planes_split(int(M), int(N), C.byref(main), C.byref(width)), "hif4_gemm_plan_planes_split")
    return main.value, width.value


def hif4_gemm_workspace_bytes_decoded_w(a_kind, M, N, K):
    return int(load().hif4_gemm_workspace_bytes_decoded_w(int(a_kind), int(M), int(N), int(K)))


def hif4_quantize(x, codes=None, meta=None, round_mode=HIF4_ROUND_RNE, stream=None):
    """x: CUDA bfloat16 [rows, K] (rows may be strided) -> (codes uint8 [rows, K/2], meta int32 [rows, K/64])."""
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    rows, K = x.shape
    if codes is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
    if meta is None:
        meta = torch.empty((rows, K // 64), dtype=torch.int32, device=x.device)
    ldx = x.stride(0) if rows > 1 else max(x.stride(0), K)
    _check(load().hif4_quantize(_ptr(x), rows, K, ldx, _ptr(codes), _ptr(meta), round_mode, _stream(stream)),
           "hif4_quantize")
    return codes, meta


_IN_DTYPES = {torch.bfloat16: 0, torch.float16: 1, torch.float32: 2}


def hif4_quantize_from(x, codes=None, meta=None, round_mode=HIF4_ROUND_RNE, stream=None):
    """As hif4_quantize for a CUDA bfloat16, float16 or float32 matrix (in_dtype from x.dtype)."""
    assert x.is_cuda and x.dtype in _IN_DTYPES and x.dim() == 2 and x.stride(1) == 1
    rows, K = x.shape
    if codes is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
    if meta is None:
        meta = torch.empty((rows, K // 64), dtype=torch.int32, device=x.device)
    ldx = x.stride(0) if rows > 1 else max(x.stride(0), K)
    _check(load().hif4_quantize_from(_IN_DTYPES[x.dtype], _ptr(x), rows, K, ldx, _ptr(codes), _ptr(meta), round_mode,
                                     _stream(stream)), "hif4_quantize_from")
    return codes, meta


def hif4_dequantize(codes, meta, y=None, stream=None):
    """codes uint8 [rows, K/2], meta int32 [rows, K/64] -> CUDA bfloat16 [rows, K]."""
    assert codes.is_cuda and codes.dtype == torch.uint8 and codes.is_contiguous()
    assert meta.dtype == torch.int32 and meta.is_contiguous()
    rows, K = codes.shape[0], codes.shape[1] * 2
    if y is None:
        y = torch.empty((rows, K), dtype=torch.bfloat16, device=codes.device)
    ldy = y.stride(0) if rows > 1 else max(y.stride(0), K)
    _check(load().hif4_dequantize(_ptr(codes), _ptr(meta), rows, K, _ptr(y), ldy, _stream(stream)), "hif4_dequantize")
    return y


def _gemm_common(a_kind, a, a_meta, w_codes, M, K):
    assert w_codes.dtype == torch.uint8 and w_codes.is_contiguous() and w_codes.shape[-1] * 2 == K
    if a_kind == HIF4_A_HIF4:
        assert a.dtype == torch.uint8 and a.is_contiguous() and a_meta is not None
        return K
    assert a.dtype == torch.bfloat16 and a.stride(1) == 1
    return a.stride(0) if M > 1 else max(a.stride(0), K)


def hif4_gemm(a_kind, a, a_meta, w_codes, w_meta, out_dtype=HIF4_OUT_BF16, c=None, workspace=None, stream=None):
    """C[M, N] = A[M, K] @ W[N, K]^T, W (and for W4A4 also A) in HiF4; fp32 accumulation."""
    M = a.shape[0]
    K = a.shape[1] * 2 if a_kind == HIF4_A_HIF4 else a.shape[1]
    N = w_codes.shape[0]
    lda = _gemm_common(a_kind, a, a_meta, w_codes, M, K)
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16 if out_dtype == HIF4_OUT_BF16 else torch.float32, device=a.device)
    need = hif4_gemm_workspace_bytes_decoded_w(a_kind, M, N, K)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
    wsz = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ldc = c.stride(0) if M > 1 else max(c.stride(0), N)
    _check(load().hif4_gemm(a_kind, _ptr(a), _ptr(a_meta), lda, _ptr(w_codes), _ptr(w_meta), M, N, K, _ptr(c), ldc,
                            out_dtype, _ptr(workspace), wsz, _stream(stream)), "hif4_gemm")
    return c


def hif4_gemm_noalloc(a_kind, a, a_meta, w_codes, w_meta, out_dtype=HIF4_OUT_BF16, c=None, stream=None):
    """hif4_gemm on the library's own static scratch: no workspace argument, nothing allocated by the call
    (c must be given by callers that may not allocate; it is created here only as a convenience)."""
    M = a.shape[0]
    K = a.shape[1] * 2 if a_kind == HIF4_A_HIF4 else a.shape[1]
    N = w_codes.shape[0]
    lda = _gemm_common(a_kind, a, a_meta, w_codes, M, K)
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16 if out_dtype == HIF4_OUT_BF16 else torch.float32, device=a.device)
    ldc = c.stride(0) if M > 1 else max(c.stride(0), N)
    _check(load().hif4_gemm_noalloc(a_kind, _ptr(a), _ptr(a_meta), lda, _ptr(w_codes), _ptr(w_meta), M, N, K, _ptr(c), ldc,
                                    out_dtype, _stream(stream)), "hif4_gemm_noalloc")
    return c


def hif4_gemm_noalloc_max_bytes():
    return int(load().hif4_gemm_noalloc_max_bytes())


def hif4_gemm_to_hif4(a_kind, a, a_meta, w_codes, w_meta, round_mode=HIF4_ROUND_RNE, c_codes=None, c_meta=None,
                      workspace=None, stream=None):
    """As hif4_gemm, the result leaving as HiF4 planes (codes uint8 [M, N/2], meta int32 [M, N/64]), units along N."""
    M = a.shape[0]
    K = a.shape[1] * 2 if a_kind == HIF4_A_HIF4 else a.shape[1]
    N = w_codes.shape[0]
    lda = _gemm_common(a_kind, a, a_meta, w_codes, M, K)
    if c_codes is None:
        c_codes = torch.empty((M, N // 2), dtype=torch.uint8, device=a.device)
    if c_meta is None:
        c_meta = torch.empty((M, N // 64), dtype=torch.int32, device=a.device)
    need = hif4_gemm_workspace_bytes_decoded_w(a_kind, M, N, K)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
    wsz = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().hif4_gemm_to_hif4(a_kind, _ptr(a), _ptr(a_meta), lda, _ptr(w_codes), _ptr(w_meta), M, N, K,
                                    _ptr(c_codes), _ptr(c_meta), round_mode, _ptr(workspace), wsz, _stream(stream)),
           "hif4_gemm_to_hif4")
    return c_codes, c_meta


def hif4_grouped_gemm(a_kind, a, a_meta, w_codes, w_meta, offs, out_dtype=HIF4_OUT_BF16, c=None, workspace=None,
                      stream=None):
    """Rows of A sorted by expert; expert e owns rows offs[e]..offs[e+1]-1 and weights w_codes[e] ([E, N, K/2])."""
    M = a.shape[0]
    K = a.shape[1] * 2 if a_kind == HIF4_A_HIF4 else a.shape[1]
    E, N = w_codes.shape[0], w_codes.shape[1]
    assert offs.dtype == torch.int32 and offs.is_cuda and offs.numel() == E + 1
    lda = _gemm_common(a_kind, a, a_meta, w_codes, M, K)
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16 if out_dtype == HIF4_OUT_BF16 else torch.float32, device=a.device)
    need = hif4_gemm_workspace_bytes(a_kind, M, K)
    if a_kind == HIF4_A_BF16_KEEP:
        need = M * K * 2  # optional: room for a reordered copy of A selects the faster kernel
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
    wsz = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ldc = c.stride(0) if M > 1 else max(c.stride(0), N)
    _check(load().hif4_grouped_gemm(a_kind, _ptr(a), _ptr(a_meta), lda, _ptr(w_codes), _ptr(w_meta), _ptr(offs), E, M,
                                    N, K, _ptr(c), ldc, out_dtype, _ptr(workspace), wsz, _stream(stream)),
           "hif4_grouped_gemm")
    return c


def hif4_grouped_gemm_to_hif4(a_kind, a, a_meta, w_codes, w_meta, offs, round_mode=HIF4_ROUND_RNE, c_codes=None, c_meta=None,
                              workspace=None, stream=None):
    """As hif4_grouped_gemm, the result leaving as HiF4 planes (codes uint8 [M, N/2], meta int32 [M, N/64]), units along N."""
    M = a.shape[0]
    K = a.shape[1] * 2 if a_kind == HIF4_A_HIF4 else a.shape[1]
    E, N = w_codes.shape[0], w_codes.shape[1]
    assert offs.dtype == torch.int32 and offs.is_cuda and offs.numel() == E + 1
    lda = _gemm_common(a_kind, a, a_meta, w_codes, M, K)
    if c_codes is None:
        c_codes = torch.empty((M, N // 2), dtype=torch.uint8, device=a.device)
    if c_meta is None:
        c_meta = torch.empty((M, N // 64), dtype=torch.int32, device=a.device)
    need = hif4_gemm_workspace_bytes(a_kind, M, K)
    if a_kind == HIF4_A_BF16_KEEP:
        need = M * K * 2  # optional: room for a reordered copy of A selects the faster kernel
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
    wsz = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().hif4_grouped_gemm_to_hif4(a_kind, _ptr(a), _ptr(a_meta), lda, _ptr(w_codes), _ptr(w_meta), _ptr(offs), E, M,
                                            N, K, _ptr(c_codes), _ptr(c_meta), round_mode, _ptr(workspace), wsz, _stream(stream)),
           "hif4_grouped_gemm_to_hif4")
    return c_codes, c_meta


# ---- comparison tools of include/hif4_compare.h (quantisation-error study, Section III-A) -------------

def _cmp_matrix(x):
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    rows, K = x.shape
    return rows, K, (x.stride(0) if rows > 1 else max(x.stride(0), K))


def hif4cmp_mxfp4_fake_quant(x, y=None, sq_err=None, stream=None):
    """x CUDA bfloat16 [rows, K]; y float64 [rows, K] or None; sq_err float64 [1] (added to) or None."""
    rows, K, ldx = _cmp_matrix(x)
    _check(load().hif4cmp_mxfp4_fake_quant(_ptr(x), rows, K, ldx, _ptr(y), _ptr(sq_err), _stream(stream)),
           "hif4cmp_mxfp4_fake_quant")
    return y


def hif4cmp_nvfp4_fake_quant(x, tensor_peak=None, y=None, sq_err=None, stream=None):
    """tensor_peak: int32 [1] written by hif4cmp_abs_max (per-tensor scaling) or None (direct cast)."""
    rows, K, ldx = _cmp_matrix(x)
    _check(load().hif4cmp_nvfp4_fake_quant(_ptr(x), rows, K, ldx, _ptr(tensor_peak), _ptr(y), _ptr(sq_err),
                                           _stream(stream)), "hif4cmp_nvfp4_fake_quant")
    return y


def hif4cmp_abs_max(x, peak, stream=None):
    """peak: int32 [1], zeroed by the caller; receives the BF16 pattern of max|x|."""
    rows, K, ldx = _cmp_matrix(x)
    _check(load().hif4cmp_abs_max(_ptr(x), rows, K, ldx, _ptr(peak), _stream(stream)), "hif4cmp_abs_max")
    return peak


def hif4cmp_sq_err_bf16(x, y, sq_err, stream=None):
    rows, K, ldx = _cmp_matrix(x)
    _, _, ldy = _cmp_matrix(y)
    assert y.shape == x.shape
    _check(load().hif4cmp_sq_err_bf16(_ptr(x), _ptr(y), rows, K, ldx, ldy, _ptr(sq_err), _stream(stream)),
           "hif4cmp_sq_err_bf16")
    return sq_err


def hif4ref_mxfp4_pack(x, stream=None):
    """CUDA bfloat16 [rows, K], K % 256 == 0 -> (cells uint8 [K/32, rows, 16], scales uint8 [K/128, rows, 4])."""
    rows, K, ldx = _cmp_matrix(x)
    cells = torch.empty((K // 32, rows, 16), dtype=torch.uint8, device=x.device)
    scales = torch.empty((K // 128, rows, 4), dtype=torch.uint8, device=x.device)
    _check(load().hif4ref_mxfp4_pack(_ptr(x), rows, K, ldx, _ptr(cells), _ptr(scales), _stream(stream)), "hif4ref_mxfp4_pack")
    return cells, scales


def hif4ref_mxfp4_gemm(a_cells, a_scales, w_cells, w_scales, out_dtype=HIF4_OUT_BF16, c=None, stream=None):
    """Speed reference on the native MXFP4 matrix instruction; operands from hif4ref_mxfp4_pack."""
    M, N, K = a_cells.shape[1], w_cells.shape[1], a_cells.shape[0] * 32
    assert w_cells.shape[0] * 32 == K
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16 if out_dtype == HIF4_OUT_BF16 else torch.float32, device=a_cells.device)
    ldc = c.stride(0) if M > 1 else max(c.stride(0), N)
    _check(load().hif4ref_mxfp4_gemm(_ptr(a_cells), _ptr(a_scales), _ptr(w_cells), _ptr(w_scales), M, N, K, _ptr(c), ldc,
                                     out_dtype, _stream(stream)), "hif4ref_mxfp4_gemm")
    return c


def hif4ref_mfma_loop(kind, iters, out, stream=None):
    """out: CUDA float32 [131072]; returns the flop count of the launch."""
    assert out.is_cuda and out.dtype == torch.float32 and out.numel() >= 131072
    _check(load().hif4ref_mfma_loop(int(kind), int(iters), _ptr(out), _stream(stream)), "hif4ref_mfma_loop")
    return 2048 * int(iters) * 8 * (131072 if kind == 1 else 32768)
