"""HiF4 CPU oracle (test infrastructure).

ctypes front end of ``hif4_oracle.c`` plus numpy comparators (MXFP4 / NVFP4) used
for the quantisation-error study of Section III-A of the paper.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` import
this package; it shares nothing with the GPU library.

All BF16 data crosses this interface as ``numpy.uint16`` bit patterns.
"""
import ctypes as C

import numpy as np

from .build import ensure_built

ROUND_RNE = 0
ROUND_RHA = 1

_lib = None


class Steps(C.Structure):
    """Mirror of the C record ``hif4o_steps``: every intermediate of Algorithm 1 for one unit."""
    _fields_ = [("V16", C.c_uint16 * 16), ("V8", C.c_uint16 * 8), ("Vmax", C.c_uint16), ("SF", C.c_uint16),
                ("E6M2", C.c_uint8), ("REC", C.c_uint16), ("P8", C.c_uint16 * 8), ("P16", C.c_uint16 * 16),
                ("E1_8", C.c_uint32), ("E1_16", C.c_uint32), ("scaled", C.c_uint16 * 64), ("S1P2", C.c_uint8 * 64),
                ("special", C.c_int)]


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(ensure_built())
        u8p, u16p, u32p = C.POINTER(C.c_uint8), C.POINTER(C.c_uint16), C.POINTER(C.c_uint32)
        i64p, f64p = C.POINTER(C.c_int64), C.POINTER(C.c_double)
        L.hif4o_bf16_to_f64.restype = C.c_double
        L.hif4o_bf16_to_f64.argtypes = [C.c_uint16]
        L.hif4o_f64_to_bf16.restype = C.c_uint16
        L.hif4o_f64_to_bf16.argtypes = [C.c_double, C.c_int]
        L.hif4o_bf16_mul.restype = C.c_uint16
        L.hif4o_bf16_mul.argtypes = [C.c_uint16, C.c_uint16, C.c_int]
        L.hif4o_e6m2_to_f64.restype = C.c_double
        L.hif4o_e6m2_to_f64.argtypes = [C.c_uint8]
        L.hif4o_bf16_to_e6m2.restype = C.c_uint8
        L.hif4o_bf16_to_e6m2.argtypes = [C.c_uint16, C.c_int]
        L.hif4o_e6m2_rec_to_bf16.restype = C.c_uint16
        L.hif4o_e6m2_rec_to_bf16.argtypes = [C.c_uint8]
        L.hif4o_to_s1p2.restype = C.c_uint8
        L.hif4o_to_s1p2.argtypes = [C.c_double, C.c_int, C.c_int]
        L.hif4o_encode_unit.restype = None
        L.hif4o_encode_unit.argtypes = [u16p, u8p, u32p, C.c_int]
        L.hif4o_decode_elem_f64.restype = C.c_double
        L.hif4o_decode_elem_f64.argtypes = [u8p, C.c_uint32, C.c_int]
        L.hif4o_decode_unit.restype = None
        L.hif4o_decode_unit.argtypes = [u8p, C.c_uint32, u16p, C.POINTER(C.c_int)]
        L.hif4o_quantize_from.restype = C.c_int
        L.hif4o_quantize_from.argtypes = [C.c_int, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, u8p, u32p, C.c_int, u16p]
        L.hif4o_encode_unit_steps.restype = None
        L.hif4o_encode_unit_steps.argtypes = [u16p, C.c_int, C.POINTER(Steps)]
        L.hif4o_f16_to_f64.restype = C.c_double
        L.hif4o_f16_to_f64.argtypes = [C.c_uint16]
        L.hif4o_quantize.restype = C.c_int
        L.hif4o_quantize.argtypes = [u16p, C.c_int64, C.c_int64, C.c_int64, u8p, u32p, C.c_int]
        L.hif4o_dequantize.restype = C.c_int
        L.hif4o_dequantize.argtypes = [u8p, u32p, C.c_int64, C.c_int64, u16p, C.c_int64]
        L.hif4o_gemm_f64.restype = C.c_int
        L.hif4o_gemm_f64.argtypes = [u16p, C.c_int64, u16p, C.c_int64, i64p, C.c_int64, i64p, C.c_int64,
                                     C.c_int64, f64p]
        L.hif4o_unit_dot.restype = C.c_double
        L.hif4o_unit_dot.argtypes = [u8p, C.c_uint32, u8p, C.c_uint32]
        L.hif4o_num_threads.restype = C.c_int
        L.hif4o_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _u16_matrix(x):
    x = np.asarray(x)
    if x.dtype != np.uint16 or x.ndim != 2 or x.strides[1] != 2 or x.strides[0] % 2:
        raise ValueError("expected a 2-D uint16 (BF16 bit pattern) array with contiguous rows")
    return x


# ---- scalar steps (exposed so that each can be pinned on its own) ----------------

def bf16_to_f64(b):
    return lib().hif4o_bf16_to_f64(int(b))


def f64_to_bf16(v, mode=ROUND_RNE):
    return lib().hif4o_f64_to_bf16(float(v), mode)


def bf16_mul(a, b, mode=ROUND_RNE):
    return lib().hif4o_bf16_mul(int(a), int(b), mode)


def e6m2_to_f64(byte):
    return lib().hif4o_e6m2_to_f64(int(byte))


def bf16_to_e6m2(sf, mode=ROUND_RNE):
    return lib().hif4o_bf16_to_e6m2(int(sf), mode)


def e6m2_rec_to_bf16(byte):
    return lib().hif4o_e6m2_rec_to_bf16(int(byte))


def to_s1p2(scaled, negative, mode=ROUND_RNE):
    return lib().hif4o_to_s1p2(float(scaled), int(bool(negative)), mode)


# ---- units -------------------------------------------------------------------------

def encode_unit(x64, mode=ROUND_RNE):
    """Algorithm 1 on 64 BF16 patterns -> (codes uint8[32], meta int)."""
    x = np.ascontiguousarray(x64, dtype=np.uint16)
    assert x.shape == (64,)
    codes = np.zeros(32, np.uint8)
    meta = C.c_uint32(0)
    lib().hif4o_encode_unit(_ptr(x, C.c_uint16), _ptr(codes, C.c_uint8), C.byref(meta), mode)
    return codes, int(meta.value)


def encode_unit_steps(x64, mode=ROUND_RNE):
    """Algorithm 1 on 64 BF16 patterns -> dict of every intermediate, under the paper's names."""
    x = np.ascontiguousarray(x64, dtype=np.uint16)
    assert x.shape == (64,)
    t = Steps()
    lib().hif4o_encode_unit_steps(_ptr(x, C.c_uint16), mode, C.byref(t))
    out = {}
    for name, _ in Steps._fields_:
        v = getattr(t, name)
        out[name] = int(v) if isinstance(v, int) else np.array(list(v), dtype=np.uint32)
    return out


def decode_unit(codes, meta):
    """Eq. 2 on one unit -> uint16[64] BF16 patterns (raises if any value were inexact)."""
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    assert c.shape == (32,)
    y = np.zeros(64, np.uint16)
    inexact = C.c_int(0)
    lib().hif4o_decode_unit(_ptr(c, C.c_uint8), int(meta), _ptr(y, C.c_uint16), C.byref(inexact))
    if inexact.value:
        raise ArithmeticError("HiF4 value not exact in BF16")
    return y


def decode_elem_f64(codes, meta, i):
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    return lib().hif4o_decode_elem_f64(_ptr(c, C.c_uint8), int(meta), int(i))


def unit_dot(codes_a, meta_a, codes_b, meta_b):
    """Eq. 4 on one pair of units."""
    a = np.ascontiguousarray(codes_a, dtype=np.uint8)
    b = np.ascontiguousarray(codes_b, dtype=np.uint8)
    return lib().hif4o_unit_dot(_ptr(a, C.c_uint8), int(meta_a), _ptr(b, C.c_uint8), int(meta_b))


# ---- matrices ----------------------------------------------------------------------

def quantize(x, mode=ROUND_RNE):
    """rows x K BF16 patterns -> (codes uint8[rows, K/2], meta uint32[rows, K/64])."""
    x = _u16_matrix(x)
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), np.uint8)
    meta = np.zeros((rows, K // 64), np.uint32)
    rc = lib().hif4o_quantize(_ptr(x, C.c_uint16), rows, K, x.strides[0] // 2,
                              _ptr(codes, C.c_uint8), _ptr(meta, C.c_uint32), mode)
    if rc:
        raise ValueError(f"hif4o_quantize failed: {rc}")
    return codes, meta


def quantize_from(x, mode=ROUND_RNE, return_bf16=False):
    """rows x K float32 or float16 matrix (numpy) -> planes: every input is rounded to BF16 first.
    return_bf16: also return those rounded inputs (uint16 patterns)."""
    x = np.ascontiguousarray(x)
    assert x.ndim == 2 and x.dtype in (np.float32, np.float16)
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), np.uint8)
    meta = np.zeros((rows, K // 64), np.uint32)
    in_dtype = 2 if x.dtype == np.float32 else 1
    xb = np.zeros((rows, K), np.uint16) if return_bf16 else None
    rc = lib().hif4o_quantize_from(in_dtype, x.ctypes.data_as(C.c_void_p), rows, K, K,
                                   _ptr(codes, C.c_uint8), _ptr(meta, C.c_uint32), mode,
                                   _ptr(xb, C.c_uint16) if return_bf16 else None)
    if rc:
        raise ValueError(f"hif4o_quantize_from failed: {rc}")
    return (codes, meta, xb) if return_bf16 else (codes, meta)


def f16_to_f64(h):
    return lib().hif4o_f16_to_f64(int(h))


def dequantize(codes, meta):
    """planes -> rows x K BF16 patterns (uint16)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.uint32)
    rows, K = codes.shape[0], codes.shape[1] * 2
    assert meta.shape == (rows, K // 64)
    y = np.zeros((rows, K), np.uint16)
    rc = lib().hif4o_dequantize(_ptr(codes, C.c_uint8), _ptr(meta, C.c_uint32), rows, K, _ptr(y, C.c_uint16), K)
    if rc:
        raise ArithmeticError(f"hif4o_dequantize failed: {rc}")
    return y


def gemm_f64(a, w, rows=None, cols=None):
    """C = a[rows] @ w[cols].T in fp64; a, w are BF16 patterns (rows x K, K-contiguous)."""
    a, w = _u16_matrix(a), _u16_matrix(w)
    K = a.shape[1]
    assert w.shape[1] == K
    r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    c = None if cols is None else np.ascontiguousarray(cols, dtype=np.int64)
    nr = a.shape[0] if r is None else r.size
    nc = w.shape[0] if c is None else c.size
    if r is not None and r.size and (r.min() < 0 or r.max() >= a.shape[0]):
        raise IndexError("row index out of range")
    if c is not None and c.size and (c.min() < 0 or c.max() >= w.shape[0]):
        raise IndexError("column index out of range")
    out = np.zeros((nr, nc), np.float64)
    rc = lib().hif4o_gemm_f64(_ptr(a, C.c_uint16), a.strides[0] // 2, _ptr(w, C.c_uint16), w.strides[0] // 2,
                              None if r is None else _ptr(r, C.c_int64), nr,
                              None if c is None else _ptr(c, C.c_int64), nc, K, _ptr(out, C.c_double))
    if rc:
        raise ValueError(f"hif4o_gemm_f64 failed: {rc}")
    return out


def bf16_bits_to_f64(bits):
    """Vectorised exact widening of BF16 patterns (numpy only; no rounding involved)."""
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def num_threads():
    return lib().hif4o_num_threads()


def set_num_threads(n):
    lib().hif4o_set_num_threads(int(n))
