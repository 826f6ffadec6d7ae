"""MXFP4 and NVFP4 fake-quantisers in plain numpy fp64 (test infrastructure).

They exist for one purpose: the quantisation-error comparison of Section III-A of
the HiF4 paper (MSE of HiF4 : NVFP4 : MXFP4 on Gaussian matrices), which pins the
HiF4 encoder statistically, and the SQNR figures the benchmark prints beside it.

MXFP4 (Section I of the paper; OCP Microscaling): groups of 32, a power-of-two
shared scale 2^(floor(log2 amax) - 2) (2 is the largest E2M1 exponent), E2M1
elements rounded to nearest-even and saturated at +-6.
NVFP4 (Section I / Section III-A): groups of 16, an FP8-E4M3 scale that brings the
group peak to 6, E2M1 elements; optionally per-tensor scaling (PTS) that first
brings the tensor peak to 2688 = 448 * 6.
"""
import numpy as np

_E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def round_e2m1(v):
    """Nearest E2M1 magnitude with ties to the even mantissa, saturating at 6; sign kept."""
    a = np.abs(v)
    out = np.empty_like(a)
    # below 2: spacing 0.5 (subnormal and first binade); [2,4): spacing 1; [4,6]: spacing 2
    lo = a < 2.0
    mid = (a >= 2.0) & (a < 4.0)
    hi = a >= 4.0
    out[lo] = np.rint(a[lo] * 2.0) / 2.0          # np.rint rounds half to even
    out[mid] = np.rint(a[mid])
    out[hi] = np.minimum(np.rint(a[hi] / 2.0) * 2.0, 6.0)
    return np.copysign(out, v)


def round_e4m3(v):
    """Nearest FP8-E4M3 (bias 7, subnormals, max 448, no inf) of non-negative v, ties to even."""
    v = np.asarray(v, dtype=np.float64)
    e = np.floor(np.log2(np.maximum(v, 2.0 ** -20)))
    e = np.maximum(e, -6.0)                        # subnormals share the spacing of 2^-6
    step = 2.0 ** (e - 3.0)
    return np.minimum(np.rint(v / step) * step, 448.0)


def mxfp4_fake_quant(x):
    """x: 2-D fp64, last dim a multiple of 32 -> dequantised fp64 of the same shape."""
    r, c = x.shape
    g = x.reshape(r, c // 32, 32)
    amax = np.abs(g).max(axis=2, keepdims=True)
    shared = np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - 2.0
    shared = np.clip(shared, -127.0, 127.0)
    scale = 2.0 ** shared
    q = round_e2m1(g / scale)
    return (q * scale).reshape(r, c)


def nvfp4_fake_quant(x, pts=False):
    """x: 2-D fp64, last dim a multiple of 16 -> dequantised fp64 of the same shape."""
    r, c = x.shape
    t = 1.0
    if pts:
        peak = np.abs(x).max()
        t = 2688.0 / peak if peak > 0 else 1.0
    g = (x * t).reshape(r, c // 16, 16)
    amax = np.abs(g).max(axis=2, keepdims=True)
    scale = round_e4m3(amax / 6.0)
    safe = np.where(scale > 0, scale, 1.0)
    q = round_e2m1(g / safe)
    deq = np.where(scale > 0, q * scale, 0.0)
    return deq.reshape(r, c) / t


def sqnr_db(x, xq):
    """10 log10( sum x^2 / sum (x - xq)^2 )."""
    num = float(np.sum(np.square(x)))
    den = float(np.sum(np.square(x - xq)))
    return float("inf") if den == 0 else 10.0 * np.log10(num / den)
