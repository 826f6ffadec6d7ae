"""Pins of the oracle's GEMM: Eq. 4 (Section III-B) in its printed nesting equals the
fp64 dot of the decoded values; the matrix product reduces to numpy's matmul and, for
units with unit scale and clear micro-exponents, to an exact integer product."""
import numpy as np

from layout import codes_to_nibbles
from paper_2602_11287_amd import synth


def rand_packed(rng, rows, K, byte_lo=40, byte_hi=60):
    codes = rng.integers(0, 256, (rows, K // 2), dtype=np.uint8)
    meta = rng.integers(0, 2 ** 24, (rows, K // 64)).astype(np.uint32) << 8
    meta |= rng.integers(byte_lo << 2, byte_hi << 2, (rows, K // 64)).astype(np.uint32)
    return codes, meta


def test_eq4_equals_dot_of_decoded_values(oracle):
    rng = np.random.default_rng(21)
    ca, ma = rand_packed(rng, 300, 64, 0, 63)
    cb, mb = rand_packed(rng, 300, 64, 0, 63)
    da = oracle.bf16_bits_to_f64(oracle.dequantize(ca, ma))
    db = oracle.bf16_bits_to_f64(oracle.dequantize(cb, mb))
    for r in range(300):
        d = oracle.unit_dot(ca[r], int(ma[r, 0]), cb[r], int(mb[r, 0]))
        # 64 products of 6-bit x 6-bit significands sum exactly in fp64 within one unit pair
        assert d == float(np.sum(da[r] * db[r]))
        # and a 1 x 1 x 64 GEMM is Eq. 4 itself
        g = oracle.gemm_f64(oracle.dequantize(ca[r:r + 1], ma[r:r + 1]), oracle.dequantize(cb[r:r + 1], mb[r:r + 1]))
        assert g[0, 0] == d


def test_eq4_integer_width(oracle):
    """The 64-term integer sum of Eq. 4 fits the S12P4 result the paper names: |sum| <= 64*49/16... in 1/16 units."""
    codes = np.full(32, 0x77, np.uint8)
    meta = (0xFFFF << 16) | (0xFF << 8) | (48 << 2)
    d = oracle.unit_dot(codes, meta, codes, meta)
    assert d == 64 * 7.0 * 7.0 and d * 16 < 2 ** 16  # 12 integer bits + 4 fraction bits


def test_gemm_matches_numpy_matmul(oracle):
    rng = np.random.default_rng(22)
    ca, ma = rand_packed(rng, 37, 320)
    cw, mw = rand_packed(rng, 53, 320)
    a, w = oracle.dequantize(ca, ma), oracle.dequantize(cw, mw)
    got = oracle.gemm_f64(a, w)
    want = oracle.bf16_bits_to_f64(a) @ oracle.bf16_bits_to_f64(w).T
    assert np.abs(got - want).max() <= 1e-12 * np.abs(want).max()
    rows, cols = np.array([5, 0, 36, 5]), np.array([52, 1])
    sub = oracle.gemm_f64(a, w, rows, cols)
    assert (sub == got[np.ix_(rows, cols)]).all()


def test_gemm_integer_special_case(oracle):
    """E6M2 = 1, all micro-exponents clear: values are quarters, the product is exact in int64."""
    rng = np.random.default_rng(23)
    ca = rng.integers(0, 256, (9, 128), dtype=np.uint8)
    cw = rng.integers(0, 256, (11, 128), dtype=np.uint8)
    one = np.full((9, 4), 48 << 2, np.uint32), np.full((11, 4), 48 << 2, np.uint32)
    got = oracle.gemm_f64(oracle.dequantize(ca, one[0]), oracle.dequantize(cw, one[1]))

    def quarters(c):
        n = codes_to_nibbles(c).astype(np.int64)
        return np.where(n & 8, -(n & 7), n & 7)

    want = quarters(ca) @ quarters(cw).T
    assert (got * 16 == want).all()


def test_gemm_weight_only_operand(oracle):
    """A may be plain BF16 (weight-only GEMM): same routine, no decoding of A."""
    rng = np.random.default_rng(24)
    a = synth.bits(synth.to_bf16(rng.standard_normal((4, 128))))
    cw, mw = rand_packed(rng, 6, 128)
    w = oracle.dequantize(cw, mw)
    got = oracle.gemm_f64(a, w)
    want = oracle.bf16_bits_to_f64(a) @ oracle.bf16_bits_to_f64(w).T
    assert np.abs(got - want).max() <= 1e-12 * np.abs(want).max()
