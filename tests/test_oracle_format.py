"""Pins of the oracle's decode side against what the paper prints (Section II-A,
Tables 1 and 2) and against Eq. 2 evaluated in exact rational arithmetic."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from layout import nibbles_to_codes

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def paper_values():
    out = {}
    for line in open(os.path.join(GOLD, "paper_code_points.txt")):
        line = line.split("#")[0].split()
        if len(line) >= 2:
            out[line[0]] = line[1]
    return out


P = paper_values()


def unit(codes_nibbles, e6m2, e8=0, e16=0):
    """Build (codes[32], meta) from 64 nibbles using the documented layout."""
    n = np.asarray(codes_nibbles, dtype=np.uint8)
    codes = nibbles_to_codes(n)
    return codes, (e16 << 16) | (e8 << 8) | e6m2


def test_e6m2_code_points(oracle):
    assert oracle.e6m2_to_f64(int(P["e6m2_max_byte"], 16)) == float(P["e6m2_max_value"]) == 2.0 ** 15 * 1.5
    assert oracle.e6m2_to_f64(int(P["e6m2_min_byte"], 16)) == 2.0 ** int(P["e6m2_min_value_log2"])
    assert math.isnan(oracle.e6m2_to_f64(int(P["e6m2_nan_byte"], 16)))
    # bias 48: exponent field 48, mantissa 0 is exactly 1
    assert oracle.e6m2_to_f64(int(P["e6m2_bias"]) << 2) == 1.0
    vals = [oracle.e6m2_to_f64(b) for b in range(255)]
    assert all(b > a for a, b in zip(vals, vals[1:])), "255 finite codes, strictly increasing"
    assert min(vals) > 0 and not any(math.isinf(v) for v in vals), "no zero, no infinity"
    exps = {math.floor(math.log2(v)) for v in vals}
    assert min(exps) == int(P["e6m2_exp_min"]) and max(exps) == int(P["e6m2_exp_max"])
    # hidden bit 1, two mantissa bits: significands are 1, 1.25, 1.5, 1.75
    assert [oracle.e6m2_to_f64((48 << 2) | m) for m in range(4)] == [1.0, 1.25, 1.5, 1.75]


def test_s1p2_code_points(oracle):
    nib = list(range(16)) + [0] * 48
    codes, meta = unit(nib, 48 << 2)
    v = [oracle.decode_elem_f64(codes, meta, i) for i in range(16)]
    assert v[0b0111] == float(P["s1p2_max"]) and v[0b1111] == -float(P["s1p2_max"])
    assert v[0b0001] == float(P["s1p2_min"]) and v[0b1001] == -float(P["s1p2_min"])
    assert v[0] == 0.0 and not math.copysign(1, v[0]) < 0
    assert v[8] == 0.0 and math.copysign(1, v[8]) < 0, "minus zero exists"
    assert v[:8] == [0.25 * m for m in range(8)], "sign-magnitude, binary point after one integer bit"


def test_intra_group_and_global_extremes(oracle):
    codes, _ = unit([7] + [1] * 63, 0)
    one = 48 << 2
    hi = oracle.decode_elem_f64(codes, (0xFFFF << 16) | (0xFF << 8) | one, 0)
    lo = oracle.decode_elem_f64(codes, one, 1)
    assert hi == float(P["intra_group_max"]) and lo == float(P["intra_group_min"])
    assert round(math.log2(hi / lo), 2) == float(P["local_range_binades"])
    gmax = oracle.decode_elem_f64(codes, (0xFFFF << 16) | (0xFF << 8) | 0xFE, 0)
    gmin = oracle.decode_elem_f64(codes, 0x00, 1)
    assert gmax == float(P["global_max"]) == 2.0 ** 18 * 1.3125
    assert gmin == 2.0 ** int(P["global_min_log2"])
    assert math.floor(math.log2(gmax)) - math.floor(math.log2(gmin)) + 1 == int(P["global_range_binades"])


def test_storage_is_4p5_bits(oracle):
    x = np.zeros((3, 128), np.uint16)
    codes, meta = oracle.quantize(x)
    assert codes.nbytes * 8 + meta.nbytes * 8 == float(P["bits_per_value"]) * x.size
    assert x.shape[1] // meta.shape[1] == int(P["group_size"])


def test_nan_unit(oracle):
    codes, meta = unit([5] * 64, 0xFF, 0x12, 0x3456)
    y = oracle.decode_unit(codes, meta)
    f = oracle.bf16_bits_to_f64(y)
    assert np.isnan(f).all()


def eq2_fraction(byte, e8bit, e16bit, nib):
    E, M = (byte >> 2) - 48, byte & 3
    scale = Fraction(4 + M, 4) * (Fraction(2) ** E)
    s1p2 = Fraction(nib & 7, 4) * (-1 if nib & 8 else 1)
    return scale * (2 ** (e8bit + e16bit)) * s1p2


def test_exhaustive_decode_all_combinations(oracle):
    """All 255 x 2 x 2 x 16 (E6M2, E1_8, E1_16, nibble) combinations, exact rationals."""
    for byte in range(255):
        for e8 in (0, 1):
            for e16 in (0, 1):
                codes, meta = unit(list(range(16)) + [0] * 48, byte, 0xFF * e8, 0xFFFF * e16)
                y = oracle.decode_unit(codes, meta)  # raises if any value were inexact in BF16
                f = oracle.bf16_bits_to_f64(y)
                for nib in range(16):
                    want = eq2_fraction(byte, e8, e16, nib)
                    assert Fraction(float(f[nib])) == want
                    assert (y[nib] >> 15) == (nib >> 3), "sign bit is the nibble's top bit, also for zero"


def test_position_mapping_of_micro_exponents(oracle):
    """Bit j of E1_8 doubles elements 8j..8j+7 only; bit k of E1_16 doubles 4k..4k+3 only."""
    base_codes, _ = unit([4] * 64, 48 << 2)
    for j in range(8):
        f = oracle.bf16_bits_to_f64(oracle.decode_unit(base_codes, ((1 << j) << 8) | (48 << 2)))
        want = np.ones(64)
        want[8 * j:8 * j + 8] = 2.0
        assert (f == want).all()
    for k in range(16):
        f = oracle.bf16_bits_to_f64(oracle.decode_unit(base_codes, ((1 << k) << 16) | (48 << 2)))
        want = np.ones(64)
        want[4 * k:4 * k + 4] = 2.0
        assert (f == want).all()
    # nibble order: byte 4j+t = element 8j+t (low nibble) and element 8j+4+t (high nibble)
    codes = np.zeros(32, np.uint8)
    codes[5] = 0x73
    f = oracle.bf16_bits_to_f64(oracle.decode_unit(codes, 48 << 2))
    assert f[8 + 1] == 0.75 and f[8 + 4 + 1] == 1.75 and f.sum() == 2.5


def test_bulk_decode_matches_elementwise(oracle):
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 256, size=(7, 96), dtype=np.uint8)
    meta = rng.integers(0, 2 ** 32, size=(7, 3), dtype=np.uint64).astype(np.uint32)
    meta[meta & 0xFF == 0xFF] ^= 1  # keep them finite here
    y = oracle.bf16_bits_to_f64(oracle.dequantize(codes, meta))
    for r in range(7):
        for u in range(3):
            for i in range(64):
                assert y[r, 64 * u + i] == oracle.decode_elem_f64(codes[r, 32 * u:32 * u + 32], int(meta[r, u]), i)
