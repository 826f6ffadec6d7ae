"""Pins of the scalar steps of Algorithm 1 (Section II-B) in the oracle: BF16
multiply, BF16_to_E6M2, E6M2_REC_to_BF16, BF16_to_S1P2.  Each is checked against a
library routine (torch's CPU bfloat16) or a brute-force nearest search in exact
rationals, never against its own formula."""
from fractions import Fraction

import numpy as np
import torch


def bf16_fraction(bits):
    """Exact rational value of a finite BF16 pattern, from the IEEE field definition."""
    s, e, m = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
    v = Fraction(m, 128) * Fraction(2) ** -126 if e == 0 else Fraction(128 + m, 128) * Fraction(2) ** (e - 127)
    return -v if s else v


def t_bf16(bits):
    return torch.from_numpy(np.asarray(bits, dtype=np.uint16).view(np.int16)).view(torch.bfloat16)


def t_bits(t):
    return t.view(torch.int16).numpy().view(np.uint16)


def test_bf16_widening_is_the_ieee_field_value(oracle):
    rng = np.random.default_rng(2)
    for b in list(rng.integers(0, 0x7F80, 300)) + [0, 1, 0x7F, 0x80, 0x7F7F, 0x8001, 0xFF7F]:
        assert Fraction(oracle.bf16_to_f64(int(b))) == bf16_fraction(int(b))


def test_bf16_mul_matches_torch_cpu_bfloat16(oracle):
    rng = np.random.default_rng(3)
    a = rng.integers(0, 0x10000, 40000).astype(np.uint16)
    b = rng.integers(0, 0x10000, 40000).astype(np.uint16)
    # plus pairs whose product is tiny (subnormal results) or huge (overflow)
    a[:4000] = rng.integers(0x0001, 0x2000, 4000)
    b[:4000] = rng.integers(0x2000, 0x4000, 4000)
    fin = ((a & 0x7FFF) < 0x7F80) & ((b & 0x7FFF) < 0x7F80)
    a, b = a[fin], b[fin]
    want = t_bits(t_bf16(a) * t_bf16(b))
    got = np.array([oracle.bf16_mul(int(x), int(y)) for x, y in zip(a, b)], dtype=np.uint16)
    assert (got == want).all()


def test_bf16_rounding_ties(oracle):
    # 1 + 2^-8 is half-way between 1 and 1 + 2^-7: even keeps 1.0, away goes up
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8, oracle.ROUND_RNE) == 0x3F80
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8, oracle.ROUND_RHA) == 0x3F81
    assert oracle.f64_to_bf16(1.0 + 3 * 2.0 ** -8, oracle.ROUND_RNE) == 0x3F82
    assert oracle.f64_to_bf16(-(1.0 + 2.0 ** -8), oracle.ROUND_RHA) == 0xBF81
    # random fp32 values against torch's conversion (round to nearest even)
    rng = np.random.default_rng(4)
    f = (rng.standard_normal(5000) * np.exp(rng.uniform(-80, 80, 5000))).astype(np.float32)
    want = t_bits(torch.from_numpy(f).to(torch.bfloat16))
    got = np.array([oracle.f64_to_bf16(float(v)) for v in f], dtype=np.uint16)
    assert (got == want).all()


def test_one_seventh_constant_is_nearest_bf16():
    target = Fraction(1, 7)
    best = min(range(0x3D80, 0x3F00), key=lambda b: abs(bf16_fraction(b) - target))
    assert best == 0x3E12 and bf16_fraction(best) == Fraction(73, 512)
    others = sorted(abs(bf16_fraction(b) - target) for b in (0x3E11, 0x3E12, 0x3E13))
    assert others[0] < others[1], "not a tie: both rounding modes agree"


def e6m2_fraction(byte):
    return Fraction(4 + (byte & 3), 4) * Fraction(2) ** ((byte >> 2) - 48)


def test_bf16_to_e6m2_round_trip_and_saturation(oracle):
    for mode in (oracle.ROUND_RNE, oracle.ROUND_RHA):
        for byte in range(255):
            bits = oracle.f64_to_bf16(float(e6m2_fraction(byte)))
            assert oracle.bf16_to_e6m2(bits, mode) == byte
        assert oracle.bf16_to_e6m2(0x0000, mode) == 0x00          # zero -> least code
        assert oracle.bf16_to_e6m2(0x0001, mode) == 0x00          # subnormal
        assert oracle.bf16_to_e6m2(oracle.f64_to_bf16(2.0 ** -60), mode) == 0x00
        assert oracle.bf16_to_e6m2(oracle.f64_to_bf16(2.0 ** 15 * 1.75), mode) == 0xFE  # would be the NaN code
        assert oracle.bf16_to_e6m2(oracle.f64_to_bf16(2.0 ** 20), mode) == 0xFE
        assert oracle.bf16_to_e6m2(0x7F7F, mode) == 0xFE
    # ties: 1.125 is half-way between 1.0 (M=0, even) and 1.25 (M=1)
    assert oracle.bf16_to_e6m2(oracle.f64_to_bf16(1.125), oracle.ROUND_RNE) == (48 << 2) | 0
    assert oracle.bf16_to_e6m2(oracle.f64_to_bf16(1.125), oracle.ROUND_RHA) == (48 << 2) | 1
    assert oracle.bf16_to_e6m2(oracle.f64_to_bf16(1.375), oracle.ROUND_RNE) == (48 << 2) | 2
    # 1.875 is half-way between 1.75 (odd) and 2.0 (next binade, even)
    assert oracle.bf16_to_e6m2(oracle.f64_to_bf16(1.875), oracle.ROUND_RNE) == (49 << 2) | 0


def test_bf16_to_e6m2_is_nearest_by_brute_force(oracle):
    """For every positive finite BF16 inside the E6M2 range the chosen code is a nearest one."""
    table = [e6m2_fraction(b) for b in range(255)]
    lo, hi = table[0], table[254]
    prev = 0
    for bits in range(0x0001, 0x7F80, 7):
        v = bf16_fraction(bits)
        got = oracle.bf16_to_e6m2(bits)
        assert got >= prev, "monotone"
        prev = got
        if v <= lo:
            assert got == 0
        elif v >= hi:
            assert got == 254
        else:
            d = abs(table[got] - v)
            assert all(d <= abs(t - v) for t in table[max(0, got - 2):got + 3])


def test_reciprocal_table_is_nearest_bf16(oracle):
    for byte in range(255):
        want = 1 / e6m2_fraction(byte)
        got = oracle.e6m2_rec_to_bf16(byte)
        d = abs(bf16_fraction(got) - want)
        assert d < abs(bf16_fraction(got - 1) - want) and d < abs(bf16_fraction(got + 1) - want)
    # the four mantissa entries, as listed in the oracle header
    assert [oracle.e6m2_rec_to_bf16((48 << 2) | m) for m in range(4)] == [0x3F80, 0x3F4D, 0x3F2B, 0x3F12]


def test_s1p2_rounding_brute_force(oracle):
    grid = [Fraction(m, 4) for m in range(8)]
    rng = np.random.default_rng(5)
    vals = [Fraction(int(n), 64) for n in rng.integers(0, 200, 400)] + [Fraction(k, 8) for k in range(20)]
    for v in vals:
        for neg in (0, 1):
            for mode in (oracle.ROUND_RNE, oracle.ROUND_RHA):
                c = oracle.to_s1p2(float(v), neg, mode)
                assert (c >> 3) == neg
                m = c & 7
                d = abs(grid[m] - v)
                assert all(d <= abs(g - v) for g in grid), "nearest representable magnitude (clamped at 1.75)"
                ties = [k for k, g in enumerate(grid) if abs(g - v) == d]
                if len(ties) == 2:
                    assert m == ([k for k in ties if k % 2 == 0][0] if mode == oracle.ROUND_RNE else max(ties))
    assert oracle.to_s1p2(1e30, 1) == 0xF and oracle.to_s1p2(1.875, 0) == 7


def nearest_bf16_by_search(v, mode):
    """Positive rational -> nearest finite positive BF16 pattern by search over all of them; an exact tie
    goes to the even pattern (mode 0) or to the larger one (mode 1)."""
    lo, hi = 0, 0x7F7F
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if bf16_fraction(mid) <= v:
            lo = mid
        else:
            hi = mid
    dl, dh = v - bf16_fraction(lo), bf16_fraction(hi) - v
    if dl != dh:
        return lo if dl < dh else hi
    return hi if mode == 1 else (lo if lo % 2 == 0 else hi)


def test_bf16_mul_half_away_on_exact_ties(oracle):
    """Products that are exact BF16 ties (found by search, not by formula): half-away takes the larger
    magnitude, half-to-even the even pattern; checked against the search above, signs included."""
    rng = np.random.default_rng(6)
    ties = 0
    pairs = [(0x4120, 0x3E12), (0x3FA0, 0x3F12), (0x40A0, 0x3F92), (0x40E0, 0x3E12)]  # 10/7, 1.25*146/256, 5*146/128, 7/7
    pairs += [(int(a), int(b)) for a, b in zip(rng.integers(0x3000, 0x5000, 3000), rng.integers(0x3000, 0x5000, 3000))]
    for a, b in pairs:
        exact = bf16_fraction(a) * bf16_fraction(b)
        for mode in (oracle.ROUND_RNE, oracle.ROUND_RHA):
            want = nearest_bf16_by_search(exact, mode)
            assert oracle.bf16_mul(a, b, mode) == want
            assert oracle.bf16_mul(a | 0x8000, b, mode) == want | 0x8000
        ties += nearest_bf16_by_search(exact, 0) != nearest_bf16_by_search(exact, 1)
    assert ties >= 3, "the list holds products on which the two roundings differ"


def test_bf16_to_e6m2_half_away_on_every_tie(oracle):
    """Every BF16 whose significand lies half-way between two E6M2 significands, at several exponents:
    1.125 and 1.625 part the two roundings, 1.375 and 1.875 do not (their even neighbour is the upper one)."""
    for e in (-40, -1, 0, 7, 14):
        for sig, rne_q, rha_q in ((1.125, 4, 5), (1.375, 6, 6), (1.625, 6, 7), (1.875, 8, 8)):
            bits = oracle.f64_to_bf16(sig * 2.0 ** e)
            for mode, q in ((oracle.ROUND_RNE, rne_q), (oracle.ROUND_RHA, rha_q)):
                ee, qq = (e + 1, 4) if q == 8 else (e, q)
                assert oracle.bf16_to_e6m2(bits, mode) == ((ee + 48) << 2) | (qq - 4)
