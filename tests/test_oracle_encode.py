"""Pins of the oracle's encoder (Algorithm 1, Section II-B): units worked by hand,
a re-derivation from torch's CPU bfloat16 arithmetic plus brute-force nearest
searches, the invariants the algorithm implies, canonical round trips, special
inputs, and the MSE ratios printed in Section III-A."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from layout import codes_to_nibbles, nibbles_to_codes
from paper_2602_11287_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers

def nibbles(codes):
    return codes_to_nibbles(codes)


def bf(values):
    """float list -> BF16 patterns via torch (exact for the short values used here)."""
    return synth.bits(torch.tensor(np.asarray(values, dtype=np.float64)).to(torch.bfloat16))


def random_units(rng, n, kind):
    if kind == "gauss":
        x = rng.standard_normal((n, 64))
    elif kind == "outlier":
        x = rng.standard_normal((n, 64))
        x[rng.random((n, 64)) < 0.02] *= 64
    elif kind == "wide":
        x = rng.standard_normal((n, 64)) * np.exp(rng.uniform(-3, 3, (n, 64)))
    elif kind == "scales":
        x = rng.standard_normal((n, 64)) * 2.0 ** rng.integers(-60, 24, (n, 1))
    elif kind == "short":  # few significant bits: ties everywhere
        x = rng.integers(-64, 65, (n, 64)) / 8.0
    elif kind == "sparse":
        x = rng.standard_normal((n, 64)) * (rng.random((n, 64)) < 0.1)
    else:
        raise ValueError(kind)
    return synth.bits(torch.from_numpy(x).to(torch.bfloat16))


KINDS = ["gauss", "outlier", "wide", "scales", "short", "sparse"]


# ------------------------------------------------------------------ hand-worked units

def load_units():
    units, cur = {}, None
    for raw in open(os.path.join(GOLD, "handworked_units.txt")):
        t = raw.split("#")[0].split()
        if not t:
            continue
        if t[0] == "unit":
            cur = units.setdefault(t[1], {"x": {}, "meta": {}, "code": {"rne": {}, "rha": {}}, "dec": {"rne": {}},
                                          "step": {"rne": [], "rha": []}})
        elif t[0] == "x":
            cur["x"][int(t[1])] = float(t[2])
        elif t[0] == "meta":
            cur["meta"][t[1]] = int(t[2], 16)
        elif t[0] == "code":
            cur["code"][t[1]][int(t[2])] = int(t[3], 16)
        elif t[0] == "dec":
            cur["dec"][t[1]][int(t[2])] = float(t[3])
        elif t[0] == "step":
            cur["step"][t[1]].append((t[2], int(t[3]), int(t[4], 16)))
    return units


@pytest.mark.parametrize("name", ["seven", "ten", "e6tie", "sf208"])
def test_handworked_units(oracle, name):
    u = load_units()[name]
    x = np.zeros(64)
    for i, v in u["x"].items():
        x[i] = v
    xb = bf(x)
    assert (synth.from_bits(xb).double().numpy() == x).all(), "inputs are exact in BF16"
    for mode_name, mode in (("rne", oracle.ROUND_RNE), ("rha", oracle.ROUND_RHA)):
        codes, meta = oracle.encode_unit(xb, mode)
        assert meta == u["meta"][mode_name], hex(meta)
        want = np.zeros(64, np.uint8)
        for i, c in u["code"][mode_name].items():
            want[i] = c
        assert (nibbles(codes) == want).all()
        # intermediates of the conversion (BF16 patterns of SF, the reciprocal, scaled values), where listed
        steps = oracle.encode_unit_steps(xb, mode)
        for field, index, value in u["step"][mode_name]:
            got = steps[field] if np.isscalar(steps[field]) else steps[field][index]
            assert int(got) == value, (mode_name, field, index, hex(int(got)), hex(value))
        assert (steps["S1P2"] == want).all() and steps["E6M2"] == (meta & 0xFF)
    codes, meta = oracle.encode_unit(xb)
    y = oracle.decode_unit(codes, meta)
    f = oracle.bf16_bits_to_f64(y)
    for i, v in u["dec"]["rne"].items():
        assert f[i] == v and np.signbit(f[i]) == np.signbit(v)


# ------------------------------------------------------------------ re-derivation

E6M2_TABLE = [Fraction(4 + (b & 3), 4) * Fraction(2) ** ((b >> 2) - 48) for b in range(255)]
S1P2_GRID = np.arange(8) / 4.0


def rederive_unit(xb):
    """Algorithm 1 again, from torch bfloat16 products and nearest searches."""
    x = synth.from_bits(xb)
    a = x.abs()
    vmax = a.max()
    inv7 = torch.tensor(1.0 / 7.0, dtype=torch.float64).to(torch.bfloat16)
    sf = Fraction(float(vmax * inv7))                      # product rounded to BF16 by torch
    if sf <= E6M2_TABLE[0]:
        byte = 0
    elif sf >= Fraction(7, 4) * 2 ** 15:
        byte = 254
    else:
        d = [abs(t - sf) for t in E6M2_TABLE]
        best = min(d)
        cands = [b for b in range(255) if d[b] == best]
        byte = cands[0] if len(cands) == 1 else [b for b in cands if b % 2 == 0][0]
    rec = torch.tensor(float(1 / E6M2_TABLE[byte]), dtype=torch.float64).to(torch.bfloat16)
    p = (a * rec).double().numpy()                         # 64 products rounded to BF16 by torch
    e8 = [int(p[8 * j:8 * j + 8].max() >= 4.0) for j in range(8)]
    e16 = [int(p[4 * k:4 * k + 4].max() * 2.0 ** -e8[k // 2] >= 2.0) for k in range(16)]
    codes = np.zeros(64, np.uint8)
    for i in range(64):
        s = p[i] * 2.0 ** -(e8[i // 8] + e16[i // 4])
        d = np.abs(S1P2_GRID - s)
        cands = np.flatnonzero(d == d.min())
        m = cands[0] if len(cands) == 1 else [c for c in cands if c % 2 == 0][0]
        codes[i] = (8 if (xb[i] >> 15) else 0) | int(m)
    meta = byte | (sum(b << j for j, b in enumerate(e8)) << 8) | (sum(b << k for k, b in enumerate(e16)) << 16)
    return codes, meta


@pytest.mark.parametrize("kind", KINDS)
def test_encoder_matches_rederivation(oracle, kind):
    rng = np.random.default_rng(100 + KINDS.index(kind))
    xs = random_units(rng, 120, kind)
    for xb in xs:
        codes, meta = oracle.encode_unit(xb)
        wc, wm = rederive_unit(xb)
        assert meta == wm, (hex(meta), hex(wm))
        assert (nibbles(codes) == wc).all()


# ---- the same re-derivation in exact rationals, for either rounding (nothing from torch: its
# bfloat16 arithmetic rounds half to even only).  Every rounding is a nearest search over the target
# grid with the tie rule stated once, in nearest().

def nearest(v, grid_floor, step, mode):
    """v >= 0 (Fraction) -> the multiple of `step` nearest to it; ties to the even multiple (mode 0)
    or away from zero (mode 1).  grid_floor is the largest multiple not above v."""
    lo, hi = grid_floor, grid_floor + step
    assert lo <= v < hi
    if v - lo != hi - v:
        return lo if v - lo < hi - v else hi
    if mode == 1:
        return hi
    return lo if (lo / step) % 2 == 0 else hi


def bf16_round_fraction(v, mode):
    """Nearest BF16 (normal range) to the positive rational v, as a Fraction."""
    e = 0
    while Fraction(2) ** (e + 1) <= v:
        e += 1
    while Fraction(2) ** e > v:
        e -= 1
    step = Fraction(2) ** (e - 7)
    return nearest(v, (v // step) * step, step, mode)


def rederive_unit_exact(xb, mode):
    x = [Fraction(float(v)) for v in oracle_widen(xb)]
    a = [abs(v) for v in x]
    vmax = max(a)
    if vmax == 0:
        return np.array([8 if (b >> 15) else 0 for b in xb], np.uint8), 0
    sf = bf16_round_fraction(vmax * Fraction(73, 512), mode)
    # E6M2: nearest value with a 3-bit significand; the range limits are not reached by these inputs
    e = 0
    while Fraction(2) ** (e + 1) <= sf:
        e += 1
    while Fraction(2) ** e > sf:
        e -= 1
    q = Fraction(2) ** (e - 2)
    s6 = nearest(sf, (sf // q) * q, q, mode)
    byte = E6M2_TABLE.index(s6)
    rec = {0: Fraction(1), 1: Fraction(205, 256), 2: Fraction(171, 256), 3: Fraction(146, 256)}[byte & 3] / Fraction(2) ** ((byte >> 2) - 48)
    p = [bf16_round_fraction(v * rec, mode) if v else Fraction(0) for v in a]
    e8 = [int(max(p[8 * j:8 * j + 8]) >= 4) for j in range(8)]
    e16 = [int(max(p[4 * k:4 * k + 4]) / 2 ** e8[k // 2] >= 2) for k in range(16)]
    codes = np.zeros(64, np.uint8)
    quarter = Fraction(1, 4)
    for i in range(64):
        s = p[i] / 2 ** (e8[i // 8] + e16[i // 4])
        m = min(7, int(nearest(s, (s // quarter) * quarter, quarter, mode) / quarter))
        codes[i] = (8 if (xb[i] >> 15) else 0) | m
    meta = byte | (sum(b << j for j, b in enumerate(e8)) << 8) | (sum(b << k for k, b in enumerate(e16)) << 16)
    return codes, meta


def oracle_widen(xb):
    """BF16 patterns -> exact floats, by the IEEE field definition (no oracle code involved)."""
    return (np.asarray(xb, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def e6m2_tie_units(rng, n):
    """Units whose peak makes SF an exact tie of the E6M2 grid (peak significands 182/128, 252/128,
    253/128, found by exhaustive search in test_which_roundings_can_change_a_unit): the one place
    where the two roundings part for good."""
    out = random_units(rng, n, "short")
    for t, row in enumerate(out):
        sig = (182, 252, 253)[t % 3]
        peak = np.uint16(((120 + t % 14) << 7) | (sig - 128))
        row[:] = np.minimum(row & 0x7FFF, peak - 1) | (row & 0x8000)
        row[int(rng.integers(0, 64))] = peak
    return out


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("kind", ["gauss", "short", "scales", "e6tie"])
def test_encoder_matches_exact_rederivation_in_both_roundings(oracle, kind, mode):
    rng = np.random.default_rng(300 + 7 * mode + len(kind))
    xs = e6m2_tie_units(rng, 30) if kind == "e6tie" else random_units(rng, 60 if kind == "scales" else 40, kind)
    if kind == "scales":   # stay inside the range where neither BF16 nor E6M2 saturates
        xs = xs[[(0x2C00 < (r & 0x7FFF).max() < 0x4600) and ((r & 0x7FFF)[(r & 0x7FFF) > 0].min() > 0x1800) for r in xs]]
        assert len(xs) >= 10
    differ = 0
    for xb in xs:
        codes, meta = oracle.encode_unit(xb, mode)
        wc, wm = rederive_unit_exact(xb, mode)
        assert meta == wm, (hex(meta), hex(wm))
        assert (nibbles(codes) == wc).all()
        differ += oracle.encode_unit(xb, 1 - mode)[1] != meta
    if kind == "e6tie":
        assert differ == len(xs), "on these units the two roundings give different E6M2 bytes"


def test_which_roundings_can_change_a_unit():
    """Exhaustive, in exact rationals, no oracle involved: of the rounding steps of Algorithm 1 only the
    rounding to E6M2 and the rounding to S1P2 can tell half-to-even from half-away in the packed unit.
    (i) SF = BF16(Vmax * 73/512): the two roundings differ for one peak significand only (160/128) and
    both results give the same E6M2 under either E6M2 rounding.  (ii) x * REC: an exact BF16 tie with
    different neighbours exists only for the reciprocal 146/256 and x = 1.25 * 2^e, and both neighbours
    compare alike against 4 and 2 and round to the same S1P2 code at every exponent and shift.
    (iii) E6M2 ties are reached from peak significands 182, 252 and 253 (of 128).  The oracle's
    intermediates at (i) and (ii) are pinned through its record of steps in the hand-worked units."""
    def e6m2_of(sf, mode):
        e = 0
        while Fraction(2) ** (e + 1) <= sf:
            e += 1
        while Fraction(2) ** e > sf:
            e -= 1
        q = Fraction(2) ** (e - 2)
        return nearest(sf, (sf // q) * q, q, mode)
    sf_differs, e6_ties = [], []
    for V in range(128, 256):
        exact = Fraction(V, 128) * Fraction(73, 512)
        a, b = bf16_round_fraction(exact, 0), bf16_round_fraction(exact, 1)
        if a != b:
            sf_differs.append(V)
            for m2 in (0, 1):
                assert e6m2_of(a, m2) == e6m2_of(b, m2)
        if e6m2_of(b, 0) != e6m2_of(b, 1):
            e6_ties.append(V)
    assert sf_differs == [160] and e6_ties == [182, 252, 253]
    quarter = Fraction(1, 4)
    product_ties = set()
    for M, rec in enumerate((Fraction(1), Fraction(205, 256), Fraction(171, 256), Fraction(146, 256))):
        for X in range(128, 256):
            for ex in range(-9, 4):
                exact = Fraction(X, 128) * Fraction(2) ** ex * rec
                pa, pb = bf16_round_fraction(exact, 0), bf16_round_fraction(exact, 1)
                if pa == pb:
                    continue
                product_ties.add((M, X))
                for thr in (4, 2):
                    assert (pa >= thr) == (pb >= thr)
                for sh in range(3):
                    for m2 in (0, 1):
                        sa, sb = pa / 2 ** sh, pb / 2 ** sh
                        ca = min(7, int(nearest(sa, (sa // quarter) * quarter, quarter, m2) / quarter))
                        cb = min(7, int(nearest(sb, (sb // quarter) * quarter, quarter, m2) / quarter))
                        assert ca == cb
    assert product_ties == {(3, 160)}


# ------------------------------------------------------------------ invariants

@pytest.mark.parametrize("kind", ["gauss", "outlier", "wide", "short"])
def test_invariants(oracle, kind):
    rng = np.random.default_rng(11)
    xs = random_units(rng, 200, kind)
    for xb in xs:
        codes, meta = oracle.encode_unit(xb)
        nib = nibbles(codes)
        x = oracle.bf16_bits_to_f64(xb)
        if not x.any():
            continue
        e8 = [(meta >> (8 + j)) & 1 for j in range(8)]
        e16 = [(meta >> (16 + k)) & 1 for k in range(16)]
        # the peak element sits at the top of the intra-group range
        i = int(np.abs(x).argmax())
        assert e8[i // 8] == 1 and e16[i // 4] == 1 and (nib[i] & 7) in (6, 7)
        # a set level-2 bit needs a set level-3 bit under it; a set level-3 bit needs an element >= 1
        for j in range(8):
            if e8[j]:
                assert e16[2 * j] or e16[2 * j + 1]
        for k in range(16):
            if e16[k]:
                assert (nib[4 * k:4 * k + 4] & 7).max() >= 4
        # error bound: half a step of the element's own scale (+ one BF16 rounding of the product)
        y = oracle.bf16_bits_to_f64(oracle.decode_unit(codes, meta))
        s = oracle.e6m2_to_f64(meta & 0xFF)
        step = np.array([0.25 * s * 2.0 ** (e8[t // 8] + e16[t // 4]) for t in range(64)])
        unclamped = (nib & 7) < 7
        assert (np.abs(y - x)[unclamped] <= (0.5 * step + np.abs(x) * 2.0 ** -6)[unclamped]).all()
        # negation flips sign bits only
        c2, m2 = oracle.encode_unit(xb ^ 0x8000)
        assert m2 == meta and (nibbles(c2) == (nib ^ 8)).all()
        # a power-of-two rescale moves only the E6M2 exponent
        for n in (-9, 5):
            xs2 = synth.bits(torch.from_numpy(x * 2.0 ** n).to(torch.bfloat16))
            c3, m3 = oracle.encode_unit(xs2)
            assert (nibbles(c3) == nib).all() and m3 == meta + (n << 2)
        # permuting elements inside one group of four permutes its codes only
        k = int(rng.integers(0, 16))
        perm = np.arange(64)
        perm[4 * k:4 * k + 4] = 4 * k + rng.permutation(4)
        c4, m4 = oracle.encode_unit(xb[perm])
        assert m4 == meta and (nibbles(c4) == nib[perm]).all()


def test_monotone_in_one_position(oracle):
    """With the rest of the unit fixed (and the peak elsewhere), a larger input never decodes smaller."""
    rng = np.random.default_rng(12)
    base = rng.standard_normal(64)
    base[0] = 9.0  # fixes the metadata
    vals = np.sort(rng.uniform(-2.5, 2.5, 300))
    prev = -np.inf
    for v in vals:
        x = base.copy()
        x[5] = v
        codes, meta = oracle.encode_unit(bf(x))
        y = oracle.bf16_bits_to_f64(oracle.decode_unit(codes, meta))[5]
        assert y >= prev
        prev = y


# ------------------------------------------------------------------ round trips

def canonical_units(rng, n):
    """Units already on a HiF4 grid in canonical form: the peak element is 7 * scale
    (code 7 under two set micro-exponents), every set level-3 bit has a code >= 4 below
    it, every set level-2 bit has a set level-3 bit below it."""
    out = []
    while len(out) < n:
        nib = rng.integers(0, 16, 64).astype(np.uint8)
        e16 = rng.integers(0, 2, 16)
        e8 = rng.integers(0, 2, 8)
        for k in range(16):
            if e16[k] and (nib[4 * k:4 * k + 4] & 7).max() < 4:
                nib[4 * k + rng.integers(0, 4)] |= 4
        for j in range(8):
            if e8[j] and not (e16[2 * j] or e16[2 * j + 1]):
                e16[2 * j] = 1
                nib[8 * j] |= 4
        j = int(rng.integers(0, 8))
        e8[j] = 1
        e16[2 * j] = 1
        nib[8 * j] |= 7
        byte = int(rng.integers(0, 255))
        meta = byte | (sum(int(b) << t for t, b in enumerate(e8)) << 8) | (sum(int(b) << t for t, b in enumerate(e16)) << 16)
        out.append((nibbles_to_codes(nib), meta))
    return out


def test_round_trip_on_canonical_units(oracle):
    rng = np.random.default_rng(13)
    for codes, meta in canonical_units(rng, 400):
        y = oracle.decode_unit(codes, meta)
        c2, m2 = oracle.encode_unit(y)
        assert m2 == meta and (c2 == codes).all()
        assert (oracle.decode_unit(c2, m2) == y).all()


def test_reencoding_is_not_idempotent_in_general(oracle):
    """A unit whose peak decodes below 7 * scale can move when encoded again (7.9375 -> 7.5 -> 7.0):
    the round trip above is a property of canonical units only."""
    x = np.zeros(64)
    x[0] = 7.9375
    c1, m1 = oracle.encode_unit(bf(x))
    y1 = oracle.decode_unit(c1, m1)
    assert oracle.bf16_bits_to_f64(y1)[0] == 7.5
    c2, m2 = oracle.encode_unit(y1)
    assert oracle.bf16_bits_to_f64(oracle.decode_unit(c2, m2))[0] == 7.0


# ------------------------------------------------------------------ special inputs

def test_special_inputs(oracle):
    z = np.zeros(64, np.uint16)
    codes, meta = oracle.encode_unit(z)
    assert meta == 0 and not codes.any()
    assert not oracle.decode_unit(codes, meta).any()
    # minus zero keeps its sign
    z2 = z.copy()
    z2[3] = 0x8000
    codes, meta = oracle.encode_unit(z2)
    assert nibbles(codes)[3] == 8 and oracle.decode_unit(codes, meta)[3] == 0x8000
    # NaN or Inf anywhere -> the NaN unit
    for special in (0x7FC0, 0xFFC1, 0x7F80, 0xFF80):
        x = bf(np.linspace(-3, 3, 64))
        x[17] = special
        codes, meta = oracle.encode_unit(x)
        assert meta == 0xFF and not codes.any()
        assert np.isnan(oracle.bf16_bits_to_f64(oracle.decode_unit(codes, meta))).all()
    # beyond the format's range: the scale saturates at its largest finite code, elements clamp
    x = np.full(64, 1.0)
    x[0], x[1], x[2] = 3.0e38, -2.0e30, 344064.0
    codes, meta = oracle.encode_unit(bf(x))
    nib = nibbles(codes)
    assert meta & 0xFF == 0xFE and nib[0] == 7 and nib[1] == 0xF and nib[2] == 7
    y = oracle.bf16_bits_to_f64(oracle.decode_unit(codes, meta))
    assert y[0] == 344064.0 and y[1] == -344064.0 and y[2] == 344064.0
    # below the format's range: the scale stops at its least code, small values flush to signed zero
    x = np.full(64, 2.0 ** -60)
    x[0], x[1], x[2] = 2.0 ** -50, -(2.0 ** -52), 2.0 ** -130
    codes, meta = oracle.encode_unit(bf(x))
    nib = nibbles(codes)
    assert meta == 0 and nib[0] == 1 and nib[1] == 8 and nib[2] == 0 and not (nib[3:] & 7).any()


def test_matrix_wrappers_follow_units(oracle):
    rng = np.random.default_rng(14)
    x = random_units(rng, 6, "outlier").reshape(2, 192)
    big = np.zeros((2, 200), np.uint16)
    big[:, :192] = x
    codes, meta = oracle.quantize(big[:, :192])  # strided rows
    for r in range(2):
        for u in range(3):
            c, m = oracle.encode_unit(x[r, 64 * u:64 * u + 64])
            assert m == meta[r, u] and (c == codes[r, 32 * u:32 * u + 32]).all()
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 100), np.uint16))


# ------------------------------------------------------------------ Section III-A

@pytest.mark.parametrize("x", [4, 11])
def test_mse_ratios_of_section_3a(oracle, x):
    """HiF4 : NVFP4 (with per-tensor scaling) : MXFP4 = 1 : 1.32 : 1.89 on Gaussian matrices."""
    from oracle import bfp4_comparators as cmp
    X = synth.gaussian_sweep(x)
    xb = synth.bits(synth.to_bf16(X))
    Xb = oracle.bf16_bits_to_f64(xb)
    codes, meta = oracle.quantize(xb)
    mse_h = np.mean((X - oracle.bf16_bits_to_f64(oracle.dequantize(codes, meta))) ** 2)
    mse_nv = np.mean((X - cmp.nvfp4_fake_quant(Xb, pts=True)) ** 2)
    mse_mx = np.mean((X - cmp.mxfp4_fake_quant(Xb)) ** 2)
    assert abs(mse_nv / mse_h - 1.32) < 0.03, mse_nv / mse_h
    assert abs(mse_mx / mse_h - 1.89) < 0.03, mse_mx / mse_h
    # in range, the direct cast of NVFP4 agrees with the scaled one
    mse_nv_direct = np.mean((X - cmp.nvfp4_fake_quant(Xb)) ** 2)
    assert abs(mse_nv_direct / mse_nv - 1.0) < 0.02


# ---- FP32 / FP16 inputs: the reading is "round to BF16 first, then Algorithm 1" --------------------

def test_quantize_from_equals_library_bf16_conversion_then_algorithm_1(oracle):
    """Under RNE the conversion step is what torch's CPU float32/float16 -> bfloat16 cast does (a library
    routine written by others); the rest is the pinned BF16 encoder."""
    import torch
    from paper_2602_11287_amd import synth
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((16, 512)) * np.exp(rng.uniform(-5, 5, (16, 1)))).astype(np.float32)
    x[0, :8] = [np.inf, -np.inf, np.nan, 3.4e38, -3.4e38, 1e-40, 0.0, -0.0]
    with np.errstate(over="ignore"):
        x16 = x.astype(np.float16)      # the large entries become infinities
    for arr in (x, x16):
        c1, m1 = oracle.quantize_from(arr)
        c2, m2 = oracle.quantize(synth.bits(torch.from_numpy(arr).to(torch.bfloat16)))
        assert (c1 == c2).all() and (m1 == m2).all()


def test_quantize_from_half_away_ties_and_overflow(oracle):
    """A BF16 tie in the input goes to the even neighbour under RNE and away from zero under RHA, and a
    float32 beyond the BF16 range turns its unit into the NaN unit (it rounds to infinity)."""
    x = np.zeros((1, 64), np.float32)
    x[0, 0] = 7.0                       # fixes the unit scale: E6M2 = 1.0, REC = 1.0
    x[0, 8] = 1.0 + 2.0 ** -8 + 0.125   # 1.12890625: BF16 neighbours 1.125 (even) and 1.1328125; own group of 8
    for mode, want_bf16 in ((0, 1.125), (1, 1.1328125)):
        c, m = oracle.quantize_from(x, mode)
        xb = np.zeros((1, 64), np.float32)
        xb[0, 0], xb[0, 8] = 7.0, want_bf16
        c2, m2 = oracle.quantize_from(xb, mode)     # exact in BF16: no conversion rounding
        assert (c == c2).all() and (m == m2).all()
    # the two roundings of that input give different codes for element 8 (low nibble of byte 4, both
    # micro-exponents of its groups clear): 1.125 is a tie of the S1P2 grid and goes to 1.0 (even);
    # 1.1328125 goes to 1.25
    c_rne, _ = oracle.quantize_from(x, 0)
    c_rha, _ = oracle.quantize_from(x, 1)
    assert (c_rne[0, 4] & 0xF) == 4 and (c_rha[0, 4] & 0xF) == 5
    big = np.zeros((1, 64), np.float32)
    big[0, 5] = 3.4e38
    c, m = oracle.quantize_from(big)
    assert m[0, 0] == 0xFF and not c.any()


def test_input_conversion_rounding_is_pinned_on_the_rounded_inputs(oracle):
    """The BF16 patterns that FP32 / FP16 inputs become, read back from the conversion itself: exact
    ties go to the even neighbour under half-to-even and away from zero under half-away; everything
    else goes to the nearer neighbour under both.  (Under half-away the direction of such a tie cannot
    change the packed unit: every decision threshold of Algorithm 1, seen from the input, is a BF16
    with an even significand, and a tie's two neighbours lie on the same side of it.  So the pin is on
    the rounded inputs.)"""
    vals = [1.0 + 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 3 * 2.0 ** -8, -(1.0 + 3 * 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -20,
            1.0 + 2.0 ** -8 - 2.0 ** -20, 6.0 + 2.0 ** -6, 2.0 ** -20 * (1 + 5 * 2.0 ** -8), 255.5, 0.0]
    want = {0: [0x3F80, 0xBF80, 0x3F82, 0xBF82, 0x3F81, 0x3F80, 0x40C0, 0x3580 + 2, 0x4380, 0x0000],
            1: [0x3F81, 0xBF81, 0x3F82, 0xBF82, 0x3F81, 0x3F80, 0x40C1, 0x3580 + 3, 0x4380, 0x0000]}
    x = np.zeros((1, 64), np.float32)
    x[0, :len(vals)] = vals
    assert (x[0, :len(vals)].astype(np.float64) == np.array(vals)).all(), "inputs are exact in FP32"
    for mode in (0, 1):
        _, _, xb = oracle.quantize_from(x, mode, return_bf16=True)
        assert [int(v) for v in xb[0, :len(vals)]] == want[mode], (mode, [hex(int(v)) for v in xb[0, :len(vals)]])
    # FP16: 1 + 2^-8 and 1 + 3 * 2^-8 are exact there (ten mantissa bits)
    h = np.zeros((1, 64), np.float16)
    h[0, :4] = [1.0 + 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -10]
    for mode, w in ((0, [0x3F80, 0xBF80, 0x3F82, 0x3F81]), (1, [0x3F81, 0xBF81, 0x3F82, 0x3F81])):
        _, _, hb = oracle.quantize_from(h, mode, return_bf16=True)
        assert [int(v) for v in hb[0, :4]] == w


def test_f16_widening_matches_numpy(oracle):
    for h in list(range(0, 65536, 7)) + [0x7C00, 0xFC00, 0x0001, 0x8001, 0x03FF, 0x0400, 0x7BFF]:
        want = float(np.uint16(h).view(np.float16))
        got = oracle.f16_to_f64(h)
        assert (np.isnan(want) and np.isnan(got)) or got == want
