"""Pins of the MXFP4 / NVFP4 comparators (oracle/bfp4_comparators.py) against what the formats fix:
the E2M1 value grid, torch's CPU float8_e4m3fn cast (a library routine), the shared-scale rule of the
Microscaling format, and exact representability of values already on a format's grid."""
import itertools

import numpy as np
import torch

from oracle import bfp4_comparators as cmp

E2M1 = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_round_e2m1_is_nearest_grid_point_with_ties_to_even_mantissa():
    v = np.concatenate([np.linspace(-8, 8, 6401), np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 7.0, 100.0])])
    got = cmp.round_e2m1(v)
    for x, g in zip(v, got):
        a = abs(x)
        d = [abs(a - p) for p in E2M1]
        best = min(d)
        cands = [i for i, di in enumerate(d) if di == best]
        # a tie goes to the grid point with the even mantissa bit: even index in the E2M1 code order
        want = E2M1[[i for i in cands if i % 2 == 0][0]] if len(cands) == 2 else E2M1[cands[0]]
        assert abs(g) == want and (g == 0 or np.sign(g) == np.sign(x)), (x, g, want)


def test_round_e4m3_matches_torch_float8_cast():
    rng = np.random.default_rng(5)
    v = np.concatenate([np.exp(rng.uniform(np.log(2.0 ** -12), np.log(440.0), 20000)),
                        [0.0, 2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -9, 448.0, 447.0, 0.0009765625 * 3]])
    v = v.astype(np.float32).astype(np.float64)   # torch casts from float32
    want = torch.from_numpy(v.astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = cmp.round_e4m3(v)
    assert (got == want).all()
    assert cmp.round_e4m3(np.array([1000.0]))[0] == 448.0   # saturation (the cast above has no such input)


def test_mxfp4_shared_scale_rule_and_grid():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((64, 128)) * np.exp(rng.uniform(-8, 8, (64, 1)))
    y = cmp.mxfp4_fake_quant(x)
    g, q = x.reshape(64, 4, 32), y.reshape(64, 4, 32)
    amax = np.abs(g).max(axis=2)
    scale = 2.0 ** (np.floor(np.log2(amax)) - 2)
    units = q / scale[:, :, None]
    assert np.isin(np.abs(units), E2M1).all()
    # the peak lies in [4, 8) scale units, so it lands on 4 or 6; errors are at most one unit (half of the
    # widest spacing), except above 6 where the value saturates
    assert (np.abs(units).max(axis=2) >= 4.0).all()
    su = np.abs(g / scale[:, :, None])
    assert (np.abs(su - np.abs(units)) <= np.maximum(1.0, su - 6.0) + 1e-12).all()
    # values already on the grid of their group come back unchanged
    assert (cmp.mxfp4_fake_quant(y) == y).all()


def test_nvfp4_group_scale_and_idempotence():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((32, 64)) * np.exp(rng.uniform(-3, 3, (32, 1)))
    y = cmp.nvfp4_fake_quant(x)
    g, q = x.reshape(32, 4, 16), y.reshape(32, 4, 16)
    scale = cmp.round_e4m3(np.abs(g).max(axis=2) / 6.0)
    units = q / scale[:, :, None]
    assert np.isin(np.abs(units), E2M1).all()
    assert (np.abs(units).max(axis=2) >= 4.0).all()      # the peak maps to about 6
    assert (cmp.nvfp4_fake_quant(y) == y).all()
    # per-tensor scaling only changes results when the direct scale would leave E4M3's range
    small = x * 2.0 ** -14
    direct, scaled = cmp.nvfp4_fake_quant(small), cmp.nvfp4_fake_quant(small, pts=True)
    assert np.mean((small - scaled) ** 2) < np.mean((small - direct) ** 2)
