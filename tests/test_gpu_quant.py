"""GPU parity of hif4_quantize / hif4_dequantize (through the C ABI) against the CPU
oracle: bit-exact codes, metadata and BF16 patterns on the same seeded inputs."""
import numpy as np
import pytest
import torch

from layout import nibbles_to_codes
from paper_2602_11287_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    from paper_2602_11287_amd import hif4
    hif4.load()
    assert torch.cuda.is_available()
    return hif4


def mixed_matrix(rows, K, seed):
    """Rows cycling through value distributions, a few special values sprinkled in."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, K))
    for r in range(rows):
        k = r % 6
        if k == 1:
            x[r, rng.random(K) < 0.02] *= 64
        elif k == 2:
            x[r] *= np.exp(rng.uniform(-3, 3, K))
        elif k == 3:
            x[r] *= 2.0 ** rng.integers(-60, 24, (K // 64, 1)).repeat(64, 0).reshape(-1)[:K]
        elif k == 4:
            x[r] = rng.integers(-64, 65, K) / 8.0
        elif k == 5:
            x[r] *= rng.random(K) < 0.1
    b = synth.bits(torch.from_numpy(x).to(torch.bfloat16)).copy()
    flat = b.reshape(-1)
    n = flat.size
    for pat in (0x7FC0, 0xFF80, 0x7F80, 0x8000, 0x0001, 0x807F, 0x7F7F, 0xFF7F, 0x0080):
        flat[rng.integers(0, n, max(1, n // 3000))] = pat
    return b


def to_dev(bits):
    return synth.from_bits(bits).cuda()


def check_encode(h, oracle, xb, mode=0, ld=None):
    rows, K = xb.shape
    if ld is None:
        xd = to_dev(xb)
    else:
        buf = torch.zeros((rows, ld), dtype=torch.bfloat16, device="cuda")
        buf[:, :K] = to_dev(xb)
        xd = buf[:, :K]
    codes, meta = h.hif4_quantize(xd, round_mode=mode)
    torch.cuda.synchronize()
    wc, wm = oracle.quantize(xb, mode)
    gm = meta.cpu().numpy().view(np.uint32)
    gc = codes.cpu().numpy()
    bad_m = np.argwhere(gm != wm)
    assert bad_m.size == 0, f"meta differs at {bad_m[:5]}: got {gm[tuple(bad_m[0])]:#x} want {wm[tuple(bad_m[0])]:#x}"
    bad_c = np.argwhere(gc != wc)
    assert bad_c.size == 0, f"codes differ at {bad_c[:5]}"
    return codes, meta


@pytest.mark.parametrize("rows,K", [(1, 64), (3, 128), (37, 192), (5, 4096), (259, 320), (64, 1024)])
@pytest.mark.parametrize("mode", [0, 1])
def test_encode_matches_oracle(h, oracle, rows, K, mode):
    print(f"encode parity rows={rows} K={K} mode={mode}", flush=True)
    check_encode(h, oracle, mixed_matrix(rows, K, 1000 + rows + K), mode)


def test_encode_strided_rows(h, oracle):
    check_encode(h, oracle, mixed_matrix(19, 256, 7), 0, ld=256 + 64)
    check_encode(h, oracle, mixed_matrix(19, 256, 8), 1, ld=256 + 8)


def test_encode_config1_full(h, oracle):
    """1024 x 4096 activations, N(0,1) with 0.1 % of entries times 64: every unit compared."""
    x = synth.activation_with_outliers()
    codes, meta = check_encode(h, oracle, synth.bits(x))
    y = h.hif4_dequantize(codes, meta)
    torch.cuda.synchronize()
    want = oracle.dequantize(codes.cpu().numpy(), meta.cpu().numpy().view(np.uint32))
    assert (synth.bits(y.cpu()) == want).all()


def test_encode_all_bf16_patterns(h, oracle):
    """Every BF16 pattern appears as the peak of some unit and as a small element of another."""
    pats = np.arange(0x10000, dtype=np.uint16)
    rng = np.random.default_rng(5)
    x = np.zeros((1024, 64 * 64), np.uint16).reshape(-1, 64)
    x[:, :] = rng.integers(0x3000, 0x3F00, x.shape).astype(np.uint16)
    x[np.arange(0x10000), rng.integers(0, 64, 0x10000)] = pats
    check_encode(h, oracle, x.reshape(1024, 4096))
    check_encode(h, oracle, x.reshape(1024, 4096), 1)


def test_decode_exhaustive(h, oracle):
    """All 256 E6M2 bytes x micro-exponent settings x 16 nibbles, at every position of the unit."""
    units = []
    for byte in range(256):
        for e8, e16 in ((0, 0), (0xFF, 0), (0, 0xFFFF), (0xFF, 0xFFFF), (0xA5, 0x3C5A)):
            units.append((e16 << 16) | (e8 << 8) | byte)
    meta = np.array(units, np.uint32).reshape(-1, 1).repeat(16, 1)         # 16 units per row
    rows = meta.shape[0]
    codes = np.zeros((rows, 16 * 32), np.uint8)
    for s in range(16):                                                       # rotate nibbles through positions
        nib = (np.arange(64) + s) % 16
        codes[:, 32 * s:32 * s + 32] = nibbles_to_codes(nib)
    y = h.hif4_dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(meta.view(np.int32)).cuda())
    torch.cuda.synchronize()
    got = synth.bits(y.cpu())
    want = oracle.dequantize(codes, meta)
    nan_rows = (meta[:, 0] & 0xFF) == 0xFF
    assert (got[nan_rows] == 0x7FC0).all() and (want[nan_rows] == 0x7FC0).all()
    assert (got == want).all()


@pytest.mark.parametrize("rows,K", [(1, 64), (7, 192), (130, 1088)])
def test_decode_random_packed(h, oracle, rows, K):
    rng = np.random.default_rng(rows)
    codes = rng.integers(0, 256, (rows, K // 2), dtype=np.uint8)
    meta = rng.integers(0, 2 ** 32, (rows, K // 64), dtype=np.uint64).astype(np.uint32)
    cd, md = torch.from_numpy(codes).cuda(), torch.from_numpy(meta.view(np.int32)).cuda()
    y = h.hif4_dequantize(cd, md)
    # strided output
    buf = torch.full((rows, K + 24), 7.0, dtype=torch.bfloat16, device="cuda")
    h.hif4_dequantize(cd, md, y=buf[:, :K])
    torch.cuda.synchronize()
    want = oracle.dequantize(codes, meta)
    assert (synth.bits(y.cpu()) == want).all()
    assert (synth.bits(buf[:, :K].cpu().contiguous()) == want).all()
    assert (buf[:, K:] == 7.0).all(), "bytes past K untouched"


def test_empty_and_errors(h):
    x = torch.zeros((0, 128), dtype=torch.bfloat16, device="cuda")
    codes, meta = h.hif4_quantize(x)
    assert codes.shape == (0, 64) and meta.shape == (0, 2)
    y = h.hif4_dequantize(codes, meta)
    assert y.shape == (0, 128)
    with pytest.raises(h.Hif4Error):
        h.hif4_quantize(torch.zeros((2, 100), dtype=torch.bfloat16, device="cuda"))


def test_encode_large_sampled_rows(h, oracle):
    """The benchmark's HBM-sized matrix (16384 x 8192): sampled rows against the oracle."""
    g = torch.Generator(device="cuda").manual_seed(3)
    x = torch.randn((16384, 8192), generator=g, device="cuda", dtype=torch.float32)
    x[torch.rand(x.shape, generator=g, device="cuda") < 0.001] *= 64
    x = x.to(torch.bfloat16)
    codes, meta = h.hif4_quantize(x)
    y = h.hif4_dequantize(codes, meta)
    torch.cuda.synchronize()
    rows = np.random.default_rng(9).choice(16384, 256, replace=False)
    rows = np.concatenate([rows, [0, 16383]])
    xs = synth.bits(x[rows].cpu())
    wc, wm = oracle.quantize(xs)
    assert (codes[rows].cpu().numpy() == wc).all()
    assert (meta[rows].cpu().numpy().view(np.uint32) == wm).all()
    assert (synth.bits(y[rows].cpu()) == oracle.dequantize(wc, wm)).all()


def wide_matrix(rows, K, seed, dtype):
    """fp32 / fp16 inputs whose low mantissa bits matter: Gaussian bulk with spread scales, exact ties of
    the BF16 rounding (odd and even neighbours), values at and beyond the edge of the BF16 range, subnormals,
    zeros of both signs, NaN and infinities."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, K)) * np.exp(rng.uniform(-4, 4, (rows, 1)))
    x = x.astype(dtype)
    flat = x.reshape(-1)
    n = flat.size
    # BF16 ties: 8 leading significand bits, then exactly one half unit in the last place
    base = (1.0 + rng.integers(0, 128, n // 50) / 128.0 + 1.0 / 256.0) * 2.0 ** rng.integers(-6, 6, n // 50)
    flat[rng.integers(0, n, n // 50)] = (base * rng.choice([-1.0, 1.0], n // 50)).astype(dtype)
    specials = [0.0, -0.0, np.inf, -np.inf, np.nan, 6.0e-8, -6.0e-8, 65504.0, -65504.0, 1.0009765625]
    if dtype == np.float32:
        specials += [3.4e38, -3.4e38, 3.3895e38, 1e-40, -1e-45, 1.17549435e-38, 2.0 ** -127 * 1.00390625]
    for v in specials:
        flat[rng.integers(0, n, max(1, n // 4000))] = dtype(v)
    return x


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("rows,K", [(1, 64), (37, 192), (259, 320), (64, 4096)])
def test_encode_from_fp32_fp16_matches_oracle(h, oracle, rows, K, mode, dtype):
    print(f"encode from {dtype.__name__} rows={rows} K={K} mode={mode}", flush=True)
    x = wide_matrix(rows, K, 500 + rows + K, dtype)
    want_c, want_m = oracle.quantize_from(x, mode)
    codes, meta = h.hif4_quantize_from(torch.from_numpy(x).cuda(), round_mode=mode)
    torch.cuda.synchronize()
    assert (meta.cpu().numpy().view(np.uint32) == want_m).all()
    assert (codes.cpu().numpy() == want_c).all()


def test_encode_from_strided_and_bf16(h, oracle):
    x = wide_matrix(33, 256, 77, np.float32)
    big = torch.zeros((33, 256 + 64), dtype=torch.float32, device="cuda")
    big[:, :256] = torch.from_numpy(x).cuda()
    codes, meta = h.hif4_quantize_from(big[:, :256])
    want_c, want_m = oracle.quantize_from(x)
    assert (codes.cpu().numpy() == want_c).all() and (meta.cpu().numpy().view(np.uint32) == want_m).all()
    # in_dtype BF16 is hif4_quantize
    xb = torch.from_numpy(x).to(torch.bfloat16).cuda()
    c1, m1 = h.hif4_quantize_from(xb)
    c2, m2 = h.hif4_quantize(xb)
    assert torch.equal(c1, c2) and torch.equal(m1, m2)


def test_encode_decode_beyond_2_to_32_elements(h, oracle):
    """A matrix of more than 2^32 elements (8.6 GB of BF16): element and byte offsets need 64 bits.
    Rows from the start, the middle and the very end against the oracle."""
    rows, K = (1 << 20) + 4096 + 3, 4096
    print(f"encode/decode rows={rows} K={K}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(77)
    x = torch.empty((rows, K), dtype=torch.bfloat16, device="cuda")
    step = 1 << 16
    for r in range(0, rows, step):
        n = min(step, rows - r)
        x[r:r + n] = (torch.randn((n, K), generator=g, device="cuda") * (1.0 + (r >> 16) % 7)).to(torch.bfloat16)
    codes, meta = h.hif4_quantize(x)
    y = h.hif4_dequantize(codes, meta)
    torch.cuda.synchronize()
    pick = np.array([0, 1, 524287, 524288, (1 << 20) - 1, 1 << 20, rows - 2, rows - 1])
    pi = torch.from_numpy(pick).cuda()
    wc, wm = oracle.quantize(synth.bits(x[pi].cpu()))
    assert (codes[pi].cpu().numpy() == wc).all()
    assert (meta[pi].cpu().numpy().view(np.uint32) == wm).all()
    assert (synth.bits(y[pi].cpu()) == oracle.dequantize(wc, wm)).all()
