"""GPU parity of hif4_gemm / hif4_grouped_gemm (through the C ABI) against the fp64 oracle
on the same decoded operands: relative Frobenius error <= 1e-4 with fp32 output; BF16
output within one BF16 ulp of the rounded oracle value."""
import numpy as np
import pytest
import torch

from paper_2602_11287_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4  # relative Frobenius error against the fp64 oracle, fp32 output


@pytest.fixture(scope="module")
def h():
    from paper_2602_11287_amd import hif4
    hif4.load()
    assert torch.cuda.is_available()
    return hif4


def dev_packed(codes, meta):
    return torch.from_numpy(codes).cuda(), torch.from_numpy(meta.view(np.int32)).cuda()


def rel_fro(got, want):
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def quantized_operands(oracle, M, N, K, seed, a_outliers=True):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((M, K))
    if a_outliers:
        a[rng.random((M, K)) < 0.002] *= 64
    w = rng.standard_normal((N, K)) * 0.02 * np.exp(rng.uniform(np.log(0.5), np.log(2.0), (N, 1)))
    ab = synth.bits(torch.from_numpy(a).to(torch.bfloat16))
    wb = synth.bits(torch.from_numpy(w).to(torch.bfloat16))
    ac, am = oracle.quantize(ab)
    wc, wm = oracle.quantize(wb)
    return ab, (ac, am), (wc, wm)


SHAPES = [(1, 1, 64), (32, 32, 64), (256, 256, 64), (257, 255, 128), (333, 520, 1024), (5, 1000, 192), (600, 70, 320),
          # up to 192 rows: one m-tile of the kernel that expands W into MFMA operands (32-row blocks, 256-column tiles)
          (65, 257, 192), (129, 520, 320), (192, 300, 1088), (160, 33, 64),
          # the same kernel with K split over the waves of a workgroup (K/64 divisible by 2 or 4 and at least 8
          # steps per part): 64-, 128- and 192-row tiles, 4 or 2 parts, 4 waves (narrow N) or 8 (wide N)
          (33, 100, 2048), (40, 100, 1024), (100, 100, 2048), (128, 257, 1024), (150, 96, 1024),
          (20, 8300, 2048), (100, 8300, 2048), (10, 16500, 1024), (70, 16500, 1024), (150, 16500, 1024),
          # up to 64 rows that kernel takes the call only against many weights (more than 24 Mi from 33 rows, 48 Mi
          # from 17); below, HiF4 activations go through the K-split kernel of the weight-only decode shape
          (40, 8300, 4096), (40, 8192, 3584), (40, 13200, 1920), (40, 16500, 1920),
          # a 192-row tile, an odd number of units (no K split) and more than 1024 strips: 8 waves per workgroup
          (150, 33000, 576),
          # 1536 rows and more against a W whose decoded copy fits the memory-side cache, too many strips for the few-row
          # kernel: both operands decoded once (the binding's default workspace has the room)
          (1600, 5100, 256)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_w4a4_prepacked(h, oracle, M, N, K):
    print(f"gemm parity M={M} N={N} K={K}", flush=True)
    _, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 31 + M + N + K)
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
    acd, amd = dev_packed(ac, am)
    wcd, wmd = dev_packed(wc, wm)
    c32 = h.hif4_gemm(h.HIF4_A_HIF4, acd, amd, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    c16 = h.hif4_gemm(h.HIF4_A_HIF4, acd, amd, wcd, wmd, out_dtype=h.HIF4_OUT_BF16)
    c32b = h.hif4_gemm(h.HIF4_A_HIF4, acd, amd, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    got = c32.cpu().numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL, rel_fro(got, want)
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max() + 1e-30
    assert torch.equal(c32, c32b), "same launch twice gives the same bits"
    # BF16 output: within one ulp of the oracle value rounded to BF16
    wb = synth.bits(torch.from_numpy(want).to(torch.bfloat16)).astype(np.int32)
    gb = synth.bits(c16.cpu()).astype(np.int32)
    key = lambda b: np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    assert np.abs(key(gb) - key(wb)).max() <= 1


def test_gemm_quantize_inside_call(h, oracle):
    M, N, K = 300, 200, 512
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 77)
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
    wcd, wmd = dev_packed(wc, wm)
    a = synth.from_bits(ab).cuda()
    c = h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    # strided A and C
    abuf = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    abuf[:, :K] = a
    cbuf = torch.full((M, N + 9), -1.0, dtype=torch.float32, device="cuda")
    h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, abuf[:, :K], None, wcd, wmd, out_dtype=h.HIF4_OUT_F32, c=cbuf[:, :N])
    torch.cuda.synchronize()
    assert rel_fro(c.cpu().numpy().astype(np.float64), want) <= TOL
    assert torch.equal(cbuf[:, :N], c) and (cbuf[:, N:] == -1.0).all()


def test_gemm_random_packed_wide_range_and_nan(h, oracle):
    """Packed planes drawn directly: every metadata pattern, scales far apart, one NaN unit each side."""
    rng = np.random.default_rng(5)
    M, N, K = 70, 90, 256
    ac = rng.integers(0, 256, (M, K // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    am = (rng.integers(0, 2 ** 24, (M, K // 64)).astype(np.uint32) << 8) | rng.integers(100, 220, (M, K // 64)).astype(np.uint32)
    wm = (rng.integers(0, 2 ** 24, (N, K // 64)).astype(np.uint32) << 8) | rng.integers(100, 220, (N, K // 64)).astype(np.uint32)
    am[3, 1] |= 0xFF
    wm[7, 2] |= 0xFF
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
    c = h.hif4_gemm(h.HIF4_A_HIF4, *dev_packed(ac, am), *dev_packed(wc, wm), out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    got = c.cpu().numpy().astype(np.float64)
    nan_want = np.isnan(want)
    assert nan_want[3].all() and nan_want[:, 7].all() and nan_want.sum() == N + M - 1
    assert (np.isnan(got) == nan_want).all()
    ok = ~nan_want
    assert np.linalg.norm(got[ok] - want[ok]) <= TOL * np.linalg.norm(want[ok])
    # each row against its own norm as well: rows differ by many binades
    for r in range(M):
        if r != 3:
            k = ok[r]
            assert np.linalg.norm(got[r][k] - want[r][k]) <= TOL * np.linalg.norm(want[r][k])


def test_gemm_extreme_scales(h, oracle):
    """Largest and smallest finite units: no overflow to inf, no flush to zero."""
    K = 64
    codes = np.full((2, 32), 0x77, np.uint8)
    hi = np.array([[0xFFFFFFFE]], np.uint32)
    lo = np.array([[0x00000000]], np.uint32)
    am = np.concatenate([hi, lo])
    wm = np.concatenate([hi, lo])
    want = oracle.gemm_f64(oracle.dequantize(codes, am), oracle.dequantize(codes, wm))
    c = h.hif4_gemm(h.HIF4_A_HIF4, *dev_packed(codes, am), *dev_packed(codes, wm), out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    got = c.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all() and (got != 0).all()
    assert np.abs(got / want - 1).max() < 1e-6


def test_gemm_empty_and_k0(h):
    wc = torch.zeros((8, 0), dtype=torch.uint8, device="cuda")
    wm = torch.zeros((8, 0), dtype=torch.int32, device="cuda")
    ac = torch.zeros((4, 0), dtype=torch.uint8, device="cuda")
    am = torch.zeros((4, 0), dtype=torch.int32, device="cuda")
    c = torch.full((4, 8), 3.0, dtype=torch.float32, device="cuda")
    h.hif4_gemm(h.HIF4_A_HIF4, ac, am, wc, wm, out_dtype=h.HIF4_OUT_F32, c=c)
    torch.cuda.synchronize()
    assert (c == 0).all()
    c0 = h.hif4_gemm(h.HIF4_A_HIF4, torch.zeros((0, 32), dtype=torch.uint8, device="cuda"),
                     torch.zeros((0, 1), dtype=torch.int32, device="cuda"),
                     torch.zeros((8, 32), dtype=torch.uint8, device="cuda"),
                     torch.zeros((8, 1), dtype=torch.int32, device="cuda"))
    assert c0.shape == (0, 8)


@pytest.mark.parametrize("counts", [[0, 130, 1, 300, 77, 0], [5], [128, 128, 128], [0, 0, 257]])
def test_grouped_gemm(h, oracle, counts):
    E, N, K = len(counts), 300, 256
    M = int(sum(counts))
    offs = np.zeros(E + 1, np.int32)
    offs[1:] = np.cumsum(counts)
    rng = np.random.default_rng(E + M)
    ab, (ac, am), _ = quantized_operands(oracle, M, 1, K, 900 + M)
    w = rng.standard_normal((E * N, K)) * 0.02
    wc, wm = oracle.quantize(synth.bits(torch.from_numpy(w).to(torch.bfloat16)))
    adec, wdec = oracle.dequantize(ac, am), oracle.dequantize(wc, wm)
    want = np.zeros((M, N))
    for e in range(E):
        if counts[e]:
            want[offs[e]:offs[e + 1]] = oracle.gemm_f64(adec[offs[e]:offs[e + 1]], wdec[e * N:(e + 1) * N])
    wcd, wmd = dev_packed(wc.reshape(E, N, K // 2), wm.reshape(E, N, K // 64))
    od = torch.from_numpy(offs).cuda()
    c = torch.full((M, N), 9.0, dtype=torch.float32, device="cuda")
    h.hif4_grouped_gemm(h.HIF4_A_HIF4, *dev_packed(ac, am), wcd, wmd, od, out_dtype=h.HIF4_OUT_F32, c=c)
    cq = h.hif4_grouped_gemm(h.HIF4_A_BF16_QUANTIZE, synth.from_bits(ab).cuda(), None, wcd, wmd, od, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    got = c.cpu().numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL
    assert torch.equal(c, cq)


@pytest.mark.parametrize("counts,N,K", [([100, 0, 130], 96, 2048), ([300, 200], 200, 1024), ([40, 50, 60, 1], 8300, 2048)])
def test_grouped_gemm_few_experts_k_split(h, oracle, counts, N, K):
    """Few experts against a long K: the grouped call has too few workgroups for the chip and splits K over the wave
    groups of a workgroup, as the dense few-row calls do (128-, 256- and 64-row tiles; 4 and 8 waves)."""
    E, M = len(counts), int(sum(counts))
    offs = np.zeros(E + 1, np.int32)
    offs[1:] = np.cumsum(counts)
    rng = np.random.default_rng(E * 1000 + M)
    ab, (ac, am), _ = quantized_operands(oracle, M, 1, K, 5150 + M)
    w = rng.standard_normal((E * N, K)) * 0.02
    wc, wm = oracle.quantize(synth.bits(torch.from_numpy(w).to(torch.bfloat16)))
    adec, wdec = oracle.dequantize(ac, am), oracle.dequantize(wc, wm)
    want = np.zeros((M, N))
    for e in range(E):
        if counts[e]:
            want[offs[e]:offs[e + 1]] = oracle.gemm_f64(adec[offs[e]:offs[e + 1]], wdec[e * N:(e + 1) * N])
    wcd, wmd = dev_packed(wc.reshape(E, N, K // 2), wm.reshape(E, N, K // 64))
    od = torch.from_numpy(offs).cuda()
    c = h.hif4_grouped_gemm(h.HIF4_A_HIF4, *dev_packed(ac, am), wcd, wmd, od, out_dtype=h.HIF4_OUT_F32)
    cq = h.hif4_grouped_gemm(h.HIF4_A_BF16_QUANTIZE, synth.from_bits(ab).cuda(), None, wcd, wmd, od, out_dtype=h.HIF4_OUT_F32)
    ck = h.hif4_grouped_gemm(h.HIF4_A_BF16_KEEP, synth.from_bits(ab).cuda(), None, wcd, wmd, od, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    assert rel_fro(c.cpu().numpy().astype(np.float64), want) <= TOL
    assert torch.equal(c, cq)
    want_k = np.zeros((M, N))
    for e in range(E):
        if counts[e]:
            want_k[offs[e]:offs[e + 1]] = oracle.gemm_f64(ab[offs[e]:offs[e + 1]], wdec[e * N:(e + 1) * N])
    assert rel_fro(ck.cpu().numpy().astype(np.float64), want_k) <= TOL


def test_grouped_gemm_random_routings(h, oracle):
    """A seeded sweep of the grouped call: 1 to 12 experts with 0 to 330 rows each (so the mean row count selects every
    tile height of the few-row kernel, and single experts overflow a tile), ragged N, 1 to 12 units of K, all kinds
    of A, the weight-only kind with and without its optional workspace, strided output."""
    rng = np.random.default_rng(424242)
    for case in range(30):
        E = int(rng.integers(1, 13))
        top = int(rng.choice([20, 70, 140, 200, 330]))
        counts = rng.integers(0, top + 1, E)
        if case % 5 == 0:
            counts[rng.integers(0, E)] = 0
        M, N, K = int(counts.sum()), int(rng.integers(1, 400)), 64 * int(rng.integers(1, 13))
        if M == 0:
            counts[0], M = 3, 3
        kind = (h.HIF4_A_HIF4, h.HIF4_A_BF16_QUANTIZE, h.HIF4_A_BF16_KEEP)[case % 3]
        with_ws = bool(rng.integers(0, 2))
        print(f"case {case}: counts={counts.tolist()} N={N} K={K} kind={kind} ws={with_ws}", flush=True)
        offs = np.zeros(E + 1, np.int32)
        offs[1:] = np.cumsum(counts)
        ab, (ac, am), _ = quantized_operands(oracle, M, 1, K, 31000 + case)
        w = rng.standard_normal((E * N, K)) * 0.02
        wc, wm = oracle.quantize(synth.bits(torch.from_numpy(w).to(torch.bfloat16)))
        aval = ab if kind == h.HIF4_A_BF16_KEEP else oracle.dequantize(ac, am)
        wdec = oracle.dequantize(wc, wm)
        want = np.zeros((M, N))
        for e in range(E):
            if counts[e]:
                want[offs[e]:offs[e + 1]] = oracle.gemm_f64(aval[offs[e]:offs[e + 1]], wdec[e * N:(e + 1) * N])
        wcd, wmd = dev_packed(wc.reshape(E, N, K // 2), wm.reshape(E, N, K // 64))
        od = torch.from_numpy(offs).cuda()
        if kind == h.HIF4_A_HIF4:
            a_dev, am_dev = dev_packed(ac, am)
        else:
            a_dev, am_dev = synth.from_bits(ab).cuda(), None
        ws = None
        if kind == h.HIF4_A_BF16_KEEP and not with_ws:
            ws = torch.empty(16, dtype=torch.uint8, device="cuda")
        cbuf = torch.full((M, N + 5), 3.0, dtype=torch.float32, device="cuda")
        h.hif4_grouped_gemm(kind, a_dev, am_dev, wcd, wmd, od, out_dtype=h.HIF4_OUT_F32, c=cbuf[:, :N], workspace=ws)
        torch.cuda.synchronize()
        assert (cbuf[:, N:] == 3.0).all()
        assert rel_fro(cbuf[:, :N].double().cpu().numpy(), want) <= TOL, case


def test_gemm_prefill_shape_sampled(h, oracle):
    """M=4096, N=11008, K=4096 (the W4A4 prefill configuration): a seeded sample of rows x columns."""
    M, N, K = 4096, 11008, 4096
    a = synth.activation_channel_outliers(M, K)
    w = synth.weight_gaussian(N, K, 0.02, config=3)
    wc, wm = oracle.quantize(synth.bits(w))
    wcd, wmd = dev_packed(wc, wm)
    c = h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a.cuda(), None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    rows = np.sort(np.concatenate([rng.choice(M, 94, replace=False), [0, M - 1]]))
    cols = np.sort(np.concatenate([rng.choice(N, 94, replace=False), [0, N - 1]]))
    ac, am = oracle.quantize(synth.bits(a)[rows])
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc[cols], wm[cols]))
    got = c[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL, rel_fro(got, want)


@pytest.mark.parametrize("M,N,K", [(16, 256, 512), (1, 16, 64), (5, 100, 192), (16, 1000, 1088), (17, 48, 256),
                                   (33, 130, 320), (64, 64, 128), (65, 300, 256), (300, 520, 448)])
def test_gemm_weight_only(h, oracle, M, N, K):
    """HiF4 weights, BF16 activations used as they are."""
    print(f"weight-only parity M={M} N={N} K={K}", flush=True)
    ab, _, (wc, wm) = quantized_operands(oracle, M, N, K, 500 + M + N + K)
    want = oracle.gemm_f64(ab, oracle.dequantize(wc, wm))
    a = synth.from_bits(ab).cuda()
    wcd, wmd = dev_packed(wc, wm)
    c32 = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    c16 = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_BF16)
    torch.cuda.synchronize()
    got = c32.cpu().numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL, rel_fro(got, want)
    wb = synth.bits(torch.from_numpy(want).to(torch.bfloat16)).astype(np.int32)
    gb = synth.bits(c16.cpu()).astype(np.int32)
    key = lambda b: np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    assert np.abs(key(gb) - key(wb)).max() <= 1


def test_gemm_weight_only_decode_config(h, oracle):
    """M=16, N=4096, K=4096: per-channel scaled weights, full output against the oracle."""
    M, N, K = 16, 4096, 4096
    w = synth.weight_gaussian(N, K, 0.02, config=2, channel_scale=True)
    a = synth.activation_gaussian(M, K, config=2)
    wc, wm = oracle.quantize(synth.bits(w))
    want = oracle.gemm_f64(synth.bits(a), oracle.dequantize(wc, wm))
    c = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a.cuda(), None, *dev_packed(wc, wm), out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    assert rel_fro(c.cpu().numpy().astype(np.float64), want) <= TOL


def test_grouped_gemm_weight_only(h, oracle):
    counts = [40, 0, 200, 3]
    E, N, K = len(counts), 270, 192
    M = sum(counts)
    offs = np.zeros(E + 1, np.int32)
    offs[1:] = np.cumsum(counts)
    rng = np.random.default_rng(8)
    ab = synth.bits(torch.from_numpy(rng.standard_normal((M, K))).to(torch.bfloat16))
    wc, wm = oracle.quantize(synth.bits(torch.from_numpy(rng.standard_normal((E * N, K)) * 0.02).to(torch.bfloat16)))
    wdec = oracle.dequantize(wc, wm)
    want = np.concatenate([oracle.gemm_f64(ab[offs[e]:offs[e + 1]], wdec[e * N:(e + 1) * N]) for e in range(E)])
    wcd, wmd = dev_packed(wc.reshape(E, N, K // 2), wm.reshape(E, N, K // 64))
    ad = synth.from_bits(ab).cuda()
    c = h.hif4_grouped_gemm(h.HIF4_A_BF16_KEEP, ad, None, wcd, wmd, torch.from_numpy(offs).cuda(), out_dtype=h.HIF4_OUT_F32)
    # without room for a reordered copy of A (the workspace is optional for this kind): the other kernel
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    c2 = h.hif4_grouped_gemm(h.HIF4_A_BF16_KEEP, ad, None, wcd, wmd, torch.from_numpy(offs).cuda(), out_dtype=h.HIF4_OUT_F32,
                             workspace=tiny)
    torch.cuda.synchronize()
    assert rel_fro(c.cpu().numpy().astype(np.float64), want) <= TOL
    assert rel_fro(c2.cpu().numpy().astype(np.float64), want) <= TOL


def test_grouped_gemm_moe_config_sampled(h, oracle):
    """64 experts, K=7168, N=2048, 8192 routed rows: two rows of every non-empty expert against the oracle."""
    E, K, N = 64, 7168, 2048
    offs = synth.moe_offsets()
    M = int(offs[-1])
    assert M == 8192
    a = synth.activation_gaussian(M, K, config=4)
    g = torch.Generator(device="cuda").manual_seed(44)
    w = (torch.randn((E * N, K), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    wcd, wmd = h.hif4_quantize(w)   # encoder output is checked against the oracle on the sampled rows below
    c = h.hif4_grouped_gemm(h.HIF4_A_BF16_QUANTIZE, a.cuda(), None, wcd.view(E, N, K // 2), wmd.view(E, N, K // 64),
                            torch.from_numpy(offs).cuda(), out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    cols = np.sort(rng.choice(N, 48, replace=False))
    errs, refs = 0.0, 0.0
    for e in range(E):
        lo, hi = int(offs[e]), int(offs[e + 1])
        if hi == lo:
            continue
        rows = np.unique([lo, hi - 1])
        ac, am = oracle.quantize(synth.bits(a)[rows])
        wrows = torch.from_numpy(e * N + cols).cuda()
        wb = synth.bits(w[wrows].cpu())
        wc, wm = oracle.quantize(wb)
        assert (wcd[wrows].cpu().numpy() == wc).all() and (wmd[wrows].cpu().numpy().view(np.uint32) == wm).all()
        want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
        got = c[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.float64)
        errs += np.sum((got - want) ** 2)
        refs += np.sum(want ** 2)
    assert np.sqrt(errs / refs) <= TOL


@pytest.mark.parametrize("kind", ["hif4", "quantize", "keep"])
def test_gemm_many_rows_decoded_w_workspace(h, oracle, kind):
    """From 1536 rows on (3328 against more than 128 Mi weights), a workspace of hif4_gemm_workspace_bytes_decoded_w() bytes makes a call on two
    HiF4 operands decode W once instead of inside the main loop: the same exact products, added in fp32 in
    another grouping, so the two results agree far inside the tolerance, and both are within it of the oracle."""
    M, N, K = 8192 + 77, 300, 320
    print(f"gemm decoded-W path kind={kind} M={M} N={N} K={K}", flush=True)
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 977)
    wcd, wmd = dev_packed(wc, wm)
    a_bf16 = synth.from_bits(ab).cuda()
    if kind == "keep":
        a_kind, a_dev, am_dev = h.HIF4_A_BF16_KEEP, a_bf16, None
        want = oracle.gemm_f64(ab, oracle.dequantize(wc, wm))
    else:
        want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
        if kind == "hif4":
            a_kind = h.HIF4_A_HIF4
            a_dev, am_dev = dev_packed(ac, am)
        else:
            a_kind, a_dev, am_dev = h.HIF4_A_BF16_QUANTIZE, a_bf16, None
    small = h.hif4_gemm_workspace_bytes(a_kind, M, K)
    big = h.hif4_gemm_workspace_bytes_decoded_w(a_kind, M, N, K)
    assert big >= small + N * K * 2 + (M * K * 2 if kind == "keep" else 0)  # BF16 activations: a reordered copy of A as well
    assert h.hif4_gemm_workspace_bytes_decoded_w(a_kind, 1535, 11008, 4096) == h.hif4_gemm_workspace_bytes(a_kind, 1535, 4096)
    assert h.hif4_gemm_workspace_bytes_decoded_w(a_kind, 1536, 11008, 4096) > h.hif4_gemm_workspace_bytes(a_kind, 1536, 4096)
    assert h.hif4_gemm_workspace_bytes_decoded_w(a_kind, 3327, 28672, 8192) == h.hif4_gemm_workspace_bytes(a_kind, 3327, 8192)
    assert h.hif4_gemm_workspace_bytes_decoded_w(a_kind, 3328, 28672, 8192) > h.hif4_gemm_workspace_bytes(a_kind, 3328, 8192)
    ws_small = torch.empty(max(small, 16), dtype=torch.uint8, device="cuda")
    ws_big = torch.empty(max(big, 16), dtype=torch.uint8, device="cuda")
    c_small = h.hif4_gemm(a_kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_F32, workspace=ws_small)
    c_big = h.hif4_gemm(a_kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_F32, workspace=ws_big)
    c_default = h.hif4_gemm(a_kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    got = c_big.cpu().numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL, rel_fro(got, want)
    assert rel_fro(c_small.cpu().numpy().astype(np.float64), want) <= TOL
    assert torch.equal(c_default, c_big)
    assert rel_fro(c_small.cpu().numpy().astype(np.float64), got) <= 1e-6


@pytest.mark.parametrize("kind", ["hif4", "keep"])
@pytest.mark.parametrize("M,N,K", [(1600, 11000, 128), (3336, 7000, 192), (2136, 11000, 64), (2336, 16250, 64)])
def test_gemm_decoded_operands_columns_in_two_tile_widths(h, oracle, kind, M, N, K):
    """Calls on decoded operands whose 256 x 256 tiles would leave the last round of workgroups mostly empty run whole
    rounds of 256-column tiles first and the remaining columns in tiles of 192 or 128 columns (a second launch): the
    whole result against the oracle, ragged in both directions, and bit for bit equal in BF16 and fp32 output kinds
    (the order of an output's additions over K does not depend on the tile it falls in)."""
    main, width = h.hif4_gemm_plan_planes_split(M, N)
    print(f"gemm split kind={kind} M={M} N={N} K={K} main={main} width={width}", flush=True)
    assert width in (192, 128)
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 31 + M)
    wcd, wmd = dev_packed(wc, wm)
    if kind == "keep":
        a_kind, a_dev, am_dev = h.HIF4_A_BF16_KEEP, synth.from_bits(ab).cuda(), None
        want = oracle.gemm_f64(ab, oracle.dequantize(wc, wm))
    else:
        a_kind = h.HIF4_A_HIF4
        a_dev, am_dev = dev_packed(ac, am)
        want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
    big = h.hif4_gemm_workspace_bytes_decoded_w(a_kind, M, N, K)
    assert h.hif4_gemm_plan_name(h.hif4_gemm_plan(a_kind, M, N, K, workspace_bytes=big)) == "hif4::gemm_planes16_kernel"
    ws = torch.empty(big, dtype=torch.uint8, device="cuda")
    cbuf = torch.full((M, N + 5), 3.0, dtype=torch.float32, device="cuda")
    c32 = h.hif4_gemm(a_kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_F32, c=cbuf[:, :N], workspace=ws)
    c16 = h.hif4_gemm(a_kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_BF16, workspace=ws)
    torch.cuda.synchronize()
    assert (cbuf[:, N:] == 3.0).all()
    assert rel_fro(c32.double().cpu().numpy(), want) <= TOL
    assert torch.equal(c16, c32.to(torch.bfloat16))


def test_gemm_many_rows_many_tiles_sampled(h, oracle):
    """16384 x 2048 x 8192 with the activations quantised inside the call: 512 tiles over the whole chip
    through the decoded-operand path (the launch shape of the large prefill benchmark leg, fewer
    columns); a seeded sample of rows x columns against the oracle."""
    M, N, K = 16384, 2048, 8192
    print(f"gemm sampled M={M} N={N} K={K}", flush=True)
    g = torch.Generator().manual_seed(synth.BASE_SEED + 55)
    z = torch.randn((M, K), generator=g)
    chi = torch.randn((4, M, K), generator=g).pow(2).sum(0)
    a = (z / torch.sqrt(chi / 4.0) / np.sqrt(2.0)).to(torch.bfloat16)      # Student-t(4), unit variance
    del z, chi
    w = synth.weight_gaussian(N, K, 0.015, config=5)
    wc, wm = oracle.quantize(synth.bits(w))
    wcd, wmd = dev_packed(wc, wm)
    ad = a.cuda()
    big = h.hif4_gemm_workspace_bytes_decoded_w(h.HIF4_A_BF16_QUANTIZE, M, N, K)
    assert big > h.hif4_gemm_workspace_bytes(h.HIF4_A_BF16_QUANTIZE, M, K)
    c = h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, ad, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32,
                    workspace=torch.empty(big, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    rows = np.sort(np.concatenate([rng.choice(M, 94, replace=False), [0, M - 1]]))
    cols = np.sort(np.concatenate([rng.choice(N, 94, replace=False), [0, N - 1]]))
    ac, am = oracle.quantize(synth.bits(a)[rows])
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc[cols], wm[cols]))
    got = c[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL, rel_fro(got, want)


def test_gemm_equals_fake_quant_linear(h):
    """The "simulated format" linear layer (quantise, dequantise, then a matrix product of the
    dequantised BF16 values, as in the paper's accuracy experiments) is what hif4_gemm with activations
    quantised inside computes: decoded values are exact in BF16, so only the fp32 summation order differs."""
    M, N, K = 200, 300, 1024
    g = torch.Generator(device="cuda").manual_seed(3)
    a = torch.randn((M, K), generator=g, device="cuda").to(torch.bfloat16)
    w = (torch.randn((N, K), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    wc, wm = h.hif4_quantize(w)
    a_fq = h.hif4_dequantize(*h.hif4_quantize(a))
    w_fq = h.hif4_dequantize(wc, wm)
    want = a_fq.double() @ w_fq.double().T
    got = h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, out_dtype=h.HIF4_OUT_F32).double()
    rel = (torch.linalg.norm(got - want) / torch.linalg.norm(want)).item()
    assert rel <= 1e-5, rel


@pytest.mark.parametrize("kind", ["hif4", "quantize", "keep"])
@pytest.mark.parametrize("M,N,K,mode", [(1, 64, 64, 0), (2100, 320, 512, 0), (2305, 576, 192, 1), (300, 22016, 128, 0),
                                        # decoded operands, columns cut into a launch of 256-column tiles and one of narrower tiles
                                        (3336, 7040, 128, 1)])
def test_gemm_to_hif4_equals_gemm_then_quantize(h, oracle, kind, M, N, K, mode):
    """The HiF4-emitting epilogue gives hif4_quantize(BF16 result of hif4_gemm) bit for bit (same products,
    same summation order, same BF16 rounding, Algorithm 1 with the encoder's arithmetic); the BF16 result
    and the encoder are each checked against the oracle elsewhere, and here the oracle's encoder is applied
    to the GPU's BF16 result as well.  Shapes on which hif4_gemm runs the same main loop as the emitting
    call (and one unit of K, whose sums are exact in any order)."""
    print(f"gemm_to_hif4 kind={kind} M={M} N={N} K={K} mode={mode}", flush=True)
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 4242 + M)
    wcd, wmd = dev_packed(wc, wm)
    if kind == "keep":
        a_kind, a_dev, am_dev = h.HIF4_A_BF16_KEEP, synth.from_bits(ab).cuda(), None
    elif kind == "hif4":
        a_kind = h.HIF4_A_HIF4
        a_dev, am_dev = dev_packed(ac, am)
    else:
        a_kind, a_dev, am_dev = h.HIF4_A_BF16_QUANTIZE, synth.from_bits(ab).cuda(), None
    c16 = h.hif4_gemm(a_kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_BF16)
    want_c, want_m = h.hif4_quantize(c16, round_mode=mode)
    got_c, got_m = h.hif4_gemm_to_hif4(a_kind, a_dev, am_dev, wcd, wmd, round_mode=mode)
    torch.cuda.synchronize()
    assert torch.equal(got_m, want_m)
    assert torch.equal(got_c, want_c)
    oc, om = oracle.quantize(synth.bits(c16.cpu()), mode)
    assert (got_c.cpu().numpy() == oc).all() and (got_m.cpu().numpy().view(np.uint32) == om).all()


@pytest.mark.parametrize("kind", ["hif4", "quantize", "keep"])
@pytest.mark.parametrize("M,N,K", [(70, 1024, 1088), (300, 320, 512), (100, 256, 2048), (150, 384, 1024), (16, 128, 512),
                                   (40, 8320, 4096), (600, 4096, 1024)])
def test_gemm_to_hif4_small_shapes(h, oracle, kind, M, N, K):
    """Shapes on which the emitting call runs the few-row kernel (one or several m-tiles, with and without K split,
    its epilogue parking the tile in LDS).  hif4_gemm may run another kernel there (up to 64 rows) or the same one
    with other wave counts, so the BF16 values agree to fp32 summation accuracy only: nearly every unit is identical,
    and decoded the result lies within HiF4's error of the fp64 product."""
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 515 + M)
    wcd, wmd = dev_packed(wc, wm)
    if kind == "keep":
        a_kind, a_dev, am_dev, a_val = h.HIF4_A_BF16_KEEP, synth.from_bits(ab).cuda(), None, ab
    elif kind == "hif4":
        a_kind, a_val = h.HIF4_A_HIF4, oracle.dequantize(ac, am)
        a_dev, am_dev = dev_packed(ac, am)
    else:
        a_kind, a_dev, am_dev, a_val = h.HIF4_A_BF16_QUANTIZE, synth.from_bits(ab).cuda(), None, oracle.dequantize(ac, am)
    c16 = h.hif4_gemm(a_kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_BF16)
    got_c, got_m = h.hif4_gemm_to_hif4(a_kind, a_dev, am_dev, wcd, wmd)
    torch.cuda.synchronize()
    gc, gm = got_c.cpu().numpy(), got_m.cpu().numpy().view(np.uint32)
    # the oracle's encoder on the call's own BF16 result
    oc, om = oracle.quantize(synth.bits(c16.cpu()))
    differing = (gm != om) | (gc.reshape(M, N // 64, 32) != oc.reshape(M, N // 64, 32)).any(axis=2)
    if M > 64:   # the same main loop with the same split of K: the planes are the oracle's, bit for bit
        assert not differing.any(), int(differing.sum())
    else:
        assert differing.mean() <= 2e-3, differing.mean()
    # every element, equal unit or not, against the fp64 product: within half a step of its own unit's grid (Algorithm 1
    # rounds to the nearest multiple of a quarter of E6M2 * 2^(E1_8 + E1_16)), plus the BF16 roundings on the way (the
    # result to BF16, the scaled value to BF16) and the fp32 accumulation error; clamped codes are exempt
    want = oracle.gemm_f64(a_val, oracle.dequantize(wc, wm))
    got = oracle.bf16_bits_to_f64(oracle.dequantize(gc, gm))
    e6 = np.array([oracle.e6m2_to_f64(int(b)) for b in range(255)] + [np.nan])[gm & 0xFF]          # [M, N/64]
    e8 = ((gm[:, :, None] >> (8 + np.arange(8))) & 1).repeat(8, axis=2)                             # [M, N/64, 64]
    e16 = ((gm[:, :, None] >> (16 + np.arange(16))) & 1).repeat(4, axis=2)
    step = (0.25 * e6[:, :, None] * 2.0 ** (e8 + e16)).reshape(M, N)
    from layout import codes_to_nibbles
    mag = codes_to_nibbles(gc) & 7
    bound = 0.5 * step + np.abs(want) * 2.0 ** -6.5 + 1e-5 * np.abs(want).max()
    free = mag < 7
    assert (np.abs(got - want)[free] <= bound[free]).all()
    assert rel_fro(got, want) <= 0.12, rel_fro(got, want)


@pytest.mark.parametrize("kind", ["hif4", "quantize", "keep"])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("counts,N,K", [([0, 130, 1, 300, 77, 0], 320, 256), ([128, 128, 128], 256, 512), ([40, 50, 60, 1], 8320, 2048),
                                        ([100, 0, 130], 128, 2048)])
def test_grouped_gemm_to_hif4_equals_oracle_encoding_of_bf16_result(h, oracle, kind, mode, counts, N, K):
    """The grouped call whose result leaves as HiF4: the planes are the oracle's Algorithm 1 on the BF16 rows that
    hif4_grouped_gemm writes with the same workspace, bit for bit; rows of no expert stay untouched."""
    E, M = len(counts), int(sum(counts))
    offs = np.zeros(E + 1, np.int32)
    offs[1:] = np.cumsum(counts)
    rng = np.random.default_rng(E * 77 + M + N)
    ab, (ac, am), _ = quantized_operands(oracle, M, 1, K, 4100 + M)
    wc, wm = oracle.quantize(synth.bits(torch.from_numpy(rng.standard_normal((E * N, K)) * 0.02).to(torch.bfloat16)))
    wcd, wmd = dev_packed(wc.reshape(E, N, K // 2), wm.reshape(E, N, K // 64))
    od = torch.from_numpy(offs).cuda()
    if kind == "hif4":
        a_kind = h.HIF4_A_HIF4
        a_dev, am_dev = dev_packed(ac, am)
    else:
        a_kind = h.HIF4_A_BF16_KEEP if kind == "keep" else h.HIF4_A_BF16_QUANTIZE
        a_dev, am_dev = synth.from_bits(ab).cuda(), None
    c16 = h.hif4_grouped_gemm(a_kind, a_dev, am_dev, wcd, wmd, od, out_dtype=h.HIF4_OUT_BF16)
    cc = torch.full((M, N // 2), 0xAB, dtype=torch.uint8, device="cuda")
    cm = torch.full((M, N // 64), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    h.hif4_grouped_gemm_to_hif4(a_kind, a_dev, am_dev, wcd, wmd, od, round_mode=mode, c_codes=cc, c_meta=cm)
    torch.cuda.synchronize()
    oc, om = oracle.quantize(synth.bits(c16.cpu()), mode)
    assert (cc.cpu().numpy() == oc).all()
    assert (cm.cpu().numpy().view(np.uint32) == om).all()
    if kind == "keep":   # without room for a reordered copy of A the tile kernel takes the call: its epilogue too
        tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
        c16t = h.hif4_grouped_gemm(a_kind, a_dev, am_dev, wcd, wmd, od, out_dtype=h.HIF4_OUT_BF16, workspace=tiny)
        cct, cmt = h.hif4_grouped_gemm_to_hif4(a_kind, a_dev, am_dev, wcd, wmd, od, round_mode=mode, workspace=tiny)
        torch.cuda.synchronize()
        oct_, omt = oracle.quantize(synth.bits(c16t.cpu()), mode)
        assert (cct.cpu().numpy() == oct_).all() and (cmt.cpu().numpy().view(np.uint32) == omt).all()


def test_gemm_to_hif4_many_rows_and_k0(h, oracle):
    """Through the decoded-operand kernel (3328+ rows, large workspace), and the empty sum."""
    M, N, K = 8192 + 40, 192, 256
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 99)
    wcd, wmd = dev_packed(wc, wm)
    acd, amd = dev_packed(ac, am)
    c16 = h.hif4_gemm(h.HIF4_A_HIF4, acd, amd, wcd, wmd, out_dtype=h.HIF4_OUT_BF16)
    want_c, want_m = h.hif4_quantize(c16)
    got_c, got_m = h.hif4_gemm_to_hif4(h.HIF4_A_HIF4, acd, amd, wcd, wmd)
    assert torch.equal(got_m, want_m) and torch.equal(got_c, want_c)
    # K == 0: C = 0, the all-zero unit everywhere
    a0 = torch.empty((5, 0), dtype=torch.uint8, device="cuda")
    am0 = torch.empty((5, 0), dtype=torch.int32, device="cuda")
    w0 = torch.empty((128, 0), dtype=torch.uint8, device="cuda")
    m0 = torch.empty((128, 0), dtype=torch.int32, device="cuda")
    cc = torch.full((5, 64), 0xAB, dtype=torch.uint8, device="cuda")
    cm = torch.full((5, 2), -1, dtype=torch.int32, device="cuda")
    h.hif4_gemm_to_hif4(h.HIF4_A_HIF4, a0, am0, w0, m0, c_codes=cc, c_meta=cm)
    assert not cc.any() and not cm.any()


@pytest.mark.parametrize("M,N,K", [(64, 12288, 1024), (33, 12298, 2048 + 128), (48, 14000, 512), (40, 16384, 128),
                                   (16, 8192, 4096), (64, 12288, 192)])
def test_gemm_weight_only_wide_weights(h, oracle, M, N, K):
    """33 to 64 rows against 12288 or more columns, K a multiple of 128: the column-split kernel, whole K per
    wave, activations through LDS by direct loads.  (The last two shapes stay on the other kernel.)"""
    print(f"weight-only streaming M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M * 7 + N)
    a = synth.to_bf16(rng.standard_normal((M, K)))
    w = synth.weight_gaussian(N, K, 0.02, config=2, tensor=3 + M, channel_scale=True)
    wc, wm = oracle.quantize(synth.bits(w))
    # a NaN unit and an all-zero unit in the weights, a subnormal activation
    wm[3, 1] = 0xFF
    wc[3, 32:64] = 0
    wm[5, 0] = 0
    wc[5, :32] = 0
    ab = synth.bits(a).copy()
    ab[M - 1, K - 1] = 0x0001
    want = oracle.gemm_f64(ab, oracle.dequantize(wc, wm))
    wcd, wmd = dev_packed(wc, wm)
    ad = synth.from_bits(ab).cuda()
    c32 = h.hif4_gemm(h.HIF4_A_BF16_KEEP, ad, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    c16 = h.hif4_gemm(h.HIF4_A_BF16_KEEP, ad, None, wcd, wmd, out_dtype=h.HIF4_OUT_BF16)
    torch.cuda.synchronize()
    got = c32.cpu().numpy().astype(np.float64)
    nan = np.isnan(want)
    assert nan[:, 3].all() and (np.isnan(got) == nan).all()
    assert rel_fro(got[~nan], want[~nan]) <= TOL, rel_fro(got[~nan], want[~nan])
    # BF16 output: one BF16 ulp of the exact value, plus the fp32 summation error, which matters for the few
    # of the 100 000+ sums that cancel to almost nothing
    g16 = c16.double().cpu().numpy()
    ok = np.abs(g16[~nan] - want[~nan]) <= 2.0 ** -8 * np.abs(want[~nan]) + 1e-5 * np.abs(want[~nan]).max()
    assert ok.all()


def test_grouped_gemm_many_experts(h, oracle):
    """More experts than lanes of a wave (the search for an m-tile's expert runs 64 experts at a time),
    many of them empty, sizes from 0 to 300 rows."""
    rng = np.random.default_rng(21)
    E, N, K = 150, 96, 128
    counts = rng.choice([0, 0, 1, 3, 40, 128, 129, 256, 300], size=E)
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    M = int(offs[-1])
    print(f"grouped gemm E={E} rows={M}", flush=True)
    ab, (ac, am), _ = quantized_operands(oracle, M, 8, K, 5)
    w = synth.to_bf16(rng.standard_normal((E * N, K)) * 0.02)
    wc, wm = oracle.quantize(synth.bits(w))
    adec, wdec = oracle.dequantize(ac, am), oracle.dequantize(wc, wm)
    want = np.zeros((M, N))
    for e in range(E):
        lo, hi = offs[e], offs[e + 1]
        if hi > lo:
            want[lo:hi] = oracle.gemm_f64(adec[lo:hi], wdec[e * N:(e + 1) * N])
    acd, amd = dev_packed(ac, am)
    wcd, wmd = dev_packed(wc, wm)
    c = h.hif4_grouped_gemm(h.HIF4_A_HIF4, acd, amd, wcd.view(E, N, K // 2), wmd.view(E, N, K // 64),
                            torch.from_numpy(offs).cuda(), out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    got = c.cpu().numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL, rel_fro(got, want)


@pytest.mark.parametrize("M,N,K", [(16, 272, 256), (40, 12288, 256), (64, 300, 256)])
def test_gemm_weight_only_strided_rows(h, oracle, M, N, K):
    """Row strides larger than the row length for A and C in the two few-row kernels; nothing is written
    between the rows of C."""
    rng = np.random.default_rng(M + N)
    a = synth.to_bf16(rng.standard_normal((M, K)))
    w = synth.to_bf16(rng.standard_normal((N, K)) * 0.02)
    wc, wm = oracle.quantize(synth.bits(w))
    wcd, wmd = dev_packed(wc, wm)
    abuf = torch.full((M, K + 64), 7.0, dtype=torch.bfloat16, device="cuda")
    abuf[:, :K] = a.cuda()
    cbuf = torch.full((M, N + 24), -1.0, dtype=torch.float32, device="cuda")
    h.hif4_gemm(h.HIF4_A_BF16_KEEP, abuf[:, :K], None, wcd, wmd, out_dtype=h.HIF4_OUT_F32, c=cbuf[:, :N])
    c = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a.cuda(), None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    assert torch.equal(cbuf[:, :N], c) and (cbuf[:, N:] == -1.0).all()
    want = oracle.gemm_f64(synth.bits(a), oracle.dequantize(wc, wm))
    assert rel_fro(c.cpu().numpy().astype(np.float64), want) <= TOL


def test_gemm_large_prefill_config_sampled(h, oracle):
    """M=16384, N=28672, K=8192 (the large prefill configuration, as the benchmark launches it: activations
    quantised inside the call, large workspace): a seeded sample of rows x columns against the oracle, and
    the same call with the result leaving as HiF4 against the oracle's encoder on sampled rows."""
    M, N, K = 16384, 28672, 8192
    print(f"gemm sampled M={M} N={N} K={K}", flush=True)
    dev = torch.device("cuda")
    g = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 5)
    a = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
    for r in range(0, M, 4096):   # Student-t(4) scaled to unit variance
        z = torch.randn((4096, K), generator=g, device=dev)
        chi = torch.randn((4, 4096, K), generator=g, device=dev).pow(2).sum(0)
        a[r:r + 4096] = (z / torch.sqrt(chi / 4.0) / np.sqrt(2.0)).to(torch.bfloat16)
    del z, chi
    w = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
    for r in range(0, N, 7168):
        w[r:r + 7168] = (torch.randn((7168, K), generator=g, device=dev) * 0.015).to(torch.bfloat16)
    wcd, wmd = h.hif4_quantize(w)
    ws = torch.empty(h.hif4_gemm_workspace_bytes_decoded_w(h.HIF4_A_BF16_QUANTIZE, M, N, K), dtype=torch.uint8, device=dev)
    c = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_BF16, c=c, workspace=ws)
    oc, om = h.hif4_gemm_to_hif4(h.HIF4_A_BF16_QUANTIZE, a, None, wcd, wmd, workspace=ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(55)
    rows = np.sort(np.concatenate([rng.choice(M, 62, replace=False), [0, M - 1]]))
    cols = np.sort(np.concatenate([rng.choice(N, 126, replace=False), [0, N - 1]]))
    ri, ci = torch.from_numpy(rows).to(dev), torch.from_numpy(cols).to(dev)
    # operands of the sample through the oracle: its own encoder on the sampled rows of A and of W
    ac, am = oracle.quantize(synth.bits(a[ri].cpu()))
    wc, wm = oracle.quantize(synth.bits(w[ci].cpu()))
    assert (wcd[ci].cpu().numpy() == wc).all() and (wmd[ci].cpu().numpy().view(np.uint32) == wm).all()
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
    got = c[ri][:, ci].double().cpu().numpy()
    # BF16 output: one BF16 ulp of the exact value plus the fp32 summation error
    assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-5 * np.abs(want).max()).all()
    # HiF4 output of whole sampled rows: the oracle's encoder applied to the GPU's BF16 rows
    ec, em = oracle.quantize(synth.bits(c[ri].cpu()))
    assert (oc[ri].cpu().numpy() == ec).all() and (om[ri].cpu().numpy().view(np.uint32) == em).all()


def test_few_row_and_grouped_kernel_strided_output(h, oracle):
    """The kernel that takes dense calls of at most 192 rows and grouped calls (HiF4 x HiF4): row stride of C
    larger than N, BF16 and fp32 results, nothing written between the rows or past an expert's last row."""
    M, N, K = 150, 290, 320
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 4242)
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
    acd, amd = dev_packed(ac, am)
    wcd, wmd = dev_packed(wc, wm)
    for dt, od in ((torch.float32, h.HIF4_OUT_F32), (torch.bfloat16, h.HIF4_OUT_BF16)):
        cbuf = torch.full((M, N + 22), -1.0, dtype=dt, device="cuda")
        h.hif4_gemm(h.HIF4_A_HIF4, acd, amd, wcd, wmd, out_dtype=od, c=cbuf[:, :N])
        torch.cuda.synchronize()
        assert (cbuf[:, N:] == -1.0).all()
        got = cbuf[:, :N].double().cpu().numpy()
        tol = TOL if dt == torch.float32 else 2.0 ** -8
        assert rel_fro(got, want) <= tol, rel_fro(got, want)
    # grouped: two experts sharing one weight matrix shape, rows 0..89 and 90..149, strided C
    E = 2
    offs = np.array([0, 90, M], np.int32)
    w2c = np.concatenate([wc, wc[::-1]]).reshape(E, N, K // 2)
    w2m = np.concatenate([wm, wm[::-1]]).reshape(E, N, K // 64)
    adec = oracle.dequantize(ac, am)
    want_g = np.concatenate([oracle.gemm_f64(adec[:90], oracle.dequantize(wc, wm)),
                             oracle.gemm_f64(adec[90:], oracle.dequantize(wc[::-1].copy(), wm[::-1].copy()))])
    cbuf = torch.full((M, N + 10), -1.0, dtype=torch.float32, device="cuda")
    h.hif4_grouped_gemm(h.HIF4_A_HIF4, acd, amd, *dev_packed(np.ascontiguousarray(w2c), np.ascontiguousarray(w2m)),
                        torch.from_numpy(offs).cuda(), out_dtype=h.HIF4_OUT_F32, c=cbuf[:, :N])
    torch.cuda.synchronize()
    assert (cbuf[:, N:] == -1.0).all()
    assert rel_fro(cbuf[:, :N].double().cpu().numpy(), want_g) <= TOL


@pytest.mark.parametrize("M,N,K", [(100, 100, 2048), (150, 300, 1024), (30, 8300, 2048), (48, 7000, 4096), (64, 300, 192)])
def test_gemm_few_rows_k_split_other_kinds(h, oracle, M, N, K):
    """The few-row kernel with K split inside the workgroup, reached by the other two kinds of A: quantised in the
    call (fused encode-to-planes pre-pass) and plain BF16 with the optional workspace."""
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 4242 + M)
    wd = oracle.dequantize(wc, wm)
    a = synth.from_bits(ab).cuda()
    wcd, wmd = dev_packed(wc, wm)
    cq = h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    assert rel_fro(cq.cpu().numpy().astype(np.float64), oracle.gemm_f64(oracle.dequantize(ac, am), wd)) <= TOL
    if h.hif4_gemm_workspace_bytes_decoded_w(h.HIF4_A_BF16_KEEP, M, N, K) == M * K * 2:  # the few-row kernel's shapes
        ck = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
        torch.cuda.synchronize()
        assert rel_fro(ck.cpu().numpy().astype(np.float64), oracle.gemm_f64(ab, wd)) <= TOL


@pytest.mark.parametrize("M,N,K", [(512, 4096, 4096), (1024, 2048, 7168), (384, 11008, 4096), (250, 28672, 2048)])
def test_gemm_few_row_kernel_several_m_tiles_sampled(h, oracle, M, N, K):
    """Small dense calls of more than 192 rows run as several m-tiles of the few-row kernel (tiles of 128, 192 or
    256 rows, with or without K split): a seeded sample of rows x columns including both ends, activations
    quantised in the call, and the weight-only kind on the same kernel."""
    gen = torch.Generator().manual_seed(1000 + M)
    a = torch.randn((M, K), generator=gen).to(torch.bfloat16)
    w = (torch.randn((N, K), generator=gen) * 0.02).to(torch.bfloat16)
    wcd, wmd = h.hif4_quantize(w.cuda())
    wc, wm = wcd.cpu().numpy(), wmd.cpu().numpy().view(np.uint32)
    c = h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a.cuda(), None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    assert h.hif4_gemm_workspace_bytes_decoded_w(h.HIF4_A_BF16_KEEP, M, N, K) == M * K * 2
    ck = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a.cuda(), None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    rng = np.random.default_rng(M)
    rows = np.sort(np.concatenate([rng.choice(M, 62, replace=False), [0, M - 1]]))
    cols = np.sort(np.concatenate([rng.choice(N, 126, replace=False), [0, N - 1]]))
    wdec = oracle.dequantize(wc[cols], wm[cols])
    ac, am = oracle.quantize(synth.bits(a)[rows])
    pick = lambda t: t[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.float64)
    want = oracle.gemm_f64(oracle.dequantize(ac, am), wdec)
    assert rel_fro(pick(c), want) <= TOL, rel_fro(pick(c), want)
    want_k = oracle.gemm_f64(synth.bits(a)[rows], wdec)
    assert rel_fro(pick(ck), want_k) <= TOL, rel_fro(pick(ck), want_k)


def test_gemm_random_shapes_every_kind_and_workspace(h, oracle):
    """A seeded sweep over shapes that straddle every row-count boundary of the dispatch (16, 32, 64, 128, 192, 256
    rows and beyond), ragged N, K of 1 to 24 units, all three kinds of A, both output types, the smallest, the
    default and no workspace, strided A and C: each result against the fp64 oracle."""
    rng = np.random.default_rng(20260711)
    edges = [1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 300, 400]
    for case in range(48):
        M = int(rng.choice(edges)) if case % 2 == 0 else int(rng.integers(1, 420))
        N = int(rng.integers(1, 700))
        K = 64 * int(rng.integers(1, 25))
        kind = (h.HIF4_A_HIF4, h.HIF4_A_BF16_QUANTIZE, h.HIF4_A_BF16_KEEP)[case % 3]
        f32 = bool(rng.integers(0, 2))
        ws_mode = int(rng.integers(0, 3))  # 0: default (the optional larger one), 1: the smallest that is legal, 2: none where legal
        print(f"case {case}: M={M} N={N} K={K} kind={kind} f32={f32} ws={ws_mode}", flush=True)
        ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 7000 + case)
        wcd, wmd = dev_packed(wc, wm)
        wdec = oracle.dequantize(wc, wm)
        pad = int(rng.integers(0, 2)) * 64
        if kind == h.HIF4_A_HIF4:
            a_dev, am_dev = dev_packed(ac, am)
            want = oracle.gemm_f64(oracle.dequantize(ac, am), wdec)
        else:
            abuf = torch.zeros((M, K + pad), dtype=torch.bfloat16, device="cuda")
            abuf[:, :K] = synth.from_bits(ab).cuda()
            a_dev, am_dev = abuf[:, :K], None
            want = oracle.gemm_f64(oracle.dequantize(ac, am) if kind == h.HIF4_A_BF16_QUANTIZE else ab, wdec)
        need = h.hif4_gemm_workspace_bytes(kind, M, K)
        ws = None
        if ws_mode == 1 or (ws_mode == 2 and need):
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        elif ws_mode == 2:
            ws = torch.empty(16, dtype=torch.uint8, device="cuda")[:0]
        dt = torch.float32 if f32 else torch.bfloat16
        cbuf = torch.full((M, N + 3), -7.0, dtype=dt, device="cuda")
        h.hif4_gemm(kind, a_dev, am_dev, wcd, wmd, out_dtype=h.HIF4_OUT_F32 if f32 else h.HIF4_OUT_BF16, c=cbuf[:, :N], workspace=ws)
        torch.cuda.synchronize()
        assert (cbuf[:, N:] == -7.0).all(), "columns beyond N untouched"
        got = cbuf[:, :N].double().cpu().numpy()
        if f32:
            assert rel_fro(got, want) <= TOL, (case, rel_fro(got, want))
        else:
            wb = synth.bits(torch.from_numpy(want).to(torch.bfloat16)).astype(np.int32)
            gb = synth.bits(cbuf[:, :N].contiguous().cpu()).astype(np.int32)
            key = lambda b: np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
            assert np.abs(key(gb) - key(wb)).max() <= 1, case


def test_gemm_weight_only_few_rows_optional_workspace(h, oracle):
    """65 to 192 rows, BF16 activations: with the optional workspace (the binding's default) the call runs the
    column-per-wave kernel on a reordered copy of A, without it the tile kernel; both against the oracle."""
    M, N, K = 130, 520, 448
    ab, _, (wc, wm) = quantized_operands(oracle, M, N, K, 9001)
    want = oracle.gemm_f64(ab, oracle.dequantize(wc, wm))
    a = synth.from_bits(ab).cuda()
    wcd, wmd = dev_packed(wc, wm)
    assert h.hif4_gemm_workspace_bytes_decoded_w(h.HIF4_A_BF16_KEEP, M, N, K) == M * K * 2
    assert h.hif4_gemm_workspace_bytes(h.HIF4_A_BF16_KEEP, M, K) == 0
    c_ws = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
    c_no = h.hif4_gemm(h.HIF4_A_BF16_KEEP, a, None, wcd, wmd, out_dtype=h.HIF4_OUT_F32,
                       workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert rel_fro(c_ws.cpu().numpy().astype(np.float64), want) <= TOL
    assert rel_fro(c_no.cpu().numpy().astype(np.float64), want) <= TOL


# ---- the kernel for at most 32 rows against at least 6144 columns: unit scales applied to the units' partial sums,
# weights expanded through the FP8 byte table.  Ragged column edges, one, odd and uneven numbers of pairs of units per
# K part, all three kinds of A, and every (column strips, K parts, column groups) shape of workgroup the launcher has,
# for both tile heights.

FEWROW_SHAPES = [(5, 6144, 256), (16, 6150, 1280), (16, 8200, 4096), (11, 11008, 2304), (9, 8200, 256), (16, 14353, 768),
                 (13, 16400, 2304), (16, 28673, 768), (1, 7000, 512), (3, 28672, 1792),
                 (17, 6144, 256), (32, 8200, 4096), (20, 8200, 256), (32, 28700, 512), (24, 16400, 256), (32, 28672, 1792)]


def fewrows_workgroup_shape(M, N, K):
    """The launcher's choice of workgroup shape (fewrows_choose in csrc/hif4_gemm_fewrows.hip), restated: used only to
    check that FEWROW_SHAPES reaches every compiled shape."""
    RM, pairs = (16 if M <= 16 else 32), (K // 64 + 1) // 2
    best, best_t = None, float("inf")
    for nwc, ks, cg in ((7, 2, 1), (3, 4, 1), (2, 4, 1), (4, 2, 1), (4, 2, 2)):
        nw = nwc * ks
        slot, meta = ks * 16 * RM * 16 + nw * cg * 1024, nw * 2 * cg * 1024
        half = nw == 4 and 3 * slot + meta <= 80 * 1024
        if ((80 if half else 160) * 1024 - meta) // slot < 3:
            continue
        per_cu = 2 if half else 1
        strips = -(-N // (16 * cg))
        wgs = -(-strips // nwc)
        rounds, steps = -(-wgs // (256 * per_cu)), -(-pairs // ks)
        t = rounds * (1 + 0.05 * (rounds - 1)) * per_cu * nw / 4 * cg * (steps + 8)
        if t < best_t:
            best, best_t = (RM, nwc, ks, cg), t
    return best


def test_few_row_shapes_cover_every_workgroup_shape():
    seen = {fewrows_workgroup_shape(*s) for s in FEWROW_SHAPES}
    assert seen == {(rm, *c) for rm in (16, 32) for c in ((7, 2, 1), (3, 4, 1), (2, 4, 1), (4, 2, 1), (4, 2, 2))}, seen


@pytest.mark.parametrize("M,N,K", FEWROW_SHAPES)
def test_gemm_few_rows_wide_weights(h, oracle, M, N, K):
    print(f"few-row gemm parity M={M} N={N} K={K}", flush=True)
    ab, (ac, am), (wc, wm) = quantized_operands(oracle, M, N, K, 900 + M + N + K)
    wdec = oracle.dequantize(wc, wm)
    wcd, wmd = dev_packed(wc, wm)
    key = lambda b: np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    for a_kind in (h.HIF4_A_BF16_KEEP, h.HIF4_A_HIF4, h.HIF4_A_BF16_QUANTIZE):
        a_bits = ab if a_kind == h.HIF4_A_BF16_KEEP else oracle.dequantize(ac, am)
        want = oracle.gemm_f64(a_bits, wdec)
        if a_kind == h.HIF4_A_HIF4:
            a_dev, a_meta = dev_packed(ac, am)
        else:
            a_dev, a_meta = synth.from_bits(ab).cuda(), None
        c32 = h.hif4_gemm(a_kind, a_dev, a_meta, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
        c16 = h.hif4_gemm(a_kind, a_dev, a_meta, wcd, wmd, out_dtype=h.HIF4_OUT_BF16)
        c32b = h.hif4_gemm(a_kind, a_dev, a_meta, wcd, wmd, out_dtype=h.HIF4_OUT_F32)
        torch.cuda.synchronize()
        got = c32.cpu().numpy().astype(np.float64)
        assert rel_fro(got, want) <= TOL, (a_kind, rel_fro(got, want))
        assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max() + 1e-30
        assert torch.equal(c32, c32b), "same launch twice gives the same bits"
        # BF16 output: within one BF16 ulp of the rounded oracle value, except where the sum cancels to (nearly) nothing:
        # there the fp32 accumulation error, bounded by 1e-5 of the largest result as checked above, exceeds the ulp
        gb = synth.bits(c16.cpu()).astype(np.int32)
        wb = synth.bits(torch.from_numpy(want).to(torch.bfloat16)).astype(np.int32)
        g16 = c16.float().cpu().numpy().astype(np.float64)
        close = (np.abs(key(gb) - key(wb)) <= 1) | (np.abs(g16 - want) <= 1e-5 * np.abs(want).max())
        assert close.all(), (a_kind, int((~close).sum()))
        assert (np.abs(key(gb) - key(wb)) <= 1).mean() > 0.9999


def test_gemm_few_rows_every_metadata_pattern_and_nan(h, oracle):
    """Packed weights drawn directly: every micro-exponent pattern, scales many binades apart, zero codes of both signs,
    a NaN unit; strided A and C."""
    rng = np.random.default_rng(55)
    M, N, K = 11, 14400, 512
    wc = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    wc[rng.random((N, K // 2)) < 0.1] &= 0x88            # zero magnitudes, signs kept
    wm = (rng.integers(0, 2 ** 24, (N, K // 64)).astype(np.uint32) << 8) | rng.integers(100, 220, (N, K // 64)).astype(np.uint32)
    wm[7, 2] |= 0xFF
    wm[14399, 7] |= 0xFF
    a = rng.standard_normal((M, K)) * np.exp(rng.uniform(-4, 4, (M, 1)))
    ab = synth.bits(torch.from_numpy(a).to(torch.bfloat16))
    want = oracle.gemm_f64(ab, oracle.dequantize(wc, wm))
    abuf = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    abuf[:, :K] = synth.from_bits(ab).cuda()
    cbuf = torch.full((M, N + 3), -1.0, dtype=torch.float32, device="cuda")
    h.hif4_gemm(h.HIF4_A_BF16_KEEP, abuf[:, :K], None, *dev_packed(wc, wm), out_dtype=h.HIF4_OUT_F32, c=cbuf[:, :N])
    torch.cuda.synchronize()
    got = cbuf[:, :N].cpu().numpy().astype(np.float64)
    assert (cbuf[:, N:] == -1.0).all()
    nan_want = np.isnan(want)
    assert nan_want[:, 7].all() and nan_want[:, 14399].all() and nan_want.sum() == 2 * M
    assert (np.isnan(got) == nan_want).all()
    ok = ~nan_want
    for r in range(M):   # each row against its own norm: rows and columns differ by many binades
        assert np.linalg.norm(got[r][ok[r]] - want[r][ok[r]]) <= TOL * np.linalg.norm(want[r][ok[r]])
    # column by column too (the unit scales are per column): a sample of columns
    for col in rng.integers(0, N, 400):
        if ok[:, col].all():
            assert np.linalg.norm(got[:, col] - want[:, col]) <= TOL * np.linalg.norm(want[:, col]) + 1e-30
