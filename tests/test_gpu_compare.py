"""GPU comparison tools (include/hif4_compare.h) against the numpy comparators of the oracle side:
dequantised values equal value by value (both sides do the same fp64 steps), squared-error sums to
fp64 summation accuracy, and the MSE ratios of Section III-A of the paper on the GPU."""
import numpy as np
import pytest
import torch

from paper_2602_11287_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    from paper_2602_11287_amd import hif4
    hif4.load()
    assert torch.cuda.is_available()
    return hif4


def matrix(rows, K, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, K)) * np.exp(rng.uniform(-6, 6, (rows, 1)))
    x[rng.random((rows, K)) < 0.003] *= 50.0
    x[0, :32] = 0.0                                   # an all-zero group
    x[1 % rows, :16] = 2.0 ** -130                    # BF16 subnormals
    return synth.to_bf16(x)


@pytest.mark.parametrize("rows,K", [(1, 32), (7, 96), (130, 1056), (64, 4096)])
def test_mxfp4_and_nvfp4_values(h, oracle, rows, K):
    from oracle import bfp4_comparators as cmp
    print(f"comparators rows={rows} K={K}", flush=True)
    xb = matrix(rows, K, 40 + rows)
    xf = oracle.bf16_bits_to_f64(synth.bits(xb))
    xd = xb.cuda()
    y = torch.empty((rows, K), dtype=torch.float64, device="cuda")
    err = torch.zeros(1, dtype=torch.float64, device="cuda")
    h.hif4cmp_mxfp4_fake_quant(xd, y, err)
    want = cmp.mxfp4_fake_quant(xf)
    assert (y.cpu().numpy() == want).all()
    assert abs(err.item() - np.sum((xf - want) ** 2)) <= 1e-12 * np.sum((xf - want) ** 2) + 1e-300
    # NVFP4, direct cast
    err.zero_()
    h.hif4cmp_nvfp4_fake_quant(xd, None, y, err)
    want = cmp.nvfp4_fake_quant(xf)
    assert (y.cpu().numpy() == want).all()
    assert abs(err.item() - np.sum((xf - want) ** 2)) <= 1e-12 * np.sum((xf - want) ** 2) + 1e-300
    # NVFP4 with per-tensor scaling
    peak = torch.zeros(1, dtype=torch.int32, device="cuda")
    h.hif4cmp_abs_max(xd, peak)
    assert oracle.bf16_bits_to_f64(np.array([[peak.item()]], np.uint16))[0, 0] == np.abs(xf).max()
    h.hif4cmp_nvfp4_fake_quant(xd, peak, y, None)
    want = cmp.nvfp4_fake_quant(xf, pts=True)
    assert (y.cpu().numpy() == want).all()


def test_sq_err_and_strided_rows(h, oracle):
    rows, K = 77, 256
    xb, yb = matrix(rows, K, 1), matrix(rows, K, 2)
    big = torch.zeros((rows, K + 64), dtype=torch.bfloat16, device="cuda")
    big[:, :K] = xb.cuda()
    err = torch.zeros(1, dtype=torch.float64, device="cuda")
    h.hif4cmp_sq_err_bf16(big[:, :K], yb.cuda(), err)
    xf, yf = oracle.bf16_bits_to_f64(synth.bits(xb)), oracle.bf16_bits_to_f64(synth.bits(yb))
    want = np.sum((xf - yf) ** 2)
    assert abs(err.item() - want) <= 1e-12 * want
    # a second call adds to the sum
    h.hif4cmp_sq_err_bf16(big[:, :K], yb.cuda(), err)
    assert abs(err.item() - 2 * want) <= 1e-12 * want


@pytest.mark.parametrize("x", [0, 9, 17])
def test_mse_ratios_of_section_3a_on_gpu(h, x):
    """HiF4 : NVFP4 (per-tensor scaled) : MXFP4 = 1 : 1.32 : 1.89 (Section III-A), all three on the GPU."""
    xb = synth.to_bf16(synth.gaussian_sweep(x)).cuda()
    err = torch.zeros(3, dtype=torch.float64, device="cuda")
    codes, meta = h.hif4_quantize(xb)
    h.hif4cmp_sq_err_bf16(xb, h.hif4_dequantize(codes, meta), err[0:1])
    peak = torch.zeros(1, dtype=torch.int32, device="cuda")
    h.hif4cmp_abs_max(xb, peak)
    h.hif4cmp_nvfp4_fake_quant(xb, peak, None, err[1:2])
    h.hif4cmp_mxfp4_fake_quant(xb, None, err[2:3])
    e = err.cpu().numpy()
    assert abs(e[1] / e[0] - 1.32) < 0.03, e[1] / e[0]
    assert abs(e[2] / e[0] - 1.89) < 0.03, e[2] / e[0]


E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def unpack_mxfp4(cells, scales):
    """Packed operand of hif4ref_mxfp4_pack -> fp64 [rows, K] by the layout the header documents."""
    cells, scales = cells.cpu().numpy(), scales.cpu().numpy()
    G, rows, _ = cells.shape
    nib = np.empty((G, rows, 32), np.uint8)
    nib[:, :, 0::2] = cells & 0xF
    nib[:, :, 1::2] = cells >> 4
    val = E2M1[nib & 7] * np.where(nib & 8, -1.0, 1.0)
    out = np.empty((rows, G * 32))
    for g in range(G):
        ks, j = divmod(g, 8)
        byte = scales[ks * 2 + j % 2, :, j // 2].astype(np.int64)
        out[:, 32 * g:32 * g + 32] = val[g] * (2.0 ** (byte - 127))[:, None]
    return out


@pytest.mark.parametrize("M,N,K", [(1, 1, 256), (300, 200, 512), (257, 513, 768), (1024, 256, 1024)])
def test_mxfp4_reference_gemm(h, oracle, M, N, K):
    """The speed reference is a correct MXFP4 GEMM: its packer gives the comparator's values, and the
    product equals the fp64 product of those values to fp32 accumulation accuracy."""
    from oracle import bfp4_comparators as cmp
    print(f"mxfp4 reference M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M + N + K)
    a = synth.to_bf16(rng.standard_normal((M, K)) * np.exp(rng.uniform(-2, 2, (M, 1))))
    w = synth.to_bf16(rng.standard_normal((N, K)) * 0.02)
    a[0, :32] = 0.0
    ac, asc = h.hif4ref_mxfp4_pack(a.cuda())
    wc, wsc = h.hif4ref_mxfp4_pack(w.cuda())
    af, wf = unpack_mxfp4(ac, asc), unpack_mxfp4(wc, wsc)
    assert (af == cmp.mxfp4_fake_quant(oracle.bf16_bits_to_f64(synth.bits(a)))).all()
    assert (wf == cmp.mxfp4_fake_quant(oracle.bf16_bits_to_f64(synth.bits(w)))).all()
    c = h.hif4ref_mxfp4_gemm(ac, asc, wc, wsc, out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    want = af @ wf.T
    got = c.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    assert rel <= 1e-5, rel


def test_mfma_only_loops_run(h):
    """The MFMA-only loops of the benchmark: every kind launches, finishes and reports its flop count."""
    scratch = torch.empty(131072, dtype=torch.float32, device="cuda")
    assert h.hif4ref_mfma_loop(0, 4, scratch) == 2048 * 4 * 8 * 32768
    assert h.hif4ref_mfma_loop(2, 4, scratch) == 2048 * 4 * 8 * 32768
    assert h.hif4ref_mfma_loop(1, 4, scratch) == 2048 * 4 * 8 * 131072
    torch.cuda.synchronize()
    for kind in (0, 1, 2):          # out[0]: the shader clock of the launch in MHz (nominal 2400, lower under load)
        h.hif4ref_mfma_loop(kind, 256, scratch)
        mhz = float(scratch[0])
        assert 300.0 < mhz < 3000.0, (kind, mhz)
