"""hif4_gemm_noalloc (the entry point for callers that cannot allocate) against hif4_gemm given a workspace
of exactly hif4_gemm_workspace_bytes() bytes: the same kernels run, so the results must be equal bit for bit.
Two calls in a row on the library's one static scratch, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2602_11287_amd import hif4 as h, synth

pytestmark = pytest.mark.gpu


def _operands(M, N, K, seed):
    g = torch.Generator().manual_seed(seed)
    a = torch.randn((M, K), generator=g).to(torch.bfloat16).cuda()
    w = (torch.randn((N, K), generator=g) * 0.02).to(torch.bfloat16).cuda()
    wc, wm = h.hif4_quantize(w)
    return a, wc, wm


@pytest.mark.parametrize("a_kind", [h.HIF4_A_BF16_QUANTIZE, h.HIF4_A_HIF4, h.HIF4_A_BF16_KEEP])
@pytest.mark.parametrize("out_dtype", [h.HIF4_OUT_BF16, h.HIF4_OUT_F32])
def test_noalloc_equals_gemm_with_exact_workspace_twice(a_kind, out_dtype):
    h.load()
    for (M, N, K), seed in (((300, 520, 1024), 5), ((48, 200, 256), 6)):   # the second call is the smaller one
        a, wc, wm = _operands(M, N, K, seed)
        a_meta = None
        if a_kind == h.HIF4_A_HIF4:
            a, a_meta = h.hif4_quantize(a)
        need = h.hif4_gemm_workspace_bytes(a_kind, M, K)
        assert need <= h.hif4_gemm_noalloc_max_bytes()
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")   # exactly the mandatory size (none for BF16 activations)
        want = h.hif4_gemm(a_kind, a, a_meta, wc, wm, out_dtype=out_dtype, workspace=ws)
        dt = torch.bfloat16 if out_dtype == h.HIF4_OUT_BF16 else torch.float32
        got = torch.full((M, N), float("nan"), dtype=dt, device="cuda")
        before = torch.cuda.memory_allocated()
        h.hif4_gemm_noalloc(a_kind, a, a_meta, wc, wm, out_dtype=out_dtype, c=got)
        assert torch.cuda.memory_allocated() == before, "the call allocated nothing through torch"
        torch.cuda.synchronize()
        assert torch.equal(got, want)


def test_noalloc_against_the_oracle_and_limits(oracle):
    """Through the C ABI against the fp64 oracle on the same decoded operands, and the size limit."""
    h.load()
    M, N, K = 70, 96, 512
    x = synth.activation_with_outliers(rows=M, K=K)
    w = synth.weight_gaussian(N, K, 0.02, config=3)
    ac, am = oracle.quantize(synth.bits(x))
    wc, wm = oracle.quantize(synth.bits(w))
    want = oracle.gemm_f64(oracle.dequantize(ac, am), oracle.dequantize(wc, wm))
    c = h.hif4_gemm_noalloc(h.HIF4_A_BF16_QUANTIZE, x.cuda(), None, torch.from_numpy(wc).cuda(),
                            torch.from_numpy(wm.view(np.int32)).cuda(), out_dtype=h.HIF4_OUT_F32)
    torch.cuda.synchronize()
    rel = np.linalg.norm(c.cpu().numpy().astype(np.float64) - want) / np.linalg.norm(want)
    assert rel <= 1e-4, rel
    # beyond the static scratch: refused with its own status, nothing enqueued (raw C ABI, no tensors that large)
    lib = h.load()
    big_m = h.hif4_gemm_noalloc_max_bytes() // (2 * K) + 1
    p = c.data_ptr()
    assert lib.hif4_gemm_noalloc(h.HIF4_A_HIF4, p, p, K, p, p, big_m, N, K, p, N, h.HIF4_OUT_F32, None) == h.HIF4_ERR_SCRATCH
    assert lib.hif4_gemm_noalloc(h.HIF4_A_HIF4, p, p, K, p, p, big_m - 1, N, 100, p, N, h.HIF4_OUT_F32, None) == h.HIF4_ERR_SHAPE
    assert b"scratch" in lib.hif4_status_string(h.HIF4_ERR_SCRATCH)
