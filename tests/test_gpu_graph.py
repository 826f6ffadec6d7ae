"""The library calls only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a sequence of them can be captured in a HIP graph.  Replays, with eager work
in between, must reproduce the eager results bit for bit."""
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


def test_graph_capture_and_replay(h):
    M, N, K = 300, 512, 1024
    g = torch.Generator(device="cuda").manual_seed(9)
    a = torch.randn((M, K), generator=g, device="cuda").to(torch.bfloat16)
    w = (torch.randn((N, K), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
    a16 = torch.randn((16, K), generator=g, device="cuda").to(torch.bfloat16)
    wc, wm = h.hif4_quantize(w)
    # every buffer the captured calls touch exists before the capture
    ac = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    am = torch.empty((M, K // 64), dtype=torch.int32, device="cuda")
    y = torch.empty_like(a)
    c = torch.empty((M, N), dtype=torch.float32, device="cuda")
    c0 = torch.empty((M, N), dtype=torch.float32, device="cuda")       # K == 0 fill kernel
    cs = torch.empty((16, N), dtype=torch.bfloat16, device="cuda")
    oc = torch.empty((M, N // 2), dtype=torch.uint8, device="cuda")
    om = torch.empty((M, N // 64), dtype=torch.int32, device="cuda")
    ws = torch.empty(h.hif4_gemm_workspace_bytes(h.HIF4_A_BF16_QUANTIZE, M, K), dtype=torch.uint8, device="cuda")
    # few rows: HiF4 activations through the K-split kernel of the decode shape (16 rows), the few-row kernel with
    # K split over wave groups (100 rows), BF16 activations on it (its optional workspace), and a grouped call
    c16q = torch.empty((16, N), dtype=torch.float32, device="cuda")
    c100 = torch.empty((100, N), dtype=torch.float32, device="cuda")
    c100k = torch.empty((100, N), dtype=torch.bfloat16, device="cuda")
    wsk = torch.empty(100 * K * 2, dtype=torch.uint8, device="cuda")
    cg = torch.empty((M, N // 2), dtype=torch.float32, device="cuda")
    offs = torch.tensor([0, 130, 300], dtype=torch.int32, device="cuda")
    wgc, wgm = wc.view(2, N // 2, K // 2), wm.view(2, N // 2, K // 64)  # two experts of N / 2 columns each

    def sequence():
        h.hif4_quantize(a, ac, am)
        h.hif4_dequantize(ac, am, y)
        h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, out_dtype=h.HIF4_OUT_F32, c=c, workspace=ws)
        h.hif4_gemm(h.HIF4_A_BF16_KEEP, a16, None, wc, wm, out_dtype=h.HIF4_OUT_BF16, c=cs)
        h.hif4_gemm_to_hif4(h.HIF4_A_HIF4, ac, am, wc, wm, c_codes=oc, c_meta=om, workspace=ws)
        h.hif4_gemm(h.HIF4_A_HIF4, ac[:, :0], am[:, :0], wc[:, :0], wm[:, :0], out_dtype=h.HIF4_OUT_F32, c=c0)
        h.hif4_gemm(h.HIF4_A_BF16_QUANTIZE, a16, None, wc, wm, out_dtype=h.HIF4_OUT_F32, c=c16q, workspace=ws)
        h.hif4_gemm(h.HIF4_A_HIF4, ac[:100], am[:100], wc, wm, out_dtype=h.HIF4_OUT_F32, c=c100, workspace=ws)
        h.hif4_gemm(h.HIF4_A_BF16_KEEP, a[:100], None, wc, wm, out_dtype=h.HIF4_OUT_BF16, c=c100k, workspace=wsk)
        h.hif4_grouped_gemm(h.HIF4_A_BF16_QUANTIZE, a, None, wgc, wgm, offs, out_dtype=h.HIF4_OUT_F32, c=cg, workspace=ws)

    outs = (ac, am, y, c, cs, oc, om, c0, c16q, c100, c100k, cg)
    sequence()                                   # eager reference (also the first-use setup of every kernel)
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        sequence()                               # warm-up on the capture stream
        torch.cuda.current_stream().synchronize()
        with torch.cuda.graph(graph, stream=side):
            sequence()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        for o in outs:
            o.zero_() if o.dtype != torch.float32 else o.fill_(float(rep))   # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, wv in zip(outs, want):
            assert torch.equal(o, wv), f"replay {rep} differs from the eager result"
