"""GEMM legs of bench.py: the HiF4 GEMM configurations on seeded synthetic tensors with the
shapes of LLM linear layers.  Big operands are drawn on the device (same distributions as
the CPU generators in synth.py) to keep the benchmark short; parity on these shapes is
covered by tests/test_gpu_gemm.py."""
import numpy as np
import torch


# HBM bytes per launch of the GEMM kernel itself (pre-passes not included), from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE in KiB per dispatch (FETCH_SIZE x 1.99988, WRITE_SIZE x 1.0, the factors of a plain device copy):
# profiles/gemm_kernels_configs2-5.md, profiles/gemm_fewrows_skinny_colwave_decode_and_grouped.md,
# profiles/gemm_planes16_column_split_prefill_4096x11008x4096.md
def _kib(fetch, write):
    return int((fetch * 1.99988 + write) * 1024)


_TRAFFIC = {
    "gemm_weight_only_M16_N4096_K4096": _kib(5151.5, 128.0),
    "gemm_weight_only_M16_N28672_K8192": _kib(78072.5, 896.0),
    "gemm_w4a4_quantize_inside_M4096_N11008_K4096": _kib(196736.0 + 84068.7, 65598.1 + 22528.8),  # the two launches of the call
    "gemm_w4a4_prepacked_M4096_N11008_K4096": _kib(196736.0 + 84068.7, 65598.1 + 22528.8),
    "gemm_w4a4_quantize_inside_small_workspace_M4096_N11008_K4096": _kib(147985.0, 89805.7),
    "grouped_gemm_w4a4_E64_rows8192_N2048_K7168": _kib(370768.1, 32768.0),
    "gemm_w4a4_quantize_inside_M16384_N28672_K8192": _kib(5505218.2, 918472.8),
    "gemm_w4a4_quantize_inside_small_workspace_M16384_N28672_K8192": _kib(2867346.8, 930189.2),
    "gemm_w4a4_to_hif4_M16384_N28672_K8192": _kib(5512239.6, 258048.0),
}


def _timed(fn, n):
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n


SETTLE_MS = 60.0


def _settle(fn, min_ms=SETTLE_MS):
    """Runs fn back to back, untimed, for at least min_ms of GPU time.  After a stretch without matrix work (the set-up
    of a leg: random draws, quantisation, allocation) the chip's power management raises the clock over some tens of
    milliseconds: measured on the prefill GEMM, 376 us per call in the first 10 calls after 2 s of idling, 302 us from
    the 120th call on; on the grouped GEMM 409 against 353.  The encoder/decoder pair, bound by memory, moves 2 % in its
    first five calls.  A leg of 20 calls of 0.3 ms would be timed inside that ramp, so every GEMM leg (the vendor and
    MXFP4 references and the MFMA-only loops alike) first runs until the clock has settled."""
    n, spent = 1, 0.0
    while spent < min_ms:
        spent += _timed(fn, n) * n
        n = min(64, 2 * n)


def _randn_bf16(shape, sigma, gen, dev, chunk_rows=8192):
    out = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    for r in range(0, shape[0], chunk_rows):
        n = min(chunk_rows, shape[0] - r)
        out[r:r + n] = (torch.randn((n, shape[1]), generator=gen, device=dev) * sigma).to(torch.bfloat16)
    return out


def _quantize_rows(hif4, w, chunk_rows=16384):
    codes = torch.empty((w.shape[0], w.shape[1] // 2), dtype=torch.uint8, device=w.device)
    meta = torch.empty((w.shape[0], w.shape[1] // 64), dtype=torch.int32, device=w.device)
    for r in range(0, w.shape[0], chunk_rows):
        hif4.hif4_quantize(w[r:r + chunk_rows], codes[r:r + chunk_rows], meta[r:r + chunk_rows])
    return codes, meta


def run(hif4, synth, dev, steps, warmup, mfma_peak_tflops, hbm_peak_gbps, large=True, only=None):
    """only: None for every leg, else a set of section names (ceiling, decode, decode_large, prefill, grouped, large)."""
    legs = {}

    def plan(a_kind, M, N, K, experts=0, ws=None, emit=False):
        """Name of the main loop the library dispatches this call to (its own host query, not a guess)."""
        return hif4.hif4_gemm_plan_name(hif4.hif4_gemm_plan(a_kind, M, N, K, experts=experts, result_as_hif4=emit, workspace_bytes=ws))
    gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 99)
    steps = max(2, min(steps, 10))

    legs["gemm_legs_untimed_settling_ms"] = SETTLE_MS   # see _settle: each GEMM leg runs that long before its timed calls
    want = (lambda s: True) if only is None else (lambda s: s in only)
    state = {"bf16_ceiling": None, "fp4_ceiling": None}

    def sec_ceiling():
        # ---- what the matrix pipeline sustains by itself on operands with random bits (power-limited clock):
        # the ceiling next to which the GEMM rates below are read; the nominal peak stays the roofline's `peak`
        scratch = torch.empty(131072, dtype=torch.float32, device=dev)
        ceiling, clock = {}, {}
        for kind, name in ((0, "bf16_32x32x16"), (2, "bf16_16x16x32"), (1, "fp4_scaled_32x32x64")):
            flop = hif4.hif4ref_mfma_loop(kind, 512, scratch)
            _settle(lambda: hif4.hif4ref_mfma_loop(kind, 512, scratch))
            ms = _timed(lambda: hif4.hif4ref_mfma_loop(kind, 512, scratch), 50)
            ceiling[name] = round(flop / ms / 1e9, 1)
            clock[name] = round(float(scratch[0]))   # shader clock of the last launch (its first wave), MHz
        legs["mfma_only_loop_random_operands_TFLOPs"] = ceiling
        legs["mfma_only_loop_shader_clock_MHz"] = dict(clock, nominal=2400)
        state["bf16_ceiling"] = max(ceiling["bf16_32x32x16"], ceiling["bf16_16x16x32"])  # the 16 x 16 x 32 form sustains more
        state["fp4_ceiling"] = ceiling["fp4_scaled_32x32x64"]


    # ---- weight-only decode shape: M=16, N=4096, K=4096 (HBM-bound weight streaming).  One matrix of packed
    # weights is 9.4 MB and stays in the caches when it is multiplied again and again, so the HBM figure comes from
    # 64 distinct weight matrices (604 MB, more than the 256 MB last-level cache) used in turn, from a HIP graph so
    # that the GPU and not the host sets the pace; the single-matrix figure is kept and labelled cache-resident.
    def graph_us(calls, replays):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            calls[0]()
            torch.cuda.current_stream().synchronize()
            with torch.cuda.graph(graph, stream=side):
                for f in calls:
                    f()
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()
        _settle(graph.replay)
        ms = _timed(graph.replay, replays) / len(calls)
        del graph
        return ms * 1e3

    def decode_leg(name, M, N, K, copies, sigma, kernel, channel_scale):
        # the small shape takes the seeded CPU tensor the tests use; the large one is drawn on the device
        w = synth.weight_gaussian(N, K, sigma, config=2, channel_scale=channel_scale).to(dev) if N * K <= (1 << 25) else _randn_bf16((N, K), sigma, gen, dev)
        a = synth.activation_gaussian(M, K, config=2).to(dev)
        wcs = torch.empty((copies, N, K // 2), dtype=torch.uint8, device=dev)
        wms = torch.empty((copies, N, K // 64), dtype=torch.int32, device=dev)
        hif4.hif4_quantize(w, wcs[0], wms[0])
        for i in range(1, copies):      # other copies: same recipe, device-side draws
            hif4.hif4_quantize(_randn_bf16((N, K), sigma, gen, dev), wcs[i], wms[i])
        c = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        mk = lambda i: (lambda: hif4.hif4_gemm(hif4.HIF4_A_BF16_KEEP, a, None, wcs[i], wms[i], out_dtype=hif4.HIF4_OUT_BF16, c=c))
        for _ in range(warmup):
            mk(0)()
        ms_host = _timed(mk(0), steps * 10)  # one Python call per launch: paced by the host, not by the GPU
        us_hbm = graph_us([mk(i) for i in range(copies)], max(steps, 5))
        us_cache = graph_us([mk(0)] * 50, max(steps, 5))
        nbytes = N * K // 64 * 36 + M * K * 2 + M * N * 2
        legs[name] = {
            "us": round(us_hbm, 2), "us_one_matrix_cache_resident": round(us_cache, 2), "us_per_python_call": round(ms_host * 1e3, 2),
            "distinct_weight_matrices": copies, "GBps": round(nbytes / us_hbm / 1e3, 1), "GFLOP": round(2 * M * N * K / 1e9, 3),
            "roofline": {"bound": "hbm", "kernel": kernel, "achieved": round(nbytes / us_hbm / 1e3, 1),
                         "peak": hbm_peak_gbps, "unit": "GB/s", "frac": round(nbytes / us_hbm / 1e3 / hbm_peak_gbps, 4),
                         "algorithmic_bytes": nbytes, "traffic": _TRAFFIC.get(name), "traffic_source": "profiles/ (not measured in this run)"}}
        return w, wcs[0], wms[0]

    def sec_decode():
        w, wc, wm = decode_leg("gemm_weight_only_M16_N4096_K4096", 16, 4096, 4096, 64, 0.02, plan(hif4.HIF4_A_BF16_KEEP, 16, 4096, 4096, ws=0), True)
        M, N, K = 16, 4096, 4096
        # the same weights against more rows (W4A4, activations quantised inside the call): the few-row kernel with K
        # split over wave groups, then several m-tiles of it, then the tile kernel; the vendor BF16 GEMM on the same
        # shape beside each
        sweep = {}
        for Ms in (32, 128, 512, 1024, 2048):
            a_s = _randn_bf16((Ms, K), 1.0, gen, dev)
            c_s = torch.empty((Ms, N), dtype=torch.bfloat16, device=dev)
            ws_s = torch.empty(max(16, hif4.hif4_gemm_workspace_bytes(hif4.HIF4_A_BF16_QUANTIZE, Ms, K)), dtype=torch.uint8, device=dev)
            fs = lambda: hif4.hif4_gemm(hif4.HIF4_A_BF16_QUANTIZE, a_s, None, wc, wm, out_dtype=hif4.HIF4_OUT_BF16, c=c_s, workspace=ws_s)
            fv = lambda: torch.matmul(a_s, w.t(), out=c_s)
            _settle(fs, SETTLE_MS / 2)
            us = _timed(fs, max(steps, 10)) * 1e3
            _settle(fv, SETTLE_MS / 2)
            us_v = _timed(fv, max(steps, 10)) * 1e3
            sweep[f"M{Ms}"] = {"us": round(us, 1), "TFLOPs": round(2.0 * Ms * N * K / us / 1e6, 1), "vendor_bf16_us": round(us_v, 1)}
            del a_s, c_s, ws_s
        legs["gemm_w4a4_quantize_inside_rows_sweep_N4096_K4096"] = sweep
        del w, wc, wm

    def sec_decode_large():
        # the decode shape of a 70B-class MLP: 16 rows against 28672 x 8192 weights (132 MB packed), 4 distinct matrices in turn
        if large:
            tmp = decode_leg("gemm_weight_only_M16_N28672_K8192", 16, 28672, 8192, 4, 0.015, plan(hif4.HIF4_A_BF16_KEEP, 16, 28672, 8192, ws=0), False)
            del tmp
            torch.cuda.empty_cache()


    def mfma_leg(name, M, N, K, fn, kernel):
        for _ in range(max(1, min(warmup, 2))):
            fn()
        _settle(fn)
        ms = _timed(fn, steps)
        tf = 2.0 * M * N * K / ms / 1e9
        legs[name] = {"ms": round(ms, 4), "TFLOPs": round(tf, 1),
                      "roofline": {"bound": "mfma", "kernel": kernel, "achieved": round(tf, 1), "peak": mfma_peak_tflops,
                                   "unit": "TFLOP/s", "frac": round(tf / mfma_peak_tflops, 4),
                                   "frac_of_mfma_only_loop": round(tf / state["bf16_ceiling"], 4) if state["bf16_ceiling"] else None,
                                   "traffic": _TRAFFIC.get(name), "traffic_source": "profiles/ (not measured in this run)"}}

    def sec_prefill():
        # ---- W4A4 prefill: M=4096, N=11008, K=4096, activations quantised inside the call
        M, N, K = 4096, 11008, 4096
        a = synth.activation_channel_outliers(M, K).to(dev)
        w = _randn_bf16((N, K), 0.02, gen, dev)
        wc, wm = _quantize_rows(hif4, w)
        c = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ref3 = lambda: torch.matmul(a, w.t(), out=c)   # the vendor library's plain BF16 GEMM on the unquantised operands
        ref3()
        _settle(ref3)
        ms = _timed(ref3, steps)
        legs["reference_bf16_library_gemm_M4096_N11008_K4096"] = {"ms": round(ms, 4), "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1)}
        del w
        ac, am = hif4.hif4_quantize(a)
        # the workspace with room for a decoded copy of W: both operands decoded once, plain BF16 main loop
        ws = torch.empty(hif4.hif4_gemm_workspace_bytes_decoded_w(hif4.HIF4_A_BF16_QUANTIZE, M, N, K), dtype=torch.uint8, device=dev)
        ws_small = torch.empty(hif4.hif4_gemm_workspace_bytes(hif4.HIF4_A_BF16_QUANTIZE, M, K), dtype=torch.uint8, device=dev)
        QK = hif4.HIF4_A_BF16_QUANTIZE
        main_cols, tail_width = hif4.hif4_gemm_plan_planes_split(M, N)   # how the library cuts this call's columns into launches
        cut = f", columns in {main_cols} tile columns of 256 + the rest in tiles of {tail_width}" if tail_width != 256 else ""
        planes = plan(QK, M, N, K, ws=ws.numel()) + cut + " (+ pre-passes: encode_to_planes, decode_planes)"
        tiles = plan(QK, M, N, K, ws=ws_small.numel()) + " (+ pre-pass: encode_to_cells)"
        mfma_leg("gemm_w4a4_quantize_inside_M4096_N11008_K4096", M, N, K,
                 lambda: hif4.hif4_gemm(hif4.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, out_dtype=hif4.HIF4_OUT_BF16, c=c, workspace=ws),
                 planes)
        mfma_leg("gemm_w4a4_quantize_inside_small_workspace_M4096_N11008_K4096", M, N, K,
                 lambda: hif4.hif4_gemm(hif4.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, out_dtype=hif4.HIF4_OUT_BF16, c=c, workspace=ws_small),
                 tiles)
        mfma_leg("gemm_w4a4_prepacked_M4096_N11008_K4096", M, N, K,
                 lambda: hif4.hif4_gemm(hif4.HIF4_A_HIF4, ac, am, wc, wm, out_dtype=hif4.HIF4_OUT_BF16, c=c, workspace=ws),
                 planes)
        del ws_small
        mc, ms_, = hif4.hif4ref_mxfp4_pack(a)
        wq = hif4.hif4ref_mxfp4_pack(hif4.hif4_dequantize(wc, wm))       # any weights of that shape: speed only
        _settle(lambda: hif4.hif4ref_mxfp4_gemm(mc, ms_, wq[0], wq[1], c=c))
        ms = _timed(lambda: hif4.hif4ref_mxfp4_gemm(mc, ms_, wq[0], wq[1], c=c), steps)
        legs["reference_native_mxfp4_mfma_gemm_M4096_N11008_K4096"] = {"ms": round(ms, 4), "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1)}
        del mc, ms_, wq
        del a, ac, am, wc, wm, c, ws


    def sec_grouped():
        # ---- grouped W4A4, MoE-shaped: 64 experts, K=7168, N=2048, 8192 routed rows
        E, K, N = 64, 7168, 2048
        offs = synth.moe_offsets()
        M = int(offs[-1])
        a = synth.activation_gaussian(M, K, config=4).to(dev)
        w = _randn_bf16((E * N, K), 0.02, gen, dev)
        wc, wm = _quantize_rows(hif4, w)
        del w
        wc, wm = wc.view(E, N, K // 2), wm.view(E, N, K // 64)
        od = torch.from_numpy(offs).to(dev)
        c = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ws = torch.empty(hif4.hif4_gemm_workspace_bytes(hif4.HIF4_A_BF16_QUANTIZE, M, K), dtype=torch.uint8, device=dev)
        mfma_leg("grouped_gemm_w4a4_E64_rows8192_N2048_K7168", M, N, K,
                 lambda: hif4.hif4_grouped_gemm(hif4.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, od, out_dtype=hif4.HIF4_OUT_BF16, c=c, workspace=ws),
                 plan(hif4.HIF4_A_BF16_QUANTIZE, M, N, K, experts=E, ws=ws.numel()) + " (+ pre-pass: encode_to_planes)")
        nbytes = E * N * K // 64 * 36 + M * K * 2 + M * N * 2
        legs["grouped_gemm_w4a4_E64_rows8192_N2048_K7168"]["GBps_algorithmic"] = round(
            nbytes / legs["grouped_gemm_w4a4_E64_rows8192_N2048_K7168"]["ms"] / 1e6, 1)
        del a, wc, wm, c, ws


    def sec_large():
        # ---- large prefill: M=16384, N=28672, K=8192, heavy-tailed activations
        if large:
            M, N, K = 16384, 28672, 8192
            a = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
            for r in range(0, M, 4096):   # Student-t(4) scaled to unit variance = z / sqrt(chi2_4 / 4) / sqrt(2)
                z = torch.randn((4096, K), generator=gen, device=dev)
                chi = torch.randn((4, 4096, K), generator=gen, device=dev).pow(2).sum(0)
                a[r:r + 4096] = (z / torch.sqrt(chi / 4.0) / np.sqrt(2.0)).to(torch.bfloat16)
            del z, chi
            w = _randn_bf16((N, K), 0.015, gen, dev)
            wc, wm = _quantize_rows(hif4, w)
            c = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            ws = torch.empty(hif4.hif4_gemm_workspace_bytes_decoded_w(hif4.HIF4_A_BF16_QUANTIZE, M, N, K), dtype=torch.uint8, device=dev)
            QK = hif4.HIF4_A_BF16_QUANTIZE
            planes = plan(QK, M, N, K, ws=ws.numel()) + " (+ pre-passes: encode_to_planes, decode_planes)"
            tiles = plan(QK, M, N, K, ws=hif4.hif4_gemm_workspace_bytes(QK, M, K)) + " (+ pre-pass: encode_to_cells)"
            mfma_leg("gemm_w4a4_quantize_inside_M16384_N28672_K8192", M, N, K,
                     lambda: hif4.hif4_gemm(hif4.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, out_dtype=hif4.HIF4_OUT_BF16, c=c, workspace=ws),
                     planes)
            small = hif4.hif4_gemm_workspace_bytes(hif4.HIF4_A_BF16_QUANTIZE, M, K)
            mfma_leg("gemm_w4a4_quantize_inside_small_workspace_M16384_N28672_K8192", M, N, K,
                     lambda: hif4.hif4_gemm(hif4.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, out_dtype=hif4.HIF4_OUT_BF16, c=c, workspace=ws[:small]),
                     tiles)
            # the result leaving as HiF4 (input of the next layer): epilogue of the same kernel, against the BF16
            # result followed by a separate encoder pass
            oc = torch.empty((M, N // 2), dtype=torch.uint8, device=dev)
            om = torch.empty((M, N // 64), dtype=torch.int32, device=dev)
            mfma_leg("gemm_w4a4_to_hif4_M16384_N28672_K8192", M, N, K,
                     lambda: hif4.hif4_gemm_to_hif4(hif4.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, c_codes=oc, c_meta=om, workspace=ws),
                     planes + " (HiF4 epilogue)")

            def two_step():
                hif4.hif4_gemm(hif4.HIF4_A_BF16_QUANTIZE, a, None, wc, wm, out_dtype=hif4.HIF4_OUT_BF16, c=c, workspace=ws)
                hif4.hif4_quantize(c, oc, om)
            mfma_leg("gemm_w4a4_then_quantize_M16384_N28672_K8192", M, N, K, two_step, planes + " + hif4::encode_kernel")
            del oc, om
            # speed reference on the same shape: CDNA4's native MXFP4 matrix instruction on the same tile kernel
            mc, ms_ = hif4.hif4ref_mxfp4_pack(a)
            wq = hif4.hif4ref_mxfp4_pack(w)
            hif4.hif4ref_mxfp4_gemm(mc, ms_, wq[0], wq[1], c=c)
            _settle(lambda: hif4.hif4ref_mxfp4_gemm(mc, ms_, wq[0], wq[1], c=c))
            ms = _timed(lambda: hif4.hif4ref_mxfp4_gemm(mc, ms_, wq[0], wq[1], c=c), steps)
            legs["reference_native_mxfp4_mfma_gemm_M16384_N28672_K8192"] = {
                "ms": round(ms, 4), "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1),
                "frac_of_mfma_only_loop": round(2.0 * M * N * K / ms / 1e9 / state["fp4_ceiling"], 4) if state["fp4_ceiling"] else None}
            del mc, ms_, wq
            # speed reference on the same shape: the vendor library's plain BF16 GEMM on the unquantised operands
            ref = lambda: torch.matmul(a, w.t(), out=c)
            ref()
            _settle(ref)
            ms = _timed(ref, max(2, steps // 2))
            legs["reference_bf16_library_gemm_M16384_N28672_K8192"] = {"ms": round(ms, 4), "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1)}
            del a, w, wc, wm, c, ws

    for name, fn in (("ceiling", sec_ceiling), ("decode", sec_decode), ("decode_large", sec_decode_large), ("prefill", sec_prefill),
                     ("grouped", sec_grouped), ("large", sec_large)):
        if want(name) and (large or name not in ("decode_large", "large")):
            fn()
            torch.cuda.empty_cache()
    torch.cuda.empty_cache()
    return legs
