"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2602_11287_amd import build, hif4
    if build.stale():
        build.build()
    return hif4.load()


def declared_functions():
    """Every function declared in any header under include/."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if not f.endswith(".h"):
            continue
        text = open(os.path.join(inc, f)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(hif4[a-z]*_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    from paper_2602_11287_amd import hif4
    names = declared_functions()
    assert sorted(hif4.EXPORTS) == names
    for n in names:
        assert hasattr(lib, n), n
        assert hasattr(hif4, n), f"binding lacks {n}"


def test_version_and_status_strings(lib):
    from paper_2602_11287_amd import hif4
    assert hif4.hif4_version() == 1
    for s in range(0, -7, -1):
        assert hif4.hif4_status_string(s) != "unknown status"
    assert hif4.hif4_status_string(-99) == "unknown status"


def test_quantize_argument_errors(lib):
    from paper_2602_11287_amd import hif4 as h
    q = lib.hif4_quantize
    p = 0x1000  # never dereferenced: every call below fails validation or is a no-op
    assert q(p, 4, 100, 100, p, p, 0, None) == h.HIF4_ERR_SHAPE      # K not a multiple of 64
    assert q(p, -1, 128, 128, p, p, 0, None) == h.HIF4_ERR_SHAPE
    assert q(p, 4, 128, 64, p, p, 0, None) == h.HIF4_ERR_SHAPE       # ldx < K
    assert q(p, 4, 128, 128, p, p, 7, None) == h.HIF4_ERR_UNSUPPORTED
    assert q(None, 4, 128, 128, p, p, 0, None) == h.HIF4_ERR_NULL
    assert q(p, 4, 128, 128, None, p, 0, None) == h.HIF4_ERR_NULL
    assert q(p + 2, 4, 128, 128, p, p, 0, None) == h.HIF4_ERR_ALIGN
    assert q(p, 4, 128, 132, p, p, 0, None) == h.HIF4_ERR_ALIGN      # row stride not 16-byte
    assert q(p, 4, 128, 128, p, p + 1, 0, None) == h.HIF4_ERR_ALIGN
    assert q(None, 0, 128, 128, None, None, 0, None) == h.HIF4_OK    # empty: no-op
    assert q(None, 5, 0, 0, None, None, 0, None) == h.HIF4_OK


def test_dequantize_argument_errors(lib):
    from paper_2602_11287_amd import hif4 as h
    d = lib.hif4_dequantize
    p = 0x1000
    assert d(p, p, 4, 96, p, 96, None) == h.HIF4_ERR_SHAPE
    assert d(p, p, 4, 128, p, 64, None) == h.HIF4_ERR_SHAPE
    assert d(p, None, 4, 128, p, 128, None) == h.HIF4_ERR_NULL
    assert d(p, p, 4, 128, p + 4, 128, None) == h.HIF4_ERR_ALIGN
    assert d(None, None, 0, 128, None, 128, None) == h.HIF4_OK


def test_gemm_argument_errors(lib):
    from paper_2602_11287_amd import hif4 as h
    g, gg = lib.hif4_gemm, lib.hif4_grouped_gemm
    p = 0x1000
    ok = dict(a_kind=h.HIF4_A_HIF4, a=p, a_meta=p, lda=256, w=p, wm=p, M=8, N=16, K=256, c=p, ldc=16, out=1, ws=p, wsz=8 * 256 * 2)

    def call(**kw):
        a = dict(ok, **kw)
        return g(a["a_kind"], a["a"], a["a_meta"], a["lda"], a["w"], a["wm"], a["M"], a["N"], a["K"], a["c"], a["ldc"],
                 a["out"], a["ws"], a["wsz"], None)

    assert call(a_kind=9) == h.HIF4_ERR_UNSUPPORTED
    assert call(out=5) == h.HIF4_ERR_UNSUPPORTED
    assert call(K=100) == h.HIF4_ERR_SHAPE
    assert call(ldc=8) == h.HIF4_ERR_SHAPE
    assert call(a_kind=h.HIF4_A_BF16_KEEP, lda=128) == h.HIF4_ERR_SHAPE
    assert call(a_meta=None) == h.HIF4_ERR_NULL
    assert call(w=None) == h.HIF4_ERR_NULL
    assert call(c=None) == h.HIF4_ERR_NULL
    assert call(w=p + 4) == h.HIF4_ERR_ALIGN
    assert call(M=0) == h.HIF4_OK and call(N=0) == h.HIF4_OK
    # HiF4 activations need a workspace of the advertised size: the decoded BF16 copy (when the call
    # quantises them itself, the packed planes never reach memory)
    need = lib.hif4_gemm_workspace_bytes(h.HIF4_A_BF16_QUANTIZE, 8, 256)
    assert need == 8 * 256 * 2
    assert lib.hif4_gemm_workspace_bytes(h.HIF4_A_HIF4, 8, 256) == 8 * 256 * 2
    assert lib.hif4_gemm_workspace_bytes(h.HIF4_A_BF16_KEEP, 8, 256) == 0
    assert call(ws=None, wsz=0) == h.HIF4_ERR_WORKSPACE
    assert call(wsz=8 * 256 * 2 - 1) == h.HIF4_ERR_WORKSPACE
    assert call(ws=p + 8) == h.HIF4_ERR_ALIGN
    assert call(a_kind=h.HIF4_A_BF16_QUANTIZE, a_meta=None, ws=None, wsz=0) == h.HIF4_ERR_WORKSPACE
    assert call(a_kind=h.HIF4_A_BF16_QUANTIZE, a_meta=None, ws=p, wsz=need - 1) == h.HIF4_ERR_WORKSPACE
    # grouped: offsets are required once there is work
    assert gg(h.HIF4_A_HIF4, p, p, 256, p, p, None, 4, 8, 16, 256, p, 16, 1, p, 4096, None) == h.HIF4_ERR_NULL
    assert gg(h.HIF4_A_HIF4, p, p, 256, p, p, None, -1, 8, 16, 256, p, 16, 1, p, 4096, None) == h.HIF4_ERR_SHAPE
    assert gg(h.HIF4_A_HIF4, p, p, 256, p, p, None, 0, 8, 16, 256, p, 16, 1, p, 4096, None) == h.HIF4_OK
    # grouped with a HiF4 result: units of the result run along N; both planes and the offsets are required
    gh = lib.hif4_grouped_gemm_to_hif4
    assert gh(h.HIF4_A_HIF4, p, p, 256, p, p, p, 4, 8, 96, 256, p, p, 0, p, 4096, None) == h.HIF4_ERR_SHAPE
    assert gh(h.HIF4_A_HIF4, p, p, 256, p, p, p, 4, 8, 128, 256, p, p, 7, p, 4096, None) == h.HIF4_ERR_UNSUPPORTED
    assert gh(h.HIF4_A_HIF4, p, p, 256, p, p, p, 4, 8, 128, 256, p, None, 0, p, 4096, None) == h.HIF4_ERR_NULL
    assert gh(h.HIF4_A_HIF4, p, p, 256, p, p, None, 4, 8, 128, 256, p, p, 0, p, 4096, None) == h.HIF4_ERR_NULL
    assert gh(h.HIF4_A_HIF4, p, p, 256, p, p, p, 4, 8, 128, 256, p, p, 1, p, 4095, None) == h.HIF4_ERR_WORKSPACE
    assert gh(h.HIF4_A_HIF4, p, p, 256, p, p, p, 4, 0, 128, 256, p, p, 1, p, 4096, None) == h.HIF4_OK


def test_product_path_has_no_cpu_fallback():
    """The binding imports neither the oracle nor any CPU implementation."""
    src = open(os.path.join(ROOT, "paper_2602_11287_amd", "hif4.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")


def test_quantize_from_argument_errors(lib):
    from paper_2602_11287_amd import hif4 as h
    q = lib.hif4_quantize_from
    p = 0x1000
    assert q(3, p, 4, 128, 128, p, p, 0, None) == h.HIF4_ERR_UNSUPPORTED      # unknown input type
    assert q(2, p, 4, 128, 128, p, p, 2, None) == h.HIF4_ERR_UNSUPPORTED      # unknown rounding
    assert q(2, p, 4, 100, 100, p, p, 0, None) == h.HIF4_ERR_SHAPE
    assert q(1, None, 4, 128, 128, p, p, 0, None) == h.HIF4_ERR_NULL
    assert q(2, p, 4, 128, 130, p, p, 0, None) == h.HIF4_ERR_ALIGN            # fp32 rows: ldx multiple of 4
    assert q(1, p, 4, 128, 132, p, p, 0, None) == h.HIF4_ERR_ALIGN            # fp16 rows: ldx multiple of 8
    assert q(2, p + 4, 4, 128, 128, p, p, 0, None) == h.HIF4_ERR_ALIGN
    assert q(2, None, 0, 128, 128, None, None, 0, None) == h.HIF4_OK


def test_compare_tools_argument_errors(lib):
    from paper_2602_11287_amd import hif4 as h
    p = 0x1000
    assert lib.hif4cmp_mxfp4_fake_quant(p, 4, 48, 48, None, None, None) == h.HIF4_ERR_SHAPE   # K % 32
    assert lib.hif4cmp_nvfp4_fake_quant(p, 4, 40, 40, None, None, None, None) == h.HIF4_ERR_SHAPE  # K % 16
    assert lib.hif4cmp_mxfp4_fake_quant(None, 4, 64, 64, None, None, None) == h.HIF4_ERR_NULL
    assert lib.hif4cmp_mxfp4_fake_quant(p, 4, 64, 64, p + 4, None, None) == h.HIF4_ERR_ALIGN
    assert lib.hif4cmp_nvfp4_fake_quant(p, 4, 64, 64, p + 2, None, None, None) == h.HIF4_ERR_ALIGN
    assert lib.hif4cmp_abs_max(p, 4, 64, 64, None, None) == h.HIF4_ERR_NULL
    assert lib.hif4cmp_sq_err_bf16(p, p, 4, 64, 64, 32, p, None) == h.HIF4_ERR_SHAPE          # ldy < K
    assert lib.hif4cmp_sq_err_bf16(p, p, 4, 64, 64, 64, None, None) == h.HIF4_ERR_NULL
    assert lib.hif4cmp_mxfp4_fake_quant(None, 0, 64, 64, None, None, None) == h.HIF4_OK
    assert lib.hif4ref_mfma_loop(3, 16, p, None) == h.HIF4_ERR_UNSUPPORTED


def test_gemm_to_hif4_argument_errors(lib):
    from paper_2602_11287_amd import hif4 as h
    f = lib.hif4_gemm_to_hif4
    p = 0x1000
    ok = (h.HIF4_A_BF16_KEEP, p, None, 128, p, p, 4, 128, 128, p, p, 0, None, 0, None)
    def call(**kw):
        names = ["a_kind", "a", "a_meta", "lda", "w_codes", "w_meta", "M", "N", "K", "c_codes", "c_meta", "round", "ws", "wsz", "stream"]
        args = list(ok)
        for k, v in kw.items():
            args[names.index(k)] = v
        return f(*args)
    assert call(N=100) == h.HIF4_ERR_SHAPE            # units of the result run along N
    assert call(round=5) == h.HIF4_ERR_UNSUPPORTED
    assert call(c_meta=None) == h.HIF4_ERR_NULL
    assert call(c_codes=None) == h.HIF4_ERR_NULL
    assert call(c_codes=p + 8) == h.HIF4_ERR_ALIGN
    assert call(a_kind=h.HIF4_A_HIF4, a_meta=p, ws=None) == h.HIF4_ERR_WORKSPACE
    assert call(M=0, a=None, c_codes=None, c_meta=None) == h.HIF4_OK


def test_build_refuses_scratch_in_kernels_that_count_their_own_loads():
    """The kernels with hand-counted s_waitcnt vmcnt literals must not spill (a spill adds vector memory instructions
    the count does not know): the build reads the compiler's resource report and fails on any scratch use in them."""
    from paper_2602_11287_amd import build
    with pytest.raises(RuntimeError):
        build._check_no_scratch("f.hip:1:1: remark: Function Name: _ZN4hif419gemm_colwave_kernelILi6ELi8EEEv [-Rpass-analysis=kernel-resource-usage]\n"
                                "f.hip:1:1: remark:     ScratchSize [bytes/lane]: 16 [-Rpass-analysis=kernel-resource-usage]")
    build._check_no_scratch("f.hip:1:1: remark: Function Name: _ZN4hif419gemm_colwave_kernelILi6ELi8EEEv [-Rpass-analysis=kernel-resource-usage]\n"
                            "f.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]")
