"""Which main loop a GEMM call runs (hif4_gemm_plan, the host function the library itself dispatches by), walked
over a grid of shapes and checked against the dispatch table written out here in plain rules.  No GPU involved."""
import itertools

import pytest

from paper_2602_11287_amd import hif4 as h

Q, P, KEEP = h.HIF4_A_BF16_QUANTIZE, h.HIF4_A_HIF4, h.HIF4_A_BF16_KEEP
MI = 1 << 20


@pytest.fixture(scope="module")
def lib():
    return h.load()


def few_rows_prefer_k_split(M, N, K):
    return M <= 16 or (M <= 32 and N * K <= 48 * MI) or (M <= 64 and N * K <= 24 * MI)


def colwave_dense_rows(M, N):
    if M <= 192:
        return M
    strips = -(-N // 32) * -(-M // 128)
    return 0 if (strips > 2048 or M > 2048) else 128   # (the tile height beyond 1024 strips does not matter here)


def decoded_w_pays(M, N, K):
    return M >= 3328 or (M >= 1536 and N * K <= 128 * MI and colwave_dense_rows(M, N) == 0)


def fewrows(M, N, K):
    ok_shape = K % 256 == 0 and N * (K // 2) < 2 ** 32
    return ok_shape and M <= 32 and N >= 6144


def expected(a_kind, M, N, K, emit, ws):
    """The table: rules in the order the library applies them (dense calls)."""
    keep = a_kind == KEEP
    a_bf16 = M * K * 2
    if K == 0:
        return "hif4::zero_kernel"
    if not emit and fewrows(M, N, K):
        return "hif4::gemm_fewrows_kernel"
    fits32 = M * 128 < 2 ** 32 and N * (K // 2) < 2 ** 32 and a_bf16 < 2 ** 32
    colwave_ok = colwave_dense_rows(M, N) > 0 and fits32 and (not keep or ws >= a_bf16)
    if keep and M <= 64 and not emit and (few_rows_prefer_k_split(M, N, K) or not colwave_ok):
        return "hif4::gemm_stream_kernel" if (M > 32 and K % 128 == 0 and N >= 12288) else "hif4::gemm_skinny_kernel"
    if decoded_w_pays(M, N, K) and ws >= -(-a_bf16 // 16) * 16 + N * K * 2:
        return "hif4::gemm_planes16_kernel"
    if not keep and not emit and M <= 64 and few_rows_prefer_k_split(M, N, K):
        return "hif4::gemm_skinny_kernel"
    if colwave_ok:
        return "hif4::gemm_colwave_kernel"
    return "hif4::gemm_kernel"


ROWS = [1, 5, 16, 17, 32, 33, 64, 65, 128, 192, 193, 512, 1024, 1535, 1536, 2048, 2049, 3327, 3328, 4096, 16384]
WEIGHTS = [(4096, 4096), (11008, 4096), (4096, 11008), (14336, 4096), (2048, 7168), (28672, 8192), (8192, 28672), (16384, 8192),
           (320, 64), (12288, 128), (28672, 320)]


def test_plan_follows_the_table(lib):
    seen = set()
    for (M, (N, K), a_kind, emit) in itertools.product(ROWS, WEIGHTS, (Q, P, KEEP), (False, True)):
        if emit and N % 64:
            continue
        need = h.hif4_gemm_workspace_bytes(a_kind, M, K)
        for ws in sorted({need, h.hif4_gemm_workspace_bytes_decoded_w(a_kind, M, N, K), need + M * K * 2}):
            plan = lib.hif4_gemm_plan(a_kind, 0, M, N, K, int(emit), ws)
            got = lib.hif4_gemm_plan_name(plan).decode()
            assert got == expected(a_kind, M, N, K, emit, ws), (a_kind, M, N, K, emit, ws, got)
            seen.add(got)
    assert seen == {"hif4::gemm_fewrows_kernel", "hif4::gemm_skinny_kernel", "hif4::gemm_stream_kernel", "hif4::gemm_colwave_kernel",
                    "hif4::gemm_planes16_kernel", "hif4::gemm_kernel"}


def test_plan_of_the_benchmark_configurations(lib):
    """The kernels the five configurations are measured on (the labels bench.py prints come from the same query)."""
    def name(a_kind, M, N, K, experts=0, big=False):
        ws = h.hif4_gemm_workspace_bytes_decoded_w(a_kind, M, N, K) if big else h.hif4_gemm_workspace_bytes(a_kind, M, K)
        return lib.hif4_gemm_plan_name(lib.hif4_gemm_plan(a_kind, experts, M, N, K, 0, ws)).decode()
    assert name(KEEP, 16, 4096, 4096) == "hif4::gemm_skinny_kernel"
    assert name(KEEP, 16, 28672, 8192) == "hif4::gemm_fewrows_kernel"
    assert name(Q, 4096, 11008, 4096) == "hif4::gemm_kernel" and name(Q, 4096, 11008, 4096, big=True) == "hif4::gemm_planes16_kernel"
    assert name(Q, 8192, 2048, 7168, experts=64) == "hif4::gemm_colwave_kernel"
    assert name(KEEP, 8192, 2048, 7168, experts=64) == "hif4::gemm_kernel"          # no room for a reordered copy of A
    assert name(Q, 16384, 28672, 8192, big=True) == "hif4::gemm_planes16_kernel"


def test_plan_rejects_what_the_calls_reject(lib):
    assert lib.hif4_gemm_plan(7, 0, 8, 64, 64, 0, 1 << 20) == h.HIF4_ERR_UNSUPPORTED
    assert lib.hif4_gemm_plan(P, 0, 8, 64, 100, 0, 1 << 20) == h.HIF4_ERR_SHAPE
    assert lib.hif4_gemm_plan(P, 0, 8, 96, 64, 1, 1 << 20) == h.HIF4_ERR_SHAPE       # a HiF4 result needs N % 64 == 0
    assert lib.hif4_gemm_plan(P, 0, 8, 64, 64, 0, 8 * 64 * 2 - 1) == h.HIF4_ERR_WORKSPACE
    assert lib.hif4_gemm_plan(P, 0, 8, 64, 0, 0, 0) == h.HIF4_PLAN_ZERO_FILL
    assert lib.hif4_gemm_plan_name(99) == b"unknown plan"


# ---- how a call on decoded operands is cut into launches (hif4_gemm_plan_planes_split)

def rounds_of_launch(tiles_m, tiles_n):
    """Rounds of one workgroup per CU: the kernels deal the tiles of a launch to the 8 XCDs (32 CUs each) in equal shares."""
    return -(-(-(-tiles_m * tiles_n // 8)) // 32)


REL = {256: 1.0, 192: 0.80, 128: 0.60}   # time of a round of narrower tiles, in rounds of 256-column tiles (measured: 0.795 for 192)
GAP = 0.04


def test_planes_split_of_known_shapes():
    assert h.hif4_gemm_plan_planes_split(4096, 11008) == (32, 192)    # 688 tiles: two rounds of 256 x 256, then 240 tiles of 256 x 192
    assert h.hif4_gemm_plan_planes_split(16384, 28672) == (0, 256)    # 28 whole rounds
    assert h.hif4_gemm_plan_planes_split(4096, 4096) == (0, 256)      # one whole round
    assert h.hif4_gemm_plan_planes_split(2048, 2048) == (0, 256)      # less than a round: nothing to gain
    assert h.hif4_gemm_plan_planes_split(0, 0) == (0, 256)
    main, width = h.hif4_gemm_plan_planes_split(4096, 14336)          # 3.5 rounds
    assert width in (192, 128) and main > 0


def test_planes_split_covers_the_columns_and_saves_rounds():
    for M in (1536, 1600, 2048, 3328, 4096, 5000, 8192, 16384):
        for N in (2048, 4096, 5120, 8192, 11008, 11000, 14336, 16384, 22016, 28672):
            main, width = h.hif4_gemm_plan_planes_split(M, N)
            tm, tn = -(-M // 256), -(-N // 256)
            assert width in (256, 192, 128) and 0 <= main < max(tn, 1)
            assert width != 256 or main == 0                           # a tail of 256-column tiles is no split at all
            if width == 256:
                continue
            assert 256 < tm * tn <= 16 * 256                           # never for one round or less, nor for many rounds
            tail_tiles = -(-(N - 256 * main) // width)
            assert tail_tiles >= 1 and 256 * main + width * tail_tiles >= N   # every column has a tile
            t_split = rounds_of_launch(tm, main) + REL[width] * rounds_of_launch(tm, tail_tiles) + (GAP if main else 0.0)
            assert t_split <= 0.97 * rounds_of_launch(tm, tn) + 1e-9, (M, N, main, width)


def test_planes_split_rejects_bad_arguments(lib):
    import ctypes as C
    a, b = C.c_int(0), C.c_int(0)
    assert lib.hif4_gemm_plan_planes_split(-1, 64, C.byref(a), C.byref(b)) == h.HIF4_ERR_SHAPE
    assert lib.hif4_gemm_plan_planes_split(64, 64, None, C.byref(b)) == h.HIF4_ERR_NULL
