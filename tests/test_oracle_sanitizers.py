"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: every entry point runs on
seeded inputs (special values, ties, negative integer sums in the unit dot product) in a separate
program built with -fsanitize=address,undefined, must finish without a report, and must return the
bytes the ordinary build returns."""
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def build_sanitized(tmp):
    exe = os.path.join(tmp, "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-ffp-contract=off", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "hif4_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0 and "static-libasan" in proc.stdout:   # toolchain without the static runtime
        cmd.remove("-static-libasan")
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout
    return exe


def test_oracle_is_clean_under_asan_and_ubsan(oracle, tmp_path):
    rows, K = 6, 256
    rng = np.random.default_rng(77)
    xf = (rng.standard_normal((rows, K)) * np.exp(rng.uniform(-6, 6, (rows, 1)))).astype(np.float32)
    xf[0, :64] = rng.integers(-64, 65, 64) / 8.0            # short values: ties at every step
    xf[1, :6] = [np.inf, -np.inf, np.nan, 3.4e38, 1e-40, -0.0]
    xf[2, 64:128] = 0.0
    xf[3, :4] = [7.875, 5.6875, 10.0, -1.25]
    with np.errstate(over="ignore"):
        xh = xf.astype(np.float16)
    import torch
    from paper_2602_11287_amd import synth
    xb = synth.bits(torch.from_numpy(xf).to(torch.bfloat16))
    xb[4, :3] = [0x7F7F, 0x0001, 0x8000]                    # largest finite, least subnormal, minus zero
    inp, outp = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        f.write(np.array([rows, K], np.int64).tobytes())
        f.write(xb.tobytes())
        f.write(xf.tobytes())
        f.write(xh.view(np.uint16).tobytes())
    exe = build_sanitized(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    proc = subprocess.run([exe, str(inp), str(outp)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                          timeout=120)
    assert proc.returncode == 0, proc.stdout
    assert "runtime error" not in proc.stdout and "AddressSanitizer" not in proc.stdout, proc.stdout

    want = b""
    for mode in (0, 1):
        c, m = oracle.quantize(xb, mode)
        want += c.tobytes() + m.tobytes() + oracle.dequantize(c, m).tobytes()
        for arr in (xf, xh):
            c2, m2 = oracle.quantize_from(arr, mode)
            want += c2.tobytes() + m2.tobytes()
    c, m = oracle.quantize(xb)
    y = oracle.dequantize(c, m)
    want += oracle.gemm_f64(y, y).tobytes()
    want += np.array([oracle.unit_dot(c[0, 32 * u:32 * u + 32], m[0, u], c[1, 32 * u:32 * u + 32], m[1, u])
                      for u in range(K // 64)], np.float64).tobytes()
    got = open(outp, "rb").read()
    assert len(got) == len(want)
    # NaN payloads compare as bytes: both builds run the same arithmetic
    assert got == want
