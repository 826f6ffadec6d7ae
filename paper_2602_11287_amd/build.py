"""Compile libhif4 (hand-written HIP, gfx950 only) in-tree with hipcc."""
import concurrent.futures
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhif4.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 arithmetic is kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


# Kernels that count their own outstanding loads (s_waitcnt vmcnt(N) literals next to LDS-writing loads the
# compiler does not see): a register spill would put vector memory instructions of the compiler's own between
# them and break the count, so the build refuses any scratch use in them.
HAND_COUNTED = ("gemm_colwave_kernel", "gemm_planes_kernel", "gemm_planes16_kernel", "gemm_fewrows_kernel", "gemm_stream_kernel")


def _check_no_scratch(remarks):
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif name and ("ScratchSize [bytes/lane]:" in line or "VGPRs Spill:" in line):
            value = int(line.split(":")[-1].split()[0])
            if value and any(k in name for k in HAND_COUNTED):
                raise RuntimeError(f"{name} uses scratch memory ({line.strip()}): its hand-counted s_waitcnt vmcnt would be wrong")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the gfx feature named above and says so: harmless noise
    lines = [l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l]
    remarks = "\n".join(l for l in lines if "kernel-resource-usage" in l)
    out = "\n".join(l for i, l in enumerate(lines) if "kernel-resource-usage" not in l and not _remark_context(lines, i))
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    _check_no_scratch(remarks)
    if verbose and out.strip():
        print(out, flush=True)


def _remark_context(lines, i):
    """The two source-context lines clang prints under each remark."""
    return any("kernel-resource-usage" in lines[j] for j in (i - 1, i - 2) if j >= 0) and ("|" in lines[i])


def build(verbose: bool = False, extra=()) -> str:
    """One hipcc -c per source, side by side (the kernels with many instantiations take most of a minute each),
    then one link.  Objects go to _build/, which is not tracked."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    jobs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
        jobs.append((obj, [hipcc, *flags, "-Rpass-analysis=kernel-resource-usage", *extra, "-c", "-o", obj, src]))
    workers = max(1, min(len(jobs), 8, os.cpu_count() or 1))
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
        for fut in [pool.submit(_run, cmd, verbose) for _, cmd in jobs]:
            fut.result()
    _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB, *[o for o, _ in jobs]], verbose)
    return LIB


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "hif4.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    build(verbose=True)
