"""Build step: compile the HIP sources under csrc/ into libmx4.so for gfx950 with hipcc."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmx4.so")
# measurement aids of bench.py (yardstick kernels that allocate their own buffers): a library of their own
BENCH_CSRC = os.path.join(HERE, "bench_csrc")
BENCH_LIB = os.path.join(HERE, "libmx4_bench.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # IEEE division and fp32 denormals: the MBS-Dynamic cost must round as its definition says
    "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
    "-Wall", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]
# MFMA results in ordinary VGPRs, where the vector ALUs consume them without copies (MBS correction)
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
# Per-source extra flags.  The large-tile plain GEMM keeps its accumulators in the accumulation registers
# and is therefore compiled without the VGPR form.
EXTRA = {"mx_gemm_wide.hip": []}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature; that is harmless
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    work = tempfile.mkdtemp(prefix="mx4_build_")
    try:
        objs = []
        jobs = []
        for src in sources():
            name = os.path.basename(src)
            obj = os.path.join(work, name + ".o")
            objs.append(obj)
            jobs.append([HIPCC] + FLAGS + EXTRA.get(name, VGPR_FORM) + ["-c", src, "-o", obj])
        with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
            list(pool.map(lambda c: _run(c, verbose), jobs))
        tmp = os.path.join(work, "libmx4.so")
        _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp], verbose)
        # a kernel the host pass failed to emit shows up only as an unresolved symbol of our own namespace
        undefined = subprocess.run(["nm", "-u", tmp], stdout=subprocess.PIPE, text=True).stdout
        missing = [l.split()[-1] for l in undefined.splitlines() if "_ZN2mx" in l]
        if missing:
            raise RuntimeError("libmx4.so has unresolved symbols: " + ", ".join(missing))
        shutil.move(tmp, LIB)
        bench_srcs = sorted(glob.glob(os.path.join(BENCH_CSRC, "*.hip")))
        tmp = os.path.join(work, "libmx4_bench.so")
        _run([HIPCC] + FLAGS + ["-shared"] + bench_srcs + ["-o", tmp], verbose)
        shutil.move(tmp, BENCH_LIB)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
