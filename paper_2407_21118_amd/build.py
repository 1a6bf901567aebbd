"""Builds the HIP shared library for gfx950 in-tree with hipcc."""

from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_NAME = "libpalu_hip.so"
LIB_PATH = os.path.join(HERE, LIB_NAME)

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",     # no packed-FP32 VALU forms
    "-fno-fast-math", "-ffp-contract=off",
    "-Wall", "-Wno-unused-function",
]
# The matrix instructions of the attention kernels write ordinary vector registers, so their float32
# epilogues read the accumulators without a copy per value; the prompt-sized projection keeps its 256
# accumulators per lane in the accumulation registers and is compiled on its own without the option.
# (The shared-key forms of the whole-head score kernel unroll 64 matrix instructions with the vector work of up to
# eight queries dealt out between them: beyond the default size limit of "#pragma unroll".)
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form", "-mllvm", "-pragma-unroll-threshold=200000"]
BUILD_DIR = os.path.join(HERE, "_build")


def sources():
    """(source file, extra flags) of every translation unit."""
    return [(os.path.join(CSRC, "api.hip"), VGPR_FORM), (os.path.join(CSRC, "encode_gemm.hip"), [])]


def _run(procs, verbose):
    for cmd, proc in procs:
        out = proc.communicate()[0]
        lines = [l for l in out.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l]
        if verbose and lines:
            print("\n".join(lines), flush=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + "\n".join(lines))


def build_library(verbose: bool = True) -> str:
    """Compile csrc/ into libpalu_hip.so next to this file and return its path."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    os.makedirs(BUILD_DIR, exist_ok=True)
    inc = ["-I", os.path.join(HERE, "..", "include")]
    objects, procs = [], []
    for src, extra in sources():
        obj = os.path.join(BUILD_DIR, os.path.splitext(os.path.basename(src))[0] + ".o")
        cmd = [hipcc] + HIPCC_FLAGS + extra + inc + ["-c", "-o", obj, src]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objects.append(obj)
    _run(procs, verbose)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objects
    if verbose:
        print(" ".join(link), flush=True)
    _run([(link, subprocess.Popen(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))], verbose)
    return LIB_PATH


if __name__ == "__main__":
    build_library()
    sys.exit(0)
