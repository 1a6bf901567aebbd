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
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",     # no packed-FP32 VALU forms
    "-fno-fast-math", "-ffp-contract=off",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [os.path.join(CSRC, "api.hip")]


def build_library(verbose: bool = True) -> str:
    """Compile csrc/ into libpalu_hip.so next to this file and return its path."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(HERE, "..", "include"), "-o", LIB_PATH] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l]
    if verbose and lines:
        print("\n".join(lines), flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
    return LIB_PATH


if __name__ == "__main__":
    build_library()
    sys.exit(0)
