"""Builds libuncomp.so (HIP kernels + C interface) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libuncomp.so")
SOURCES = ["api.hip", "gram.hip", "jacobi.hip", "tridiag.hip", "budgets.hip", "score.hip", "select.hip", "select_wide.hip", "decode.hip", "hidden.hip", "prepare.hip", "subspace.hip", "subspace_mfma.hip", "peaks.hip", "noalloc.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",                           # MFMA results straight into VGPRs (no AGPR copies)
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
