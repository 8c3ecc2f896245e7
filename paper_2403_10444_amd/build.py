"""Build libspecverify.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "specverify.hip")
LIB = os.path.join(HERE, "libspecverify.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
    # no implicit fused multiply-adds: a shift computed as m * k must be the SAME rounded number
    # wherever it is used (the kernels write every fma they want explicitly)
    "-ffp-contract=off",
    # no NaN ever enters the arithmetic (logits are finite by contract; -inf marks positions beyond a
    # row and is only ever compared, scaled or exponentiated): lets max/min compile to one instruction
    "-fno-honor-nans",
    # keep the compiler from forming packed-FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
    sys.exit(0)
