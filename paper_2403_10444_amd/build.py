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


PROFILE_LIB = os.path.join(HERE, "libspecverify_profile.so")


def build(verbose: bool = False, profile: bool = False) -> str:
    """Builds the library.  `profile`: a second library for tuning, libspecverify_profile.so, whose fused kernel
    also stores per-workgroup timestamps (-DSV_PROFILE adds the entry point spec_verify_debug_profile and the
    stores); the product library holds neither."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = PROFILE_LIB if profile else LIB
    cmd = [hipcc, *HIPCC_FLAGS, *(["-DSV_PROFILE"] if profile else []), "-o", out, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(verbose=True, profile="--profile" in sys.argv[1:]))
    sys.exit(0)
