"""Builds ``libjigsaw.so`` (HIP, gfx950) in-tree with hipcc.  Host-only: hipcc cross-compiles."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "jigsaw.hip")
LIB = os.path.join(HERE, "libjigsaw.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # No packed FP32 VALU instructions (v_pk_fma_f32 and friends) in any kernel of this library.  The flag acts
    # on the gfx950 pass (a float2 multiply-add compiles to two scalar-lane FMAs with it, to one v_pk_fma_f32
    # without); the x86 host pass does not know the feature and says so in a warning.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_hip(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra, "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build_hip(verbose=True, extra=sys.argv[1:])
