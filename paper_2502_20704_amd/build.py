"""Builds libfsd.so (HIP kernels + C ABI) for gfx950 next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "fsd_kernels.hip")
LIB = os.path.join(HERE, "libfsd.so")

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    # no implicit fusing of a*b+c: the kernels say fmaf() where they want one, and both the
    # bit-exact Gumbel transform and "equal rows give exactly zero" rely on separately rounded products
    "-ffp-contract=off",
    # packed-fp32 instructions are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"),
]


def build(verbose: bool = False) -> str:
    cmd = ["hipcc", *FLAGS, "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
