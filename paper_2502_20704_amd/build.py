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


# a development variant with cycle counters between the phases of the reduction kernel
# (`python -m paper_2502_20704_amd.build --phase-timing`, read by `bench.py --phase-split`)
LIB_PHASE_TIMING = os.path.join(HERE, "libfsd_phase_timing.so")


def build(verbose: bool = False, phase_timing: bool = False) -> str:
    lib = LIB_PHASE_TIMING if phase_timing else LIB
    cmd = ["hipcc", *FLAGS, *(["-DFSD_PHASE_TIMING"] if phase_timing else []), "-o", lib, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(verbose=True, phase_timing="--phase-timing" in sys.argv[1:]))
