"""Builds libsnn_mi355x.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsnn_mi355x.so")
SOURCES = ["snn_kernels.hip", "snn_api.cpp", "snn_schedule.cpp"]

# -ffp-contract=off: the forward/recompute arithmetic must not fuse multiply-adds (bit-exact spike
# trains); packed fp32 instructions are disabled for the whole library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-result"]


def build(verbose: bool = False) -> str:
    cmd = ["hipcc", *FLAGS, "-x", "hip", *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
