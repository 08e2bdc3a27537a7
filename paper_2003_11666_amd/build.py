"""Builds libpb_hip.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpb_hip.so")
SOURCES = ["pb_kernels.hip", "pb_host.cpp"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-ffp-contract=off", "-Wall", "-Wno-unused-function"]


TIMING_LIB = os.path.join(HERE, "libpb_hip_timing.so")


def build(verbose=True, timing=False):
    """timing=True: the development build with a time stamp at the start and the end of every
    workgroup (libpb_hip_timing.so, read by wg_timeline.py); the shipped library has none."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = TIMING_LIB if timing else LIB
    cmd = [hipcc] + FLAGS + (["-DPB_TIMING=2"] if timing else []) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print("built", build(timing="--timing" in sys.argv[1:]))
