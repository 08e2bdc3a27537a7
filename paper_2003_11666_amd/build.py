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


def build(verbose=True, timing=False, stamps=False):
    """timing=True: the development build with a time stamp at the start and the end of every
    workgroup (libpb_hip_timing.so, read by wg_timeline.py); stamps=True: the same library with the
    stamps inside the GEMM step as well (read by gemm_stamps.py; the stamps cost time themselves); the shipped library has none."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = TIMING_LIB if (timing or stamps) else LIB
    cmd = [hipcc] + FLAGS + (["-DPB_TIMING=1"] if stamps else ["-DPB_TIMING=2"] if timing else []) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out]
    cmd += ["-Rpass-analysis=kernel-resource-usage"]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    usage = check_resources(r.stderr)
    noise = ("kernel-resource-usage", "is not a recognized feature")
    rest = [l for l in r.stderr.splitlines() if l.strip() and not any(n in l for n in noise)
            and not l.lstrip().startswith(("|", "^")) and not l.lstrip()[:5].strip().isdigit()]
    if verbose or r.returncode:
        print("\n".join(rest), file=sys.stderr, flush=True)
    if r.returncode:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    if verbose:
        for name, u in usage.items():
            print(f"{name}: {u.get('VGPRs')} VGPRs, scratch {u.get('ScratchSize [bytes/lane]')} B/lane, "
                  f"{u.get('VGPRs Spill')} VGPR spills, LDS {u.get('LDS Size [bytes/block]')} B", flush=True)
    for name, u in usage.items():
        # every step of a tick is inlined into k_phase; a change that makes it spill slows every step down
        # (a spilling build measured 32 us instead of 12 us for a ResNet-20 launch)
        if "k_phase" in name and not (timing or stamps) and int(u.get("ScratchSize [bytes/lane]", 0)) > MAX_SCRATCH_BYTES:
            os.remove(out)      # a library that spills must not be the one that gets loaded
            raise RuntimeError(f"{name} uses {u['ScratchSize [bytes/lane]']} bytes of scratch memory per lane "
                               f"(limit {MAX_SCRATCH_BYTES}): a step spills registers")
    return out


MAX_SCRATCH_BYTES = 16


def check_resources(stderr_text):
    """Per kernel, the figures of the compiler's resource-usage remarks."""
    import re
    usage, cur = {}, None
    for line in stderr_text.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            cur = usage.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z \[\]/]+): (\S+) \[-Rpass-analysis", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = m.group(2)
    return usage


if __name__ == "__main__":
    print("built", build(timing="--timing" in sys.argv[1:], stamps="--stamps" in sys.argv[1:]))
