"""Runs the fused SC+LWP update over plain arrays, and a plain copy of known size beside it.

Used under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` to read the HBM traffic of the update
kernel: the copy kernel (torch's `copy_`, n floats read and n written) calibrates what the counter
reports per byte moved.

    python3 -m paper_2003_11666_amd.update_bench [--elements N] [--reps R]
"""
from __future__ import annotations

import argparse
import json
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--elements", type=int, default=256 * 1024 * 1024)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    import torch
    from paper_2003_11666_amd import update_standalone

    dev = torch.device("cuda:0")
    n = args.elements
    w = torch.randn(n, device=dev)
    v = torch.zeros(n, device=dev)
    g = torch.randn(n, device=dev)
    wh = torch.empty(n, device=dev)
    dst = torch.empty(n, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.reps):
        update_standalone(w, v, g, wh, 0.005, 0.9, 0.5, 4.0, 0.05)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.reps):
        dst.copy_(w)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    print(json.dumps({"elements": n, "reps": args.reps,
                      "update_bytes_per_launch": 24 * n, "update_us": 1e6 * (t1 - t0) / args.reps,
                      "copy_bytes_per_launch": 8 * n, "copy_us": 1e6 * (t2 - t1) / args.reps}))


if __name__ == "__main__":
    main()
