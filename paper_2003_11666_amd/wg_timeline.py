"""Start and end of every workgroup inside the launches of one steady-state tick.

    python3 paper_2003_11666_amd/build.py --timing        # libpb_hip_timing.so (-DPB_TIMING=2)
    python3 -m paper_2003_11666_amd.wg_timeline CONFIG     # on the GPU

The timing build stamps `s_memrealtime` (100 MHz) at the start and the end of every workgroup and
stores the stamps of its four wavefronts in a buffer indexed by workgroup.  Printed per launch of
the tick: by step kind, the number of workgroups, mean start, mean and longest duration and last
end (microseconds from the first workgroup of the launch), the workgroups that end last, and a
histogram of start times.  Launches of one tick must differ in grid size to be told apart.
"""
from __future__ import annotations

import collections
import ctypes as C
import os
import sys

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(_HERE))

KINDS = {0: "gn_stats", 1: "gap_fwd", 2: "conv_fwd", 3: "post_fwd", 4: "ce", 5: "gnb_reduce", 6: "gnb_apply",
         7: "conv_bwd_x", 8: "conv_bwd_w", 9: "copy", 10: "gemm", 11: "bias_grad", 12: "ingest", 13: "update",
         14: "head", 15: "gn_bwd", 16: "dot_fwd", 17: "dot_bwd_x", 18: "fc_fwd", 19: "fc_bwd_x", 20: "fc_bwd_w"}
SLOTS, REC = 16384, 100


def main():
    cfg = sys.argv[1] if len(sys.argv) > 1 else "resnet20"
    from paper_2003_11666_amd import binding
    lib_file = os.path.join(_HERE, "libpb_hip_timing.so")
    if not os.path.exists(lib_file):
        raise SystemExit("build the timing library first: python3 paper_2003_11666_amd/build.py --timing")
    binding.lib_path = lambda: lib_file
    import pb_workloads as W
    net = W.config(cfg)
    eng = binding.PBEngine(net, lr=net["lr"], momentum=net["momentum"], seed=W.WEIGHT_SEED)
    lib = binding.load_library()
    x, y = W.sample_pool(net)
    grids = (C.c_int32 * 64)()
    lib.pb_debug_phase_grids.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int]
    n_ph = lib.pb_debug_phase_grids(eng.ctx, grids, 64)
    grids = [int(grids[i]) for i in range(n_ph)]
    print(f"{cfg}: {n_ph} launches per tick, workgroups {grids}")
    warm = 2 * len(net["stages"]) + 8 if "stages" in net else 120
    t = 0
    for ph, grid in enumerate(grids):
        if grids.count(grid) > 1 or grid > SLOTS:
            print(f"launch {ph}: grid {grid} not unique in the tick or above {SLOTS} workgroups, skipped")
            continue
        lib.pb_debug_clear()
        lib.pb_debug_set_grid(C.c_int(grid))
        lib.pb_debug_set_tick(C.c_int(t + warm))
        for _ in range(warm + 4):
            eng.tick(x[t % len(x)], int(y[t % len(x)]))
            t += 1
        eng.sync()
        buf = np.zeros(SLOTS * REC, dtype=np.int64)
        lib.pb_debug_dump(buf.ctypes.data_as(C.POINTER(C.c_longlong)), C.c_int(SLOTS))
        r = buf.reshape(SLOTS, REC)
        rows = []
        for i in range(grid):
            ts = r[i, 4:].reshape(4, 24)
            st, en = ts[:, 0], ts[:, 11]
            if (st > 0).any():
                rows.append((i, KINDS.get(int(r[i, 0]), "?"), int(r[i, 1]), int(r[i, 2]) & 7, int(r[i, 3]),
                             st[st > 0].min() / 100.0, en.max() / 100.0))
        if not rows:
            print(f"launch {ph}: no records")
            continue
        t0 = min(q[5] for q in rows)
        print(f"launch {ph} (grid {grid}): {len(rows)} workgroups recorded, first start to last end "
              f"{max(q[6] for q in rows) - t0:.2f} us")
        agg = collections.defaultdict(list)
        for q in rows:
            agg[(q[1], q[3])].append((q[5] - t0, q[6] - q[5]))
        for k, v in sorted(agg.items()):
            print(f"  {k[0]:<10s} gm {k[1]}  n {len(v):5d}  mean start {np.mean([a for a, b in v]):6.2f}  "
                  f"mean dur {np.mean([b for a, b in v]):6.2f}  max dur {max(b for a, b in v):6.2f}  "
                  f"last end {max(a + b for a, b in v):6.2f}")
        for q in sorted(rows, key=lambda q: -q[6])[:8]:
            print(f"    wg {q[0]:5d} {q[1]:<9s} stage {q[2]:2d} gm {q[3]} tile {q[4]:4d}  start {q[5] - t0:6.2f}  "
                  f"end {q[6] - t0:6.2f}")
        edges = [0, 0.5, 1, 2, 4, 6, 8, 10, 15, 20, 50, 100, 1e9]
        hist = np.histogram([q[5] - t0 for q in rows], bins=edges)[0]
        print("  start-time histogram (us: workgroups): " +
              ", ".join(f"{edges[i]:g}-: {hist[i]}" for i in range(len(hist)) if hist[i]))


if __name__ == "__main__":
    main()
