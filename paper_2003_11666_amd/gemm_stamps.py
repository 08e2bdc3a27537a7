"""Where the time of a GEMM tile goes, per GEMM step of one steady-state tick.

    python3 paper_2003_11666_amd/build.py --stamps          # libpb_hip_timing.so with -DPB_TIMING=1
    python3 -m paper_2003_11666_amd.gemm_stamps CONFIG [LAUNCH ...]     # on the GPU

The stamps build reads `s_memrealtime` (100 MHz) at fixed points of the GEMM step (the stamps cost a
little time themselves).  Printed per GEMM step of the chosen launches (default: all whose grid size is
unique in the tick): its shape and tiling from the plan, the number of workgroups, their mean duration,
the time the tile's MFMAs would take if the workgroup had a compute unit's four matrix pipes to itself
("ideal": 2 M N Q of the tile / 614.4 GFLOP/s), the resulting efficiency with two workgroups per
compute unit (ideal / (duration / 2)), and for the second chunk of the reduction of wavefront 0 (steps
with at least two chunks): storing the prefetched patch into LDS (with the wait for its loads), storing
the A block (with what was not prefetched), the barrier, issuing the next chunk's requests, the MFMA
loop; then the epilogue.
"""
from __future__ import annotations

import collections
import ctypes as C
import os
import re
import sys

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(_HERE))
SLOTS, REC = 16384, 100
CU_GFLOPS = 614.4      # one compute unit: 4 pipes x 64 flop per cycle x 2.4 GHz


def main():
    cfg = sys.argv[1] if len(sys.argv) > 1 else "resnet20"
    from paper_2003_11666_amd import binding
    lib_file = os.path.join(_HERE, "libpb_hip_timing.so")
    if not os.path.exists(lib_file):
        raise SystemExit("build the stamps library first: python3 paper_2003_11666_amd/build.py --stamps")
    binding.lib_path = lambda: lib_file
    import pb_workloads as W
    net = W.config(cfg)
    plan = {}
    for l in binding.plan_summary(net).splitlines():
        m = re.match(r"stage\s+(\d+) phase (\d+) gemm\s+tiles\s+(\d+) .*\| gm(\d) M(\d+) N(\d+) Q(\d+) waves (\S+) ni(\d) "
                     r"tile (\d+)x(\d+) x(\d+) chunks (\d+)/(\d+) QC(\d+)", l)
        if m:
            v = m.groups()
            plan[(int(v[0]), int(v[3]), int(v[4]))] = dict(N=int(v[5]), Q=int(v[6]), waves=v[7], tile=f"{v[9]}x{v[10]}x{v[11]}",
                                                           chunks=f"{v[12]}/{v[13]}", QC=int(v[14]))
    eng = binding.PBEngine(net, lr=net["lr"], momentum=net["momentum"], seed=W.WEIGHT_SEED)
    lib = binding.load_library()
    x, y = W.sample_pool(net)
    grids = (C.c_int32 * 64)()
    lib.pb_debug_phase_grids.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int]
    n_ph = lib.pb_debug_phase_grids(eng.ctx, grids, 64)
    grids = [int(grids[i]) for i in range(n_ph)]
    which = [int(a) for a in sys.argv[2:]] or [i for i, g in enumerate(grids) if grids.count(g) == 1]
    print(f"{cfg}: {n_ph} launches per tick, workgroups {grids}")
    warm = 2 * len(net["stages"]) + 8
    t = 0
    for ph in which:
        grid = grids[ph]
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
        agg = collections.defaultdict(list)
        other = collections.defaultdict(float)
        for i in range(min(grid, SLOTS)):
            ts = r[i, 4:].reshape(4, 24) / 100.0
            if ts[0, 0] <= 0:
                continue
            if int(r[i, 0]) == 10:
                agg[(int(r[i, 1]), int(r[i, 2]) & 7, int(r[i, 2]) >> 3)].append(ts[0])
            else:
                other[int(r[i, 0])] += float(ts[:, 11].max() - ts[0, 0])
        print(f"launch {ph} (grid {grid}): microseconds; chunk columns are means over the step's workgroups")
        print("stage gm      M     N     Q tile      chunks   QC waves     n    dur  ideal   eff | patch     A  barr issue  mfma |  epi")
        rows = []
        for k, v in agg.items():
            a = np.array(v)

            def dl(p, q):
                # a stamp the workgroup did not pass keeps the value of an earlier workgroup: outside its own interval
                m = (a[:, p] > a[:, 0]) & (a[:, q] >= a[:, 0]) & (a[:, p] <= a[:, 11]) & (a[:, q] <= a[:, 11]) & (a[:, p] >= a[:, q])
                return float(np.mean(a[m, p] - a[m, q])) if m.any() else float("nan")
            dur = float(np.mean(a[:, 11] - a[:, 0]))
            pl = plan.get(k)
            if pl is None:
                continue
            ideal = 2.0 * k[2] * pl["N"] * pl["Q"] / len(v) / (CU_GFLOPS * 1e3)
            rows.append((len(v) * dur, k, pl, len(v), dur, ideal, ideal / (dur / 2),
                         dl(14, 12), dl(15, 14), dl(16, 15), dl(13, 16), dl(17, 13), dl(11, 8)))
        rows.sort(key=lambda q: -q[0])
        tot = sum(q[0] for q in rows)
        tot_ideal = sum(q[3] * q[5] * 2 for q in rows)
        for q in rows:
            k, pl = q[1], q[2]
            print(f"{k[0]:5d} {k[1]:2d} {k[2]:6d} {pl['N']:5d} {pl['Q']:5d} {pl['tile']:9s} {pl['chunks']:>6s} {pl['QC']:4d} {pl['waves']:5s} "
                  f"{q[3]:5d} {q[4]:6.1f} {q[5]:6.1f} {100 * q[6]:5.0f}% | " + " ".join(f"{z:5.2f}" for z in q[7:12]) + f" | {q[12]:4.2f}")
        print(f"GEMM workgroups: {tot:.0f} workgroup-us ({tot / 512:.0f} us over 512 slots), ideal {tot_ideal:.0f}: "
              f"efficiency {100 * tot_ideal / max(tot, 1):.0f} %; other step kinds {sum(other.values()):.0f} workgroup-us")


if __name__ == "__main__":
    main()
