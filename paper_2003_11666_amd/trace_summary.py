"""Text summary of a rocprofv3 kernel trace (or counter collection) of a bench.py run.

    rocprofv3 --kernel-trace --stats -d OUT -o run -- python3 bench.py ...
    python3 -m paper_2003_11666_amd.trace_summary OUT [--steps CONFIG]
    python3 -m paper_2003_11666_amd.trace_summary OUT --counters

Reads the .db file rocprofv3 leaves under OUT (its rocpd SQLite output) and prints
  * the kernels by total time (the `top_kernels` view),
  * the `k_phase` launches grouped by grid size, i.e. by phase of the tick,
  * with --steps CONFIG, for a run made with `bench.py --launch-mode 1`
    (one launch per step, in step-table order): the mean duration of every step of the tick,
  * with --counters, for a `--pmc` run: the mean counter value per kernel.
"""
from __future__ import annotations

import argparse
import collections
import glob
import os
import re
import sqlite3
import sys


def find_db(path):
    if os.path.isfile(path):
        return path
    hits = sorted(glob.glob(os.path.join(path, "**", "*.db"), recursive=True))
    if not hits:
        raise SystemExit(f"no .db file under {path}")
    return hits[0]


def top_kernels(cur, limit=8):
    print("kernel | calls | total us | mean us | % of kernel time")
    for name, calls, total, avg, pct in cur.execute(
            "select name,total_calls,total_duration,average,percentage from top_kernels limit ?", (limit,)):
        print(f"{name[:70]} | {calls} | {total:.1f} | {avg:.3f} | {pct:.2f}")


def phases(cur):
    rows = list(cur.execute("select grid_x, workgroup_x, (end-start)/1000.0 from kernels where name like '%pb::k_phase%'"))
    agg = collections.OrderedDict()
    for gx, wx, d in rows:
        agg.setdefault(gx // max(wx, 1), []).append(d)
    print("k_phase launches by grid size (workgroups) | launches | mean us | min | max")
    for g, v in sorted(agg.items(), key=lambda kv: -len(kv[1]))[:10]:
        print(f"{g:6d} | {len(v)} | {sum(v) / len(v):.2f} | {min(v):.2f} | {max(v):.2f}")


def steps(cur, config):
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import pb_workloads as W
    from paper_2003_11666_amd import binding as B
    plan = B.plan_summary(W.config(config)).strip().split("\n")
    rows = list(cur.execute("select start, end from kernels where name like '%pb::k_phase%' order by start"))
    n = len(plan)
    ticks = [rows[i:i + n] for i in range(0, len(rows) - n + 1, n)]
    ticks = ticks[len(ticks) // 2:]            # steady state: every stage busy
    print(f"{n} steps per tick, {len(ticks)} ticks averaged; mean us (max over stages) x stages | step")
    agg, phmax = collections.OrderedDict(), {}
    for si, line in enumerate(plan):
        d = sum((t[si][1] - t[si][0]) / 1000.0 for t in ticks) / len(ticks)
        ph = int(re.search(r"phase (\d+)", line).group(1))
        phmax[ph] = max(phmax.get(ph, 0.0), d)
        key = re.sub(r"first_tick +\d+ ", "", re.sub(r"stage +\d+ ", "", line))
        agg.setdefault(key, []).append(d)
    for k, v in sorted(agg.items(), key=lambda kv: -max(kv[1])):
        print(f"{sum(v) / len(v):6.2f} ({max(v):6.2f}) x{len(v):2d} | {k[:170]}")
    # streaming steps (the plan gives their algorithmic bytes): achieved bandwidth per step class
    cls = collections.OrderedDict()
    for si, line in enumerate(plan):
        m = re.search(r"phase \d+ (\w+) .*\| bytes (\d+)", line)
        if not m:
            continue
        d = sum((t[si][1] - t[si][0]) / 1000.0 for t in ticks) / len(ticks)
        c = cls.setdefault(m.group(1), [0, 0.0, 0, 0.0])
        c[0] += int(m.group(2)); c[1] += d; c[2] += 1
        c[3] = max(c[3], int(m.group(2)) / d / 1e3)
    print("step class | steps per tick | algorithmic MB per tick | us per tick (one launch per step) | GB/s over the class | "
          "best single step GB/s | % of 8 TB/s (class, best step)")
    for k, (b, us, n, best) in cls.items():
        print(f"{k} | {n} | {b / 1e6:.2f} | {us:.1f} | {b / us / 1e3:.0f} | {best:.0f} | {b / us / 1e3 / 80:.1f}, {best / 80:.1f}")
    print("slowest step per phase (us):", {k: round(v, 2) for k, v in sorted(phmax.items())})


def counters(cur):
    q = ("select kernel_name, counter_name, avg(value), count(*) from counters_collection "
         "group by kernel_name, counter_name")
    print("kernel | counter | mean per dispatch | dispatches")
    for k, c, v, n in cur.execute(q):
        print(f"{k[:70]} | {c} | {v:.1f} | {n}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("out")
    ap.add_argument("--steps", default=None, metavar="CONFIG")
    ap.add_argument("--counters", action="store_true")
    args = ap.parse_args()
    cur = sqlite3.connect(find_db(args.out)).cursor()
    if args.counters:
        counters(cur)
        return
    top_kernels(cur)
    phases(cur)
    if args.steps:
        steps(cur, args.steps)


if __name__ == "__main__":
    main()
