#!/usr/bin/env python3
"""PB ticks/s at batch 1 on one MI355X, the tick's share of its roofline, the
fused update kernel's share of HBM peak and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config resnet20]

A step is one pipeline tick: ingest of one sample, every stage's forward and
backward work, the fused SC+LWP update.  Samples come from a pool resident in
HBM before the timed region starts.  Prints ONE JSON line:

  value / ms_per_step   exactly --steps ticks of --config, host clock, synchronised on both sides
  steady_state          median of 5 windows of >= 1000 ticks (HIP events around each window, host clock beside)
  roofline              the dominant kernel k_phase: algorithmic bytes per launch / mean launch duration
  all_configs           the other benchmark configurations measured the same way, oracle beside each
  update_standalone     the update arithmetic over 1 GiB arrays: the kernel's ceiling beyond every cache
  cpu_baseline          the float64 oracle on the host, one thread (primary) and all cores
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
# Bytes that crossed the L2 / fabric boundary per algorithmic byte of a k_phase launch, from `rocprofv3 --pmc
# FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this script (each scaled by what the counter reads for a plain copy of
# known size): profiles/k_phase_counters_all_configs.md.  A figure from those runs, not a measurement of this run.
KPHASE_TRAFFIC_PER_ALGORITHMIC_BYTE = {"resnet20": 2.59, "mlp": 1.76, "vgg11": 0.88, "wide": 1.26, "resnet50": 1.64}
TRAFFIC_SOURCE = "profiles/k_phase_counters_all_configs.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes over this command; not measured by this run)"
UPDATE_TRAFFIC_PER_ALGORITHMIC_BYTE = 1.0   # profiles/k_update_flat_1GiB_arrays.md


def tick_algorithmic_bytes(net, n_params):
    """36 B per parameter (update 20 B + 4 B predicted-weight write, 4 B gradient write by
    backward-weights, 4 B forward read of the predicted weights, 4 B backward-data read of the
    weights) + 6 accesses of every stage-boundary activation element (forward write/read, ring
    write/read is the same storage here, gradient write/read)."""
    import pb_workloads as W
    a = sum(c * h * w for (_, (c, h, w)) in W.stage_shapes(net)[:-1])
    return 36 * n_params + 6 * a * 4


def oracle_rate(net, budget_s, threads):
    """Steady-state ticks/s of the oracle as it stands (never tuned), on `threads` host threads."""
    import torch
    import pb_workloads as W
    from oracle import pb_oracle as O
    torch.set_num_threads(threads)
    xs, ys = W.sample_pool(net, n=min(net["n_pool"], 128))
    orc = O.PBOracle(net)
    S = len(net["stages"])
    for t in range(2 * (S - 1) + 1):          # fill: every stage busy afterwards
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
    n, t0 = 0, time.perf_counter()
    while True:
        t = orc.t
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
        n += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s:
            break
    return n / dt, n, dt, orc.t - n


def cpu_baseline(net, budget_s=10.0):
    import torch
    all_threads = torch.get_num_threads()
    r1, n1, dt1, fill = oracle_rate(net, budget_s, 1)
    ra, na, dta, _ = oracle_rate(net, budget_s, all_threads)
    torch.set_num_threads(all_threads)
    return {"value": r1, "unit": "ticks/s", "threads": 1, "cores": os.cpu_count(), "kind": "oracle",
            "all_cores": {"value": ra, "threads": all_threads},
            "sample": f"{n1} steady-state ticks of the same workload after {fill} fill ticks on one thread ({dt1:.1f} s), "
                      f"{na} on {all_threads} threads ({dta:.1f} s); float64 PyTorch-CPU oracle"}


def measure(name, steps, warmup, windows=5, window_ticks=1000, update_share=False, launch_mode=0):
    """Ticks/s of one configuration: the CLI's --steps window (host clock) and `windows` steady-state
    windows of `window_ticks` ticks (HIP events + host clock)."""
    import torch
    import pb_workloads as W
    from paper_2003_11666_amd import PBEngine
    net = W.config(name)
    S = len(net["stages"])
    xs, ys = W.sample_pool(net)
    dev = torch.device("cuda:0")
    xd, yd = torch.from_numpy(xs).to(dev), torch.from_numpy(ys).to(dev)
    eng = PBEngine(net, mitigation=3)
    if launch_mode:
        eng.set_launch_mode(launch_mode)
    n_params = eng.n_params
    warm = max(warmup, 2 * (S - 1) + 1)       # steady state: every stage busy
    eng.run_resident(xd, yd, 0, warm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.run_resident(xd, yd, warm, steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    done = warm + steps
    ev_ms, wall_ms = [], []
    for _ in range(windows):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        e0.record()
        eng.run_resident(xd, yd, done, window_ticks)
        e1.record()
        torch.cuda.synchronize()
        wall_ms.append(1e3 * (time.perf_counter() - w0))
        ev_ms.append(e0.elapsed_time(e1))
        done += window_ticks
    # launches per tick (one HIP event pair per launch, a few ticks only)
    eng.profile_begin(64 * 16)
    eng.run_resident(xd, yd, done, 16)
    n_launch, _ = eng.profile_end(0)
    done += 16
    launches = n_launch / 16
    tick_us = 1e3 * statistics.median(ev_ms) / window_ticks
    tick_bytes = tick_algorithmic_bytes(net, n_params)
    res = {"net": net, "S": S, "n_params": n_params, "warm": warm, "dt": dt, "ticks_per_s_cli": steps / dt,
           "steady": {"ticks_per_s": 1e6 / tick_us, "us_per_tick": tick_us, "windows": windows, "window_ticks": window_ticks,
                      "event_ms_per_window": [round(x, 3) for x in ev_ms],
                      "ticks_per_s_host_clock": 1e3 * window_ticks / statistics.median(wall_ms)},
           "launches": launches, "tick_bytes": tick_bytes, "pool": len(ys)}
    if update_share:
        # the update steps inside the tick, one launch per step: 24 B per parameter (w, v, g read; w, v, w_hat written)
        eng.set_launch_mode(1)
        k = 20
        eng.profile_begin(1024 * k)
        eng.run_resident(xd, yd, done, k)
        n_upd, ms_upd = eng.profile_end(1)
        eng.set_launch_mode(launch_mode)
        us = 1e3 * ms_upd / k
        res["update_in_tick"] = {"kernel": "k_phase, update steps only (one launch per stage)", "bound": "hbm",
                                 "achieved": 24 * n_params / (us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": 24 * n_params / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "us_per_tick": us,
                                 "launches_per_tick": n_upd / k, "algorithmic_bytes_per_tick": 24 * n_params}
    losses = eng.loss_history()
    assert len(losses) and all(l == l for l in losses[-100:]), f"{name}: non-finite loss"
    res["final_loss"] = float(losses[-200:].mean())
    eng.close()
    del xd, yd
    return res


def roofline_of(r, name):
    """k_phase of one configuration: algorithmic bytes per launch over the mean launch duration.  The
    launches of a window run back to back on one stream, so the window's event time over its number
    of launches bounds the mean kernel duration from above (it holds the dispatch gaps too)."""
    per_launch = r["tick_bytes"] / r["launches"]
    launch_us = r["steady"]["us_per_tick"] / r["launches"]
    achieved = per_launch / (launch_us * 1e-6) / 1e9
    ratio = KPHASE_TRAFFIC_PER_ALGORITHMIC_BYTE.get(name)
    return {"kernel": "k_phase (every step of a tick: forward, backward and update of all stages)", "bound": "hbm",
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": ratio * per_launch if ratio else None, "traffic_source": TRAFFIC_SOURCE if ratio else None,
            "avg_launch_us": launch_us, "launches_per_tick": r["launches"], "algorithmic_bytes_per_launch": per_launch}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--config", default="resnet20")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-standalone", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true", help="measure --config only")
    ap.add_argument("--windows", type=int, default=5)
    ap.add_argument("--window-ticks", type=int, default=0, help="ticks per steady-state window (0: 1000, 2000 for the MLP)")
    ap.add_argument("--launch-mode", type=int, default=0, help="1 = one launch per step (profiling aid)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the pipeline on ONE GPU only; --gpus must be 1 "
              "(sharding the pipeline's stages over several GPUs is described in the design notes, not built)", file=sys.stderr)
        sys.exit(2)

    import torch
    import pb_workloads as W
    from paper_2003_11666_amd import update_standalone

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wt = args.window_ticks or 1000
    r = measure(args.config, args.steps, args.warmup, args.windows, wt, launch_mode=args.launch_mode)
    net, S = r["net"], r["S"]
    out = {
        "metric": "PB ticks/sec (batch 1)", "value": r["ticks_per_s_cli"], "unit": "ticks/s", "n_gpus": 1,
        "steps": args.steps, "warmup": r["warm"], "ms_per_step": 1e3 * r["dt"] / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{net['name']}: {S} pipeline stages, input {net['in_c']}x{net['in_h']}x{net['in_w']}, "
                               f"{r['n_params']} parameters, batch 1, SC_D+LWP_D, lr {net['lr']}, momentum {net['momentum']}, "
                               f"pool of {r['pool']} resident samples"},
        "steady_state": r["steady"],
        "roofline": roofline_of(r, args.config),
        "tick_roofline": {"bound": "hbm", "algorithmic_bytes": r["tick_bytes"],
                          "frac": r["tick_bytes"] / (r["steady"]["us_per_tick"] * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "final_loss_mean_last_200": r["final_loss"],
    }

    if not args.no_all_configs:
        allc = {}
        for name in W.BENCH_CONFIGS:
            if name == args.config:
                continue
            ticks = args.window_ticks or (2000 if name == "mlp" else 1000)
            q = measure(name, 100, 0, args.windows, ticks, update_share=(name == "resnet50"))
            rf = roofline_of(q, name)
            e = {"stages": q["S"], "parameters": q["n_params"], "ticks_per_s": q["steady"]["ticks_per_s"],
                 "us_per_tick": q["steady"]["us_per_tick"], "ticks_per_s_host_clock": q["steady"]["ticks_per_s_host_clock"],
                 "windows": f"{q['steady']['windows']} x {q['steady']['window_ticks']} ticks, median",
                 "launches_per_tick": q["launches"], "algorithmic_bytes_per_tick": q["tick_bytes"],
                 "tick_roofline_frac": q["tick_bytes"] / (q["steady"]["us_per_tick"] * 1e-6) / 1e9 / HBM_PEAK_GBS,
                 "traffic_per_algorithmic_byte": KPHASE_TRAFFIC_PER_ALGORITHMIC_BYTE.get(name), "traffic_source": TRAFFIC_SOURCE,
                 "avg_launch_us": rf["avg_launch_us"], "final_loss_mean_last_200": q["final_loss"],
                 "dtype": "f32 (activations rounded to bf16 at stage boundaries)" if q["net"].get("act_dtype") == "bf16" else "f32"}
            if "update_in_tick" in q:
                e["update_in_tick"] = q["update_in_tick"]
            if not args.no_cpu_baseline:
                th = torch.get_num_threads()
                rate, n, dt, fill = oracle_rate(q["net"], 4.0, th)
                e["cpu_oracle"] = {"ticks_per_s": rate, "threads": th, "cores": os.cpu_count(),
                                   "sample": f"{n} steady-state ticks after {fill} fill ticks ({dt:.1f} s)"}
            allc[name] = e
        out["all_configs"] = allc

    if not args.no_standalone:
        n = 256 * 1024 * 1024            # 1 GiB per array: far beyond L2 and Infinity Cache
        w = torch.randn(n, device=dev); v = torch.zeros(n, device=dev); g = torch.randn(n, device=dev)
        wh = torch.empty(n, device=dev)
        for _ in range(3):
            update_standalone(w, v, g, wh, 0.005, 0.9, 0.5, 4.0, 0.05)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record()
        for _ in range(reps):
            update_standalone(w, v, g, wh, 0.005, 0.9, 0.5, 4.0, 0.05)
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / reps
        gbs = 24 * n / (us * 1e-6) / 1e9
        out["update_standalone"] = {"kernel": "k_update_flat (the update step's arithmetic over plain arrays: the kernel's "
                                              "ceiling beyond every cache, not a figure of the tick)",
                                    "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": gbs / HBM_PEAK_GBS, "elements": n, "avg_launch_us": us,
                                    "algorithmic_bytes_per_launch": 24 * n,
                                    "traffic": UPDATE_TRAFFIC_PER_ALGORITHMIC_BYTE * 24 * n,
                                    "traffic_source": "profiles/k_update_flat_1GiB_arrays.md"}
        del w, v, g, wh

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(net)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
