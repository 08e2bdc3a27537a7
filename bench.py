#!/usr/bin/env python3
"""PB ticks/s at batch 1 on one MI355X, with the fused update kernel's share
of HBM peak and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config resnet20]

A step is one pipeline tick: ingest of one sample, every stage's forward and
backward work, the fused SC+LWP update.  Samples come from a pool resident in
HBM before the timed region starts.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# measured HBM bytes per algorithmic byte of the update kernel (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)
UPDATE_TRAFFIC_PER_ALGORITHMIC_BYTE = 1.0
HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
# k_phase: bytes that crossed the L2 / fabric boundary per algorithmic byte of the launch, from
# `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this script (FETCH_SIZE scaled by 2, WRITE_SIZE
# by 1: what the counters read for a plain copy of known size): profiles/k_phase_hbm_traffic.md
KPHASE_TRAFFIC_PER_ALGORITHMIC_BYTE = {"resnet20": 2.55, "mlp": 1.84, "vgg11": 1.13, "wide": 1.27, "resnet50_fp32": 1.98}


def tick_algorithmic_bytes(net, n_params, lwp=True):
    """36 B per parameter (update 20 B + 4 B predicted-weight write, 4 B
    gradient write by backward-weights, 4 B forward read of the predicted
    weights, 4 B backward-data read of the weights) + 6 accesses of every
    stage-boundary activation element (forward write/read, ring write/read is
    the same storage here, gradient write/read)."""
    import pb_workloads as W
    a = sum(c * h * w for (_, (c, h, w)) in W.stage_shapes(net)[:-1])
    return 36 * n_params + 6 * a * 4


def cpu_baseline(net, budget_s=15.0):
    import torch
    import pb_workloads as W
    from oracle import pb_oracle as O
    xs, ys = W.sample_pool(net, n=min(net["n_pool"], 128))
    orc = O.PBOracle(net)
    S = len(net["stages"])
    fill = 2 * (S - 1) + 1
    t_begin = time.perf_counter()
    for t in range(fill):
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
        if time.perf_counter() - t_begin > 4 * budget_s:
            break
    n, t0 = 0, time.perf_counter()
    while True:
        t = orc.t
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
        n += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s:
            break
    return {"value": n / dt, "unit": "ticks/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"{n} steady-state ticks of the same workload after {orc.t - n} fill ticks "
                      f"(float64 PyTorch-CPU oracle, {dt:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--config", default="resnet20")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-standalone", action="store_true")
    ap.add_argument("--launch-mode", type=int, default=0, help="1 = one launch per step (profiling aid)")
    ap.add_argument("--no-step-profile", action="store_true",
                    help="skip the pass that launches every step on its own (keeps a kernel trace of this run clean)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the pipeline on ONE GPU only; --gpus must be 1 "
              "(sharding the pipeline's stages over several GPUs is described in the design notes, not built)", file=sys.stderr)
        sys.exit(2)

    import torch
    import pb_workloads as W
    from paper_2003_11666_amd import PBEngine, update_standalone

    net = W.config(args.config)
    S = len(net["stages"])
    xs, ys = W.sample_pool(net)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    xd = torch.from_numpy(xs).to(dev)
    yd = torch.from_numpy(ys).to(dev)
    eng = PBEngine(net, mitigation=3)
    if args.launch_mode:
        eng.set_launch_mode(args.launch_mode)
    n_params = eng.n_params

    warm = max(args.warmup, 2 * (S - 1) + 1)      # steady state: every stage busy
    eng.run_resident(xd, yd, 0, warm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.run_resident(xd, yd, warm, args.steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ticks_per_s = args.steps / dt

    # second pass over the same region with HIP events around every launch
    # (a) the launches as timed above; (b) one launch per step, which isolates the
    # duration of the update steps inside the tick
    prof_ticks = min(args.steps, 500)
    eng.profile_begin(64 * prof_ticks)
    eng.run_resident(xd, yd, warm + args.steps, prof_ticks)
    n_ph, ms_ph = eng.profile_end(0)
    prof2 = 0 if args.no_step_profile else min(args.steps, 200)
    n_upd = n_in = 0
    ms_upd = ms_in = 0.0
    if prof2:
        eng.set_launch_mode(1)
        eng.profile_begin(512 * prof2)
        eng.run_resident(xd, yd, warm + args.steps + prof_ticks, prof2)
        n_upd, ms_upd = eng.profile_end(1)
        n_in, ms_in = eng.profile_end(2)
    eng.set_launch_mode(args.launch_mode)
    # update steps of one tick (one launch per stage in this mode): 24 B per parameter
    # (w, v, g read; w, v, w_hat written)
    upd_us_tick = 1e3 * ms_upd / max(prof2, 1)
    upd_bytes = 24 * n_params
    upd_gbs = upd_bytes / (upd_us_tick * 1e-6) / 1e9 if prof2 else None
    # the dominant kernel: k_phase, all steps of a phase in one launch
    tick_bytes = tick_algorithmic_bytes(net, n_params)
    ph_us_tick = 1e3 * ms_ph / prof_ticks
    launches = n_ph / prof_ticks
    achieved = tick_bytes / (ph_us_tick * 1e-6) / 1e9
    losses = eng.loss_history()
    assert len(losses) and all(l == l for l in losses[-100:]), "non-finite loss"

    out = {
        "metric": "PB ticks/sec (batch 1)", "value": ticks_per_s, "unit": "ticks/s", "n_gpus": 1,
        "steps": args.steps, "warmup": warm, "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{net['name']}: {S} pipeline stages, input {net['in_c']}x{net['in_h']}x{net['in_w']}, "
                               f"{n_params} parameters, batch 1, SC_D+LWP_D, lr {net['lr']}, momentum {net['momentum']}, "
                               f"pool of {len(ys)} resident samples"},
        "roofline": {"kernel": "k_phase (every step of a tick: forward, backward and update of all stages)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (KPHASE_TRAFFIC_PER_ALGORITHMIC_BYTE[args.config] * tick_bytes / launches
                                 if args.config in KPHASE_TRAFFIC_PER_ALGORITHMIC_BYTE else None),
                     "avg_launch_us": ph_us_tick / launches, "launches_per_tick": launches,
                     "algorithmic_bytes_per_launch": tick_bytes / launches},
        "update_in_tick": {"kernel": "k_phase, update steps only (one launch per stage)", "bound": "hbm",
                           "achieved": upd_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": upd_gbs / HBM_PEAK_GBS if prof2 else None,
                           "us_per_tick": upd_us_tick, "launches_per_tick": n_upd / max(prof2, 1),
                           "algorithmic_bytes_per_tick": upd_bytes},
        "tick_roofline": {"bound": "hbm", "algorithmic_bytes": tick_bytes,
                          "frac": tick_bytes / (dt / args.steps) / 1e9 / HBM_PEAK_GBS},
        "kernel_time_us_per_tick": {"phase_launches": ph_us_tick, "launches_per_tick": launches,
                                    "update_steps_alone": upd_us_tick,
                                    "ingest_alone": 1e3 * ms_in / max(prof2, 1)},
        "final_loss_mean_last_200": float(losses[-200:].mean()),
    }
    eng.close()

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
        out["update_standalone"] = {"kernel": "k_update_flat (the update step's arithmetic over plain arrays)",
                                    "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": gbs / HBM_PEAK_GBS, "elements": n, "avg_launch_us": us,
                                    "algorithmic_bytes_per_launch": 24 * n,
                                    # FETCH_SIZE + WRITE_SIZE of this kernel at this size, each scaled by what the
                                    # counter reads for a plain copy: profiles/k_update_flat_1GiB_arrays.md
                                    "traffic": UPDATE_TRAFFIC_PER_ALGORITHMIC_BYTE * 24 * n}
        del w, v, g, wh

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(net)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
