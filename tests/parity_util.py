"""Helpers that drive the HIP engine and the CPU oracle on the same seeded
inputs and compare them tensor by tensor."""
import numpy as np

import pb_workloads as W
from oracle import pb_oracle as O

TOL = 1e-5   # per-tick relative weight tolerance for fp32 (stated by the benchmark spec)
# A ReLU mask is an integer decision taken on a floating-point value.  When a
# pre-activation lands within rounding error of zero, fp32 and fp64 arithmetic
# may legitimately decide differently, and the gradient of that sample then
# differs by a finite amount (one element's contribution).  The oracle's own
# conditioning tells when that happens: a second oracle whose initial weights
# are perturbed by PERTURB (about the rounding error of an fp32 forward pass)
# is run alongside (two of them, with different perturbations); while the
# oracles agree to WELL_CONDITIONED the trajectory is well conditioned and the
# strict tolerance applies, after a tie event the tolerance for the remaining
# ticks is SENS_FACTOR times the oracles' own disagreement.
PERTURB = (3e-7, 1e-6)
SENS_FACTOR = 4.0
WELL_CONDITIONED = 1e-5   # oracle-vs-perturbed-oracle disagreement up to which TOL applies (the perturbation itself reaches ~5e-6 on large tensors)


def tensor_slices(net):
    """[(stage, name, start, stop)] of the canonical flat parameter vector."""
    out, off = [], 0
    for s, st in enumerate(net["stages"]):
        for name, shape, _ in O.stage_param_specs(st):
            n = int(np.prod(shape))
            out.append((s, name, off, off + n))
            off += n
    return out


def median_rel_error(a, b, slices):
    """Median over tensors of max|d|/max|ref|: robust against the few tensors a
    ReLU-mask tie touches."""
    errs = []
    for s, name, lo, hi in slices:
        r = b[lo:hi]
        mx = np.abs(r).max()
        if mx > 0:
            errs.append(np.abs(a[lo:hi].astype(np.float64) - r).max() / mx)
    return float(np.median(errs)) if errs else 0.0


def rel_errors(a, b, slices):
    """Worst per-tensor max|d|/max|ref| and ||d||2/||ref||2 (ref = b)."""
    worst_inf, worst_l2, where = 0.0, 0.0, None
    for s, name, lo, hi in slices:
        x, r = a[lo:hi].astype(np.float64), b[lo:hi]
        d = x - r
        mx = np.abs(r).max()
        if mx == 0.0:
            assert np.abs(d).max() == 0.0, (s, name, "reference is zero, engine is not")
            continue
        e_inf = np.abs(d).max() / mx
        e_l2 = np.linalg.norm(d) / np.linalg.norm(r)
        if e_inf > worst_inf:
            worst_inf, where = e_inf, (s, name)
        worst_l2 = max(worst_l2, e_l2)
    return worst_inf, worst_l2, where


def perturbed_oracle(net, seed, mitigation, eps, gen_seed=12345, lr=None, bwd_weights=0):
    import torch
    orc = O.PBOracle(net, seed=seed, mitigation=mitigation, lr=lr, bwd_weights=bwd_weights)
    g = torch.Generator().manual_seed(gen_seed)
    for p in orc.w:
        for k in p:
            p[k] = p[k] * (1.0 + eps * torch.randn(p[k].shape, generator=g, dtype=torch.float64))
    return orc


def run_parity(engine_cls, net, K, mitigation=3, seed=42, every=1, engine_kwargs=None, verbose=False, lr=None,
               perturb=PERTURB, bwd_weights=0):
    xs, ys = W.sample_pool(net)
    orc = O.PBOracle(net, seed=seed, mitigation=mitigation, lr=lr, bwd_weights=bwd_weights)
    orcs = [perturbed_oracle(net, seed, mitigation, e, 12345 + i, lr=lr, bwd_weights=bwd_weights) for i, e in enumerate(perturb)]
    eng = engine_cls(net, seed=seed, mitigation=mitigation, lr=lr, bwd_weights=bwd_weights, **(engine_kwargs or {}))
    slices = tensor_slices(net)
    w0 = eng.read_weights()
    assert w0.size == orc.read_weights().size
    # same initial weights (both sides implement the same counter-based generator)
    assert np.abs(w0.astype(np.float64) - orc.read_weights()).max() <= 1e-7
    worst = (0.0, 0.0, None, -1)
    violations, strict_ticks, checked = [], 0, 0
    for t in range(K):
        i = t % len(ys)
        orc.tick(xs[i], ys[i])
        for o2 in orcs:
            o2.tick(xs[i], ys[i])
        eng.tick(xs[i], ys[i])
        if (t + 1) % every == 0 or t == K - 1:
            ref = orc.read_weights()
            e_inf, e_l2, where = rel_errors(eng.read_weights(), ref, slices)
            s_inf = max(max(rel_errors(o2.read_weights(), ref, slices)[:2]) for o2 in orcs)
            tol = TOL if s_inf <= WELL_CONDITIONED else max(TOL, SENS_FACTOR * s_inf)
            checked += 1
            strict_ticks += tol == TOL
            if verbose:
                print(f"tick {t}: inf {e_inf:.2e} l2 {e_l2:.2e} at {where} (oracle sens {s_inf:.1e})", flush=True)
            if max(e_inf, e_l2) > tol:
                violations.append((t, e_inf, e_l2, where, tol))
            if e_inf > worst[0]:
                worst = (e_inf, max(e_l2, worst[1]), where, t)
    med = median_rel_error(eng.read_weights(), orc.read_weights(), slices)
    lg, lo = eng.loss_history(), orc.loss_history()
    ev, ov = eng.read_velocity(), orc.read_velocity()
    l_sens = max(np.abs(o2.loss_history() - lo).max() for o2 in orcs) if len(lo) else 0.0
    v_sens = max(np.abs(o2.read_velocity() - ov).max() for o2 in orcs) / np.abs(ov).max()
    v_err = np.abs(ev - ov).max() / np.abs(ov).max()
    eng.close()
    return dict(worst_inf=worst[0], worst_l2=worst[1], where=worst[2], tick=worst[3],
                violations=violations, strict_ticks=strict_ticks, checked=checked, median_final=med,
                loss_gpu=lg, loss_cpu=lo, loss_tol=max(1e-4, SENS_FACTOR * l_sens), v_err=v_err, v_tol=max(10 * TOL, SENS_FACTOR * v_sens))
