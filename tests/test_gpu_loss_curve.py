"""Loss-curve agreement of the HIP path with the CPU oracle over 10 000 ticks (5 000 for the wide network).

The oracle's window means are stored under tests/golden/ (written by
tests/golden/make_loss_curves.py, which runs the oracle only).  Individual
weights of the two trajectories drift apart over thousands of ticks (fp32 vs
fp64, ReLU ties), the training loss as a curve does not: every window mean
must agree within 2 % or 0.02, whichever is larger.
"""
import os

import numpy as np
import pytest

import pb_workloads as W

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _read(name):
    ticks = win = pool = None
    vals = []
    with open(os.path.join(GOLDEN, f"loss_curve_{name}.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("ticks"):
                ticks = int(line.split()[1])
            elif line.startswith("window"):
                win = int(line.split()[1])
            elif line.startswith("pool"):
                pool = int(line.split()[1])
            else:
                vals.append(float(line))
    return ticks, win, pool, np.asarray(vals)


@pytest.mark.parametrize("name", ["mlp", "tiny_vgg", "small_resnet", "resnet20", "vgg11", "wide"])
def test_loss_curve_matches_oracle(name):
    import torch
    from paper_2003_11666_amd import PBEngine
    ticks, win, pool, ref = _read(name)
    net = W.config(name)
    xs, ys = W.sample_pool(net, n=pool)
    dev = torch.device("cuda:0")
    xd, yd = torch.from_numpy(xs).to(dev), torch.from_numpy(ys).to(dev)
    eng = PBEngine(net, mitigation=3)
    eng.run_resident(xd, yd, 0, ticks)
    loss = np.asarray(eng.loss_history(), dtype=np.float64)
    eng.close()
    S = len(net["stages"])
    assert len(loss) == ticks - S + 1
    means = loss[: len(ref) * win].reshape(len(ref), win).mean(axis=1)
    err = np.abs(means - ref)
    tol = np.maximum(0.02, 0.02 * np.abs(ref))
    worst = int(np.argmax(err / tol))
    print(f"{name}: {len(ref)} windows of {win}; worst window {worst}: gpu {means[worst]:.5f} oracle {ref[worst]:.5f}; "
          f"first-window difference {err[0]:.2e}")
    assert np.all(np.isfinite(means))
    assert np.all(err <= tol), (worst, means[worst], ref[worst])
