"""HIP engine vs CPU oracle, element by element, through the C ABI."""
import sys

import numpy as np
import pytest

import pb_workloads as W
from tests.parity_util import TOL, run_parity

pytestmark = pytest.mark.gpu


def _engine():
    from paper_2003_11666_amd import PBEngine
    return PBEngine


def _check(res, K, S):
    print(f"worst inf {res['worst_inf']:.3e} l2 {res['worst_l2']:.3e} at {res['where']} tick {res['tick']}; "
          f"strict 1e-5 tolerance in force on {res['strict_ticks']}/{res['checked']} checked ticks",
          file=sys.stderr, flush=True)
    assert not res["violations"], res["violations"][:3]
    assert len(res["loss_gpu"]) == len(res["loss_cpu"]) == max(0, K - S + 1)
    assert np.allclose(res["loss_gpu"], res["loss_cpu"], rtol=1e-4, atol=1e-5)
    assert res["v_err"] <= res["v_tol"], (res["v_err"], res["v_tol"])


@pytest.mark.parametrize("name", ["tiny_mlp", "tiny_vgg", "tiny_resnet", "small_resnet"])
@pytest.mark.parametrize("mit", [3, 0])
def test_small_nets_100_ticks(name, mit):
    net = W.config(name)
    K = 100
    res = run_parity(_engine(), net, K, mitigation=mit)
    _check(res, K, len(net["stages"]))


@pytest.mark.parametrize("mit", [1, 2])
def test_single_mitigations(mit):
    net = W.config("tiny_resnet")
    res = run_parity(_engine(), net, 60, mitigation=mit)
    _check(res, 60, len(net["stages"]))


def test_per_step_launch_mode_is_bit_identical():
    """One launch per phase and one launch per step run the same arithmetic."""
    PBEngine = _engine()
    net = W.config("small_resnet")
    xs, ys = W.sample_pool(net)
    outs = []
    for mode in (0, 1):
        e = PBEngine(net)
        e.set_launch_mode(mode)
        for t in range(40):
            e.tick(xs[t % len(ys)], ys[t % len(ys)])
        outs.append((e.read_weights(), e.loss_history()))
        e.close()
    assert np.array_equal(outs[0][0], outs[1][0])
    assert np.array_equal(outs[0][1], outs[1][1])


def test_resident_pool_equals_host_ticks():
    import torch
    PBEngine = _engine()
    net = W.config("small_resnet")
    xs, ys = W.sample_pool(net)
    a = PBEngine(net)
    for t in range(50):
        a.tick(xs[t % len(ys)], ys[t % len(ys)])
    b = PBEngine(net)
    xd, yd = torch.from_numpy(xs).cuda(), torch.from_numpy(ys).cuda()
    b.run_resident(xd, yd, 0, 20)
    b.run_resident(xd, yd, 20, 30)
    assert np.array_equal(a.read_weights(), b.read_weights())
    assert np.array_equal(a.loss_history(), b.loss_history())
    a.close(); b.close()


def test_mlp_config_100_ticks():
    net = W.config("mlp")
    res = run_parity(_engine(), net, 100)
    _check(res, 100, len(net["stages"]))


def test_resnet20_config_100_ticks():
    net = W.config("resnet20")
    res = run_parity(_engine(), net, 100, every=5)
    _check(res, 100, len(net["stages"]))
