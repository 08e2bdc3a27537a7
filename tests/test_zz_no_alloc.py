"""pb_init_static (the entry point that allocates nothing: the arena is a device array inside the
library) against pb_init, through the C ABI: same kernels, same arithmetic, so weights, velocities and
losses must be bit-identical -- on two calls in a row, the second on a smaller network, which finds
the array full of the first one's data."""
import ctypes as C

import numpy as np
import pytest

import pb_workloads as W

pytestmark = pytest.mark.gpu


def _run(net, K, static):
    import torch
    from paper_2003_11666_amd import PBEngine
    xs, ys = W.sample_pool(net)
    e = PBEngine(net, static_arena=static)
    for t in range(K // 2):
        e.tick(xs[t % len(ys)], ys[t % len(ys)])
    xd, yd = torch.from_numpy(xs).cuda(), torch.from_numpy(ys).cuda()
    e.run_resident(xd, yd, K // 2, K - K // 2)
    out = (e.read_weights(), e.read_velocity(), e.loss_history())
    e.close()
    return out


def test_static_arena_matches_pb_init_twice_in_a_row():
    for name, K in (("small_resnet", 60), ("tiny_resnet", 40)):     # the second network is the smaller one
        net = W.config(name)
        ref = _run(net, K, static=False)
        got = _run(net, K, static=True)
        assert len(ref[2]) == K - len(net["stages"]) + 1
        for a, b in zip(got, ref):
            assert np.array_equal(a, b), name
        assert np.all(np.isfinite(got[0]))


def test_static_arena_limits():
    from paper_2003_11666_amd import PBEngine
    from paper_2003_11666_amd.binding import PBError, load_library
    lib = load_library()
    assert lib.pb_static_arena_bytes() == 64 << 20
    with pytest.raises(PBError, match="static arena holds"):
        PBEngine(W.config("vgg11"), static_arena=True)             # 193 MiB do not fit
    a = PBEngine(W.config("tiny_resnet"), static_arena=True)
    with pytest.raises(PBError, match="held by another context"):
        PBEngine(W.config("tiny_mlp"), static_arena=True)          # one context per GPU at a time
    a.close()
    b = PBEngine(W.config("tiny_mlp"), static_arena=True)          # released by the destroy
    b.close()
    # the headline configuration fits
    c = PBEngine(W.config("resnet20"), static_arena=True)
    c.close()
