"""Pins of the CPU oracle against what the paper and the mathematics fix.
None of these tests touches the GPU path."""
import math

import numpy as np
import pytest
import torch

import pb_workloads as W
from oracle import pb_oracle as O
from tests import torch_ref as R

torch.set_num_threads(4)


# ---------------------------------------------------------------- generator
def test_splitmix64_first_output_of_zero_state():
    # widely published first output of splitmix64 started from state 0
    z = O._mix64(np.array([0], dtype=np.uint64) + O._GOLD)
    assert int(z[0]) == 0xE220A8397B1DCDAF


def test_gauss_tensor_is_standard_normal_and_counter_based():
    from scipy import stats
    g = O.gauss_tensor(42, 3, 200000)
    assert abs(g.mean()) < 0.01 and abs(g.std() - 1.0) < 0.01
    assert stats.kstest(g, "norm").pvalue > 1e-3
    # element e does not depend on how many elements are drawn
    assert np.array_equal(O.gauss_tensor(42, 3, 10), g[:10])
    # different tensors / seeds decorrelate
    h = O.gauss_tensor(42, 4, 200000)
    assert abs(np.corrcoef(g, h)[0, 1]) < 0.01


def test_init_is_kaiming_normal_and_fp32_representable():
    net = W.config("resnet20")
    ps = O.init_params(net, 42)
    w = ps[5]["w"]
    fan_in = w.shape[1] * 9
    assert abs(float(w.std()) - math.sqrt(2.0 / fan_in)) < 0.05 * math.sqrt(2.0 / fan_in)
    assert torch.equal(w, w.float().double())
    assert torch.all(ps[5]["gamma"] == 1) and torch.all(ps[5]["beta"] == 0)
    assert sum(O.stage_sizes(net)) == 272282
    assert sum(O.stage_sizes(W.config("mlp"))) == 42634
    assert sum(O.stage_sizes(W.config("vgg11"))) == 9228362


# ------------------------------------------------------- optimizer closed forms
def test_sc_coefficients_definition_and_edges():
    a, b = O.sc_coefficients(0.9, 5)
    assert a == pytest.approx(0.9 ** 5) and b == pytest.approx(sum(0.9 ** k for k in range(5)))
    assert O.sc_coefficients(0.9, 0) == (1.0, 0.0)       # D=0: SGDM (Section "Spike Compensation")
    assert O.sc_coefficients(0.0, 0) == (1.0, 0.0)
    assert O.sc_coefficients(0.0, 3) == (0.0, 1.0)
    assert O.sc_coefficients(1.0, 4) == (1.0, 4.0)


def test_sc_delay_one_is_nesterov():
    # caption of the root heat-map figure: for a delay of one, Nesterov
    # momentum is equivalent to Spike Compensation
    torch.manual_seed(0)
    m, lr = 0.8, 0.03
    gs = torch.randn(25, 7, dtype=torch.float64)
    p = torch.zeros(7, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=lr, momentum=m, nesterov=True)
    w, v = torch.zeros(7, dtype=torch.float64), torch.zeros(7, dtype=torch.float64)
    a, b = O.sc_coefficients(m, 1)
    for g in gs:
        p.grad = g.clone()
        opt.step()
        w, v = O.gsc_update(w, v, g, lr, m, a, b)
        assert torch.allclose(w, p.detach(), rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("D", [0, 1, 4, 9])
def test_sc_impulse_response(D):
    # one gradient at step 0: immediate displacement -lr(a+b)g, then the
    # no-delay response shifted by D; total -lr g/(1-m) for every D
    m, lr, g = 0.9, 0.1, 2.0
    a, b = O.sc_coefficients(m, D)
    w, v = 0.0, 0.0
    disp = []
    for k in range(400):
        w_new, v = O.gsc_update(w, v, g if k == 0 else 0.0, lr, m, a, b)
        disp.append(w_new - w)
        w = w_new
    assert disp[0] == pytest.approx(-lr * g * sum(m ** t for t in range(D + 1)))
    for k in range(1, 20):
        assert disp[k] == pytest.approx(-lr * g * m ** (D + k))
    assert w == pytest.approx(-lr * g / (1 - m), rel=1e-10)


def test_lwp_exact_for_constant_velocity():
    # T = D corresponds to g_hat = (1-m) v, i.e. a constant velocity; then the
    # prediction equals the weights D steps ahead
    m, lr, D = 0.9, 0.05, 7
    v0 = torch.tensor([0.3, -1.2, 2.0], dtype=torch.float64)
    w = torch.tensor([1.0, 2.0, 3.0], dtype=torch.float64)
    pred = O.lwp_predict(w, v0, lr, D)
    v = v0.clone()
    for _ in range(D):
        w, v = O.gsc_update(w, v, (1 - m) * v, lr, m, 1.0, 0.0)
    assert torch.allclose(v, v0) and torch.allclose(w, pred, rtol=1e-13)


def _poly(kind, D, m, el, a, b, T):
    """Characteristic polynomial coefficients, highest power first (Section
    "Analysis for a Convex Quadratic"); el = lr*lambda.  The constant term of
    the GDM polynomial is +el (sign as derived from the SGDM state-transition
    equation of the appendix)."""
    if kind == "gdm":
        c = np.zeros(D + 2)
        c[0], c[1], c[2] = 1.0, -(1 + m), m
        c[-1] += el
        return c
    if kind in ("gsc", "lwp"):
        if kind == "lwp":
            a, b = 1.0, 0.0
            lin, const = el * (1 + T), -el * T
        else:
            lin, const = el * (a + b), -el * m * b
        c = np.zeros(D + 3)
        c[0], c[1], c[2] = 1.0, -(1 + m), m
        c[-2] += lin
        c[-1] += const
        return c
    if kind == "cmb":
        c = np.zeros(D + 4)
        c[0], c[1], c[2] = 1.0, -(1 + m), m
        c[-3] += el * (a + b) * (T + 1)
        c[-2] += -el * ((T + 1) * m * b + T * (a + b))
        c[-1] += el * T * m * b
        return c
    raise KeyError(kind)


@pytest.mark.parametrize("kind,D", [("gdm", 1), ("gdm", 3), ("gsc", 1), ("gsc", 4), ("lwp", 1),
                                    ("lwp", 5), ("cmb", 1), ("cmb", 3)])
def test_scalar_quadratic_follows_characteristic_polynomial(kind, D):
    m, lr, lam = 0.8, 0.02, 1.7
    a, b = O.sc_coefficients(m, D) if kind in ("gsc", "cmb") else (1.0, 0.0)
    T = float(D) if kind in ("lwp", "cmb") else 0.0
    phi = O.scalar_quadratic_run(lam, lr, m, D, a, b, T, 400, w_form=(kind == "cmb"))
    c = _poly(kind, D, m, lr * lam, a, b, T)
    n = len(c) - 1
    # the trajectory satisfies the linear recurrence  sum_j c_j phi_{t+n-j} = 0
    t0 = D + 4
    res = [sum(c[j] * phi[t + n - j] for j in range(n + 1)) for t in range(t0, 380 - n)]
    scale = max(abs(phi[t0:]).max(), 1e-30)
    assert max(abs(r) for r in res) < 1e-12 * scale + 1e-15
    # and decays with the dominant root's modulus
    rmax = max(abs(np.roots(c)))
    assert rmax < 1.0
    tail = np.abs(phi[150:400])
    rate = (tail[200:].max() / tail[:50].max()) ** (1.0 / 200)
    assert rate == pytest.approx(rmax, rel=0.02)


def test_velocity_form_lwp_matches_weight_form_without_sc():
    m, lr, lam, D = 0.9, 0.01, 2.0, 4
    p1 = O.scalar_quadratic_run(lam, lr, m, D, 1.0, 0.0, float(D), 200, w_form=False)
    p2 = O.scalar_quadratic_run(lam, lr, m, D, 1.0, 0.0, float(D), 200, w_form=True)
    assert np.allclose(p1, p2, rtol=1e-12, atol=1e-15)


def test_gsc_equals_lwp_on_linear_gradient():
    # a = 1 - (1-m)T/m, b = T/m gives the same recurrence as LWP with horizon T
    m, lr, lam, D, T = 0.8, 0.02, 1.3, 3, 3.0
    a, b = 1 - (1 - m) * T / m, T / m
    c1 = _poly("gsc", D, m, lr * lam, a, b, 0.0)
    c2 = _poly("lwp", D, m, lr * lam, 1.0, 0.0, T)
    assert np.allclose(c1, c2)
    p_gsc = O.scalar_quadratic_run(lam, lr, m, D, a, b, 0.0, 300)
    n = len(c2) - 1
    res = [sum(c2[j] * p_gsc[t + n - j] for j in range(n + 1)) for t in range(D + 4, 280 - n)]
    assert max(abs(r) for r in res) < 1e-12


# ------------------------------------------------------------- layer math
NETS = ["tiny_mlp", "tiny_vgg", "tiny_resnet", "tiny_bottleneck"]


def _oracle_full_grad(net, params, x, label):
    """Chain the oracle's stage routines with the same weights forward and
    backward: must give the true gradient."""
    stages = net["stages"]
    xs, saved = [], []
    h = torch.as_tensor(x, dtype=O.DT).reshape(net["in_c"], net["in_h"], net["in_w"])
    loss = None
    for s, st in enumerate(stages):
        xs.append(h)
        src = O.skip_source(st)
        h, l, sv = O.stage_forward(st, params[s], h, xs[src] if src >= 0 else None,
                                   label if s == len(stages) - 1 else None)
        saved.append(sv)
        loss = l if l is not None else loss
    dy, skipgrad, grads = None, {}, [None] * len(stages)
    for s in range(len(stages) - 1, -1, -1):
        dx, g, dskip = O.stage_backward(stages[s], params[s], saved[s], dy, need_dx=(s > 0))
        if s > 0 and s in skipgrad:
            dx = dx + skipgrad.pop(s)
        src = O.skip_source(stages[s])
        if src >= 0:
            skipgrad[src] = dskip
        grads[s] = g
        dy = dx
    return float(loss), grads


@pytest.mark.parametrize("name", NETS)
def test_layer_backward_matches_autograd(name):
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    params = R.leaf_params(net, 7)
    # perturb GroupNorm affine so that gamma != 1, beta != 0 are exercised
    g = torch.Generator().manual_seed(1)
    with torch.no_grad():
        for p in params:
            for k in ("gamma", "beta", "b"):
                if k in p:
                    p[k] += 0.3 * torch.randn(p[k].shape, generator=g, dtype=torch.float64)
    loss = R.forward_loss(net, params, xs[0], ys[0])
    loss.backward()
    plain = [{k: t.detach() for k, t in p.items()} for p in params]
    l2, grads = _oracle_full_grad(net, plain, xs[0], int(ys[0]))
    assert l2 == pytest.approx(float(loss), rel=1e-12)
    for s, p in enumerate(params):
        for k, t in p.items():
            assert torch.allclose(grads[s][k], t.grad, rtol=1e-9, atol=1e-12), (s, k)


@pytest.mark.parametrize("name", NETS)
def test_finite_differences(name):
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    params = O.init_params(net, 3)
    g = torch.Generator().manual_seed(2)
    for p in params:
        for k in ("gamma", "beta", "b"):
            if k in p:
                p[k] = p[k] + 0.3 * torch.randn(p[k].shape, generator=g, dtype=torch.float64)
    _, grads = _oracle_full_grad(net, params, xs[1], int(ys[1]))
    rng = np.random.default_rng(0)
    h = 1e-6
    for s, p in enumerate(params):
        for k, t in p.items():
            flat = t.reshape(-1)
            for idx in rng.choice(flat.numel(), size=min(3, flat.numel()), replace=False):
                old = float(flat[idx])
                flat[idx] = old + h
                lp, _ = _oracle_full_grad(net, params, xs[1], int(ys[1]))
                flat[idx] = old - h
                lm, _ = _oracle_full_grad(net, params, xs[1], int(ys[1]))
                flat[idx] = old
                fd = (lp - lm) / (2 * h)
                an = float(grads[s][k].reshape(-1)[idx])
                assert fd == pytest.approx(an, rel=2e-5, abs=2e-7), (s, k, int(idx))


# ----------------------------------------------------- pipeline bookkeeping
@pytest.mark.parametrize("name", NETS)
def test_zero_delay_is_sgdm(name):
    """All delays zero: the algorithm is SGD with momentum (library optimizer
    on an autograd model), and SC / LWP are identity modifications."""
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    n = 12
    params = R.leaf_params(net, 42)
    opt = torch.optim.SGD([t for p in params for t in p.values()], lr=net["lr"],
                          momentum=net["momentum"])
    ref_losses = []
    for i in range(n):
        opt.zero_grad()
        loss = R.forward_loss(net, params, xs[i], ys[i])
        loss.backward()
        opt.step()
        ref_losses.append(float(loss))
    ref = R.flat(params)
    outs = []
    for mit in (0, 1, 2, 3):
        hist, losses = O.run_sample_indexed(net, n, xs, ys, delays=[0] * S, mitigation=mit)
        outs.append(torch.cat([t.reshape(-1) for s in range(S) for t in hist[s][n][0].values()]))
        assert np.allclose(losses, ref_losses, rtol=1e-9)
    assert torch.allclose(outs[0], ref, rtol=1e-8, atol=1e-11)
    for o in outs[1:]:
        assert torch.equal(o, outs[0])


@pytest.mark.parametrize("name", NETS)
@pytest.mark.parametrize("mit", [0, 3])
def test_tick_form_equals_sample_indexed_form(name, mit):
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    K = 4 * S + 5
    orc = O.PBOracle(net, mitigation=mit)
    for t in range(K):
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
    n = K - (S - 1)
    hist, losses = O.run_sample_indexed(net, n, xs, ys, mitigation=mit)
    assert len(orc.losses) == K - S + 1
    assert np.allclose(orc.loss_history(), losses[:K - S + 1], rtol=1e-10)
    for s in range(S):
        k = max(0, K - 2 * (S - 1) + s)
        wv, vv = hist[s][k]
        for name_, t_ in wv.items():
            assert torch.allclose(orc.w[s][name_], t_, rtol=1e-10, atol=1e-13), (s, name_)
            assert torch.allclose(orc.v[s][name_], vv[name_], rtol=1e-10, atol=1e-13)


def test_pipeline_timing():
    """A sample needs 2S-1 time steps; stage s gets its first gradient at tick
    2(S-1)-s; the loss of sample i appears at tick i+S-1."""
    net = W.config("tiny_resnet")
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    orc = O.PBOracle(net)
    w0 = [{k: t.clone() for k, t in p.items()} for p in orc.w]
    first_change = [None] * S
    for t in range(2 * S + 2):
        orc.tick(xs[t], ys[t])
        assert len(orc.losses) == max(0, t + 1 - (S - 1))
        for s in range(S):
            if first_change[s] is None and not torch.equal(orc.w[s]["w"], w0[s]["w"]):
                first_change[s] = t
    assert first_change == [2 * (S - 1) - s for s in range(S)]
    assert first_change[0] + 1 == 2 * S - 1


@pytest.mark.parametrize("name", ["tiny_vgg", "tiny_resnet"])
def test_lr_zero_reproduces_fixed_network(name):
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    orc = O.PBOracle(net, lr=0.0)
    params = R.leaf_params(net, 42)
    K = 2 * S + 3
    seen = {}
    for t in range(K):
        orc.tick(xs[t], ys[t])
        for s in range(S):
            j = t - 2 * (S - 1) + s
            if j >= 0:
                seen[(s, j)] = orc.last_grads[s]
    for i in range(K - S + 1):
        for p in params:
            for t_ in p.values():
                t_.grad = None
        loss = R.forward_loss(net, params, xs[i], ys[i])
        assert orc.losses[i] == pytest.approx(float(loss), rel=1e-12)
        loss.backward()
        for s in range(S):
            if (s, i) in seen:
                for k, t_ in params[s].items():
                    assert torch.allclose(seen[(s, i)][k], t_.grad, rtol=1e-9, atol=1e-12)
    assert np.array_equal(orc.read_weights(), R.flat(params).numpy())


def test_stash_mode_gives_true_gradient_of_forward_weights():
    """Weight stashing: G(x; F, F) is the plain gradient at the forward
    weights (Eq. sgdpb_weight_stash)."""
    net = W.config("tiny_resnet")
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    D = O.natural_delays(S)
    n = 3 * S
    hist, _ = O.run_sample_indexed(net, n, xs, ys, mitigation=2, bwd_weights=1)
    i = n - 1
    F_i = []
    for s in range(S):
        wv, vv = hist[s][max(0, i - D[s])]
        F_i.append({k: O.lwp_predict(wv[k], vv[k], net["lr"], float(D[s])).clone().requires_grad_(True)
                    for k in wv})
    loss = R.forward_loss(net, F_i, xs[i % len(ys)], ys[i % len(ys)])
    loss.backward()
    m, lr = net["momentum"], net["lr"]
    for s in range(S):
        w_prev, v_prev = hist[s][i]
        w_next, v_next = hist[s][i + 1]
        for k in w_prev:
            g = v_next[k] - m * v_prev[k]
            assert torch.allclose(g, F_i[s][k].grad, rtol=1e-8, atol=1e-11)


def test_bf16_rounding_points():
    net = dict(W.config("tiny_bottleneck"))
    net["act_dtype"] = "bf16"
    xs, ys = W.sample_pool(net)
    orc = O.PBOracle(net)
    S = len(net["stages"])
    for t in range(2 * S):
        orc.tick(xs[t], ys[t])
    for s, y in orc.fwd_mail.items():
        assert torch.equal(y, y.float().bfloat16().double())
    for s, g in orc.grad_mail.items():
        assert torch.equal(g, g.float().bfloat16().double())
    assert np.isfinite(orc.loss_history()).all()


# --------------------------------------------------------------------------
# Over-compensation (Section "Combined Mitigation": LWP_2D, SC_2D and their combination)
# --------------------------------------------------------------------------
def test_overcompensation_coefficients_and_forms():
    """The scaled variants are the same update with the coefficients of delay
    scale*D: a = m^(2D), b = (1 - m^(2D))/(1 - m), T = 2D for the doubled forms;
    the tick form and the sample-indexed form agree with them switched on."""
    net = W.config("tiny_resnet")
    S = len(net["stages"])
    m = net["momentum"]
    orc = O.PBOracle(net, mitigation=3, sc_scale=2.0, lwp_scale=2.0)
    for s in range(S):
        D = 2 * (S - 1 - s)
        a, b, T = orc.coef[s]
        assert a == pytest.approx(m ** (2 * D), rel=1e-14)
        assert b == pytest.approx(sum(m ** i for i in range(2 * D)), rel=1e-12)   # geometric sum, Eq. scd
        assert T == 2 * D
    xs, ys = W.sample_pool(net)
    K = 4 * S + 3
    for t in range(K):
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
    hist, losses = O.run_sample_indexed(net, K - (S - 1), xs, ys, mitigation=3, sc_scale=2.0, lwp_scale=2.0)
    assert np.allclose(orc.loss_history(), losses[:K - S + 1], rtol=1e-10)
    plain = O.PBOracle(net, mitigation=3)
    for t in range(K):
        plain.tick(xs[t % len(ys)], ys[t % len(ys)])
    differs = False
    for s in range(S):
        k = max(0, K - 2 * (S - 1) + s)
        for name_, t_ in hist[s][k][0].items():
            assert torch.allclose(orc.w[s][name_], t_, rtol=1e-10, atol=1e-13), (s, name_)
            differs |= not torch.allclose(orc.w[s][name_], plain.w[s][name_], rtol=1e-6, atol=1e-9)
    assert differs


def test_overcompensated_lwp_on_the_quadratic():
    """LWP with horizon T on the scalar quadratic: with constant velocity the
    prediction lands exactly T steps ahead (Eq. lwp_v_form), whatever the delay."""
    lr, m = 0.1, 0.0
    # m = 0, lam = 0 would be static; use the predictor alone: w_t = w_0 - lr*v*t
    w0, v = torch.tensor([1.0, -2.0], dtype=O.DT), torch.tensor([0.3, 0.7], dtype=O.DT)
    for T in (0, 3, 8):
        pred = O.lwp_predict(w0, v, lr, float(T))
        assert torch.allclose(pred, w0 - lr * T * v, rtol=0, atol=1e-15)


# --------------------------------------------------------------------------
# LWP in its weight-difference form (Eq. lwp_w_form)
# --------------------------------------------------------------------------
def test_lwp_weight_form():
    """w_hat = w + T (w - w_prev).  Without Spike Compensation w - w_prev = -lr v, so the form equals
    the velocity form exactly (Section "Linear Weight Prediction"); with SC the two differ; the tick
    form and the sample-indexed form agree on it."""
    net = W.config("tiny_resnet")
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    K = 4 * S + 3
    a, b = O.PBOracle(net, mitigation=2, lwp_form="w"), O.PBOracle(net, mitigation=2)
    c, d = O.PBOracle(net, mitigation=3, lwp_form="w"), O.PBOracle(net, mitigation=3)
    for t in range(K):
        for o in (a, b, c, d):
            o.tick(xs[t % len(ys)], ys[t % len(ys)])
    assert np.abs(a.read_weights() - b.read_weights()).max() <= 1e-13
    assert np.abs(c.read_weights() - d.read_weights()).max() > 1e-4
    hist, losses = O.run_sample_indexed(net, K - (S - 1), xs, ys, mitigation=3, lwp_form="w")
    assert np.allclose(c.loss_history(), losses[:K - S + 1], rtol=1e-10)
    for s in range(S):
        k = max(0, K - 2 * (S - 1) + s)
        for name_, t_ in hist[s][k][0].items():
            assert torch.allclose(c.w[s][name_], t_, rtol=1e-10, atol=1e-13), (s, name_)


# ---- hyper-parameter scaling with the update size (Appendix "Small Batch Size Training", Eq. hpscale)
@pytest.mark.parametrize("lr_r,m_r,n_r,n", [(0.1, 0.9, 128, 1), (0.1, 0.9, 32, 1), (0.05, 0.95, 64, 8),
                                            (0.2, 0.5, 4, 16), (0.1, 0.0, 8, 1)])
def test_hyperparameter_scaling_invariants(lr_r, m_r, n_r, n):
    """What the appendix states in words: the momentum's decay per SAMPLE is unchanged, and the
    effective learning rate lr/(1-m) is proportional to the update size."""
    lr, m = O.scale_hyperparameters(lr_r, m_r, n_r, n)
    assert m ** (1.0 / n) == pytest.approx(m_r ** (1.0 / n_r), rel=1e-12, abs=1e-300)
    assert lr / (1.0 - m) / n == pytest.approx(lr_r / (1.0 - m_r) / n_r, rel=1e-12)
    # identity at the reference size, and scaling in two hops equals scaling in one
    assert O.scale_hyperparameters(lr_r, m_r, n_r, n_r) == pytest.approx((lr_r, m_r), rel=1e-15)
    lr1, m1 = O.scale_hyperparameters(lr_r, m_r, n_r, 4)
    assert O.scale_hyperparameters(lr1, m1, 4, n) == pytest.approx((lr, m), rel=1e-12)


def test_hyperparameter_scaling_keeps_the_trajectory_of_a_constant_gradient():
    """Plain momentum SGD (the update routine with a = 1, b = 0) on a stream of samples that all
    have gradient 1: with update size 128 (mean gradient per update) and with update size 1 at the
    scaled values, the weight has moved by the same amount after the same number of samples --
    total contribution per sample lr/((1-m) n) and decay per sample m^(1/n) are both kept."""
    lr_r, m_r, n_r = 0.1, 0.9, 128
    lr, m = O.scale_hyperparameters(lr_r, m_r, n_r, 1)
    n_samples = n_r * 400
    w_r = v_r = 0.0
    for _ in range(n_samples // n_r):
        w_r, v_r = O.gsc_update(w_r, v_r, 1.0, lr_r, m_r, 1.0, 0.0)
    w = v = 0.0
    for _ in range(n_samples):
        w, v = O.gsc_update(w, v, 1.0, lr, m, 1.0, 0.0)
    assert w == pytest.approx(w_r, rel=5e-3)
    # a swapped ratio (n_ref/n instead of n/n_ref) would be off by orders of magnitude
    assert abs(w) > 1.0


def test_hyperparameter_scaling_limit_of_unit_momentum():
    lr, m = O.scale_hyperparameters(0.1, 1.0, 8, 2)
    lr_near, m_near = O.scale_hyperparameters(0.1, 1.0 - 1e-9, 8, 2)
    assert m == 1.0 and lr == pytest.approx(lr_near, rel=1e-6)
