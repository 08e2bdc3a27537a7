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


# --------------------------------------------------------------------------
# The analysis of the convex quadratic, driven through the oracle's own
# per-sample pipeline routine (delay bookkeeping, coefficients, prediction,
# update) instead of a scalar helper
# --------------------------------------------------------------------------
@pytest.mark.parametrize("kind,D", [("gdm", 1), ("gdm", 3), ("gsc", 1), ("gsc", 4), ("lwp", 2), ("lwp", 5),
                                    ("cmb", 1), ("cmb", 3)])
def test_sample_indexed_pipeline_on_a_quadratic_follows_characteristic_polynomial(kind, D, monkeypatch):
    """run_sample_indexed with a one-stage "network" whose layer math is replaced by the scalar
    quadratic loss lam/2 phi^2 (forward gradient lam * phi_hat, phi_hat the predicted weight the
    forward pass was handed): the weight history it keeps must satisfy the linear recurrence whose
    characteristic polynomial the paper prints for that method (Section "Analysis for a Convex
    Quadratic": plain delayed momentum, SC_D, LWP_D, LWP^w_D + SC_D).  A wrong version index in the
    forward pass, a prediction from the wrong velocity, swapped a / b or a wrong horizon all break
    the recurrence."""
    lam = 1.7
    m, lr = 0.8, 0.02

    def fwd(stage, P, x, skip_x, label, bf16=False, relu_shift=0.0):
        phi_hat = P["w"].reshape(())
        return None, 0.5 * lam * phi_hat * phi_hat, [dict(phi=phi_hat)]

    def bwd(stage, Wb, saved, dy, need_dx=True, bf16=False):
        return None, {"w": (lam * saved[0]["phi"]).reshape(1, 1)}, None

    monkeypatch.setattr(O, "stage_forward", fwd)
    monkeypatch.setattr(O, "stage_backward", bwd)
    net = dict(name="quad", stages=[[W.linear(1, 1, bias=0), W.ce()]], in_c=1, in_h=1, in_w=1, n_classes=1,
               lr=lr, momentum=m, n_pool=1, seed_data=1, ticks=0, act_dtype="fp32")
    mit = {"gdm": 0, "gsc": 1, "lwp": 2, "cmb": 3}[kind]
    n = 400
    hist, _ = O.run_sample_indexed(net, n, np.zeros((1, 1, 1, 1), np.float32), np.zeros(1, np.int32), delays=[D],
                                   mitigation=mit, lwp_form="w" if kind == "cmb" else "v")
    phi = np.array([float(hist[0][k][0]["w"]) for k in range(n + 1)])
    assert phi[0] != 0.0
    a, b = O.sc_coefficients(m, D) if kind in ("gsc", "cmb") else (1.0, 0.0)
    T = float(D) if kind in ("lwp", "cmb") else 0.0
    c = _poly(kind, D, m, lr * lam, a, b, T)
    nn = len(c) - 1
    t0 = D + 4
    res = [sum(c[j] * phi[t + nn - j] for j in range(nn + 1)) for t in range(t0, 380 - nn)]
    assert max(abs(r) for r in res) < 1e-12 * abs(phi[t0:]).max() + 1e-15
    # and the helper on the same problem gives the same trajectory
    ref = O.scalar_quadratic_run(lam, lr, m, D, a, b, T, n, w_form=(kind == "cmb"), phi0=phi[0])
    assert np.allclose(phi, ref, rtol=1e-12, atol=1e-15)


# --------------------------------------------------------------------------
# Layer routines against plain loops written from the definitions
# --------------------------------------------------------------------------
def _naive_conv(x, w, b, stride, pad):
    C, H, Wd = x.shape
    K, _, k, _ = w.shape
    OH, OW = (H + 2 * pad - k) // stride + 1, (Wd + 2 * pad - k) // stride + 1
    y = np.zeros((K, OH, OW))
    for co in range(K):
        for oh in range(OH):
            for ow in range(OW):
                acc = 0.0 if b is None else b[co]
                for ci in range(C):
                    for kh in range(k):
                        for kw in range(k):
                            ih, iw = oh * stride - pad + kh, ow * stride - pad + kw
                            if 0 <= ih < H and 0 <= iw < Wd:
                                acc += w[co, ci, kh, kw] * x[ci, ih, iw]
                y[co, oh, ow] = acc
    return y


@pytest.mark.parametrize("C,H,Wd,K,k,stride,pad", [(3, 7, 6, 4, 3, 2, 1), (2, 5, 5, 3, 1, 2, 0), (2, 6, 7, 2, 3, 1, 1),
                                                  (1, 9, 8, 2, 5, 2, 2)])
def test_conv_routines_against_plain_loops(C, H, Wd, K, k, stride, pad):
    rng = np.random.default_rng(5)
    x, w, b = rng.standard_normal((C, H, Wd)), rng.standard_normal((K, C, k, k)), rng.standard_normal(K)
    y = O.conv_forward(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), stride, pad).numpy()
    y_ref = _naive_conv(x, w, b, stride, pad)
    assert y.shape == y_ref.shape and np.allclose(y, y_ref, rtol=1e-12, atol=1e-12)
    # backward: dW[co,ci,kh,kw] = sum dy[co,oh,ow] x[ci,oh*s-p+kh,ow*s-p+kw]; dX = the transposed map
    dy = rng.standard_normal(y_ref.shape)
    dx, dw = O.conv_backward(torch.from_numpy(dy), torch.from_numpy(x), torch.from_numpy(w), stride, pad)
    dw_ref, dx_ref = np.zeros_like(w), np.zeros_like(x)
    OH, OW = y_ref.shape[1:]
    for co in range(K):
        for oh in range(OH):
            for ow in range(OW):
                for ci in range(C):
                    for kh in range(k):
                        for kw in range(k):
                            ih, iw = oh * stride - pad + kh, ow * stride - pad + kw
                            if 0 <= ih < H and 0 <= iw < Wd:
                                dw_ref[co, ci, kh, kw] += dy[co, oh, ow] * x[ci, ih, iw]
                                dx_ref[ci, ih, iw] += dy[co, oh, ow] * w[co, ci, kh, kw]
    assert np.allclose(dw.numpy(), dw_ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(dx.numpy(), dx_ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k,stride,pad,H,Wd", [(2, 2, 0, 6, 6), (3, 2, 1, 7, 8), (3, 2, 1, 5, 5)])
def test_maxpool_forward_and_gradient_routing_against_plain_loops(k, stride, pad, H, Wd):
    """Through the oracle's stage routines: the pooled value is the window maximum and the gradient
    goes to the FIRST maximum in row-major window order (ties are planted: post-ReLU zeros and
    repeated values)."""
    rng = np.random.default_rng(9)
    C = 3
    x = np.round(rng.standard_normal((C, H, Wd)) * 2) / 2      # many repeated values
    x[x < 0] = 0.0                                              # as after a ReLU
    # a 1x1 convolution with identity weights in front, so that the stage has its weight layer and the
    # oracle's own backward routine routes the gradient
    stage = [W.conv(C, C, 1, 1, 0), W.maxpool(k, stride, pad)]
    Wid = {"w": torch.eye(C, dtype=O.DT).reshape(C, C, 1, 1)}
    y, _, saved = O.stage_forward(stage, Wid, torch.from_numpy(x), None, None)
    PH, PW = (H + 2 * pad - k) // stride + 1, (Wd + 2 * pad - k) // stride + 1
    dy = rng.standard_normal((C, PH, PW))
    y_ref, dx_ref = np.zeros((C, PH, PW)), np.zeros_like(x)
    for c in range(C):
        for ph in range(PH):
            for pw in range(PW):
                best, arg = -np.inf, None
                for kh in range(k):
                    for kw in range(k):
                        ih, iw = ph * stride - pad + kh, pw * stride - pad + kw
                        if 0 <= ih < H and 0 <= iw < Wd and x[c, ih, iw] > best:
                            best, arg = x[c, ih, iw], (ih, iw)
                y_ref[c, ph, pw] = best
                dx_ref[c, arg[0], arg[1]] += dy[c, ph, pw]
    assert np.array_equal(y.numpy(), y_ref)
    dx, _, _ = O.stage_backward(stage, Wid, saved, torch.from_numpy(dy), need_dx=True)
    assert np.array_equal(dx.numpy(), dx_ref)


def test_groupnorm_and_cross_entropy_against_plain_loops():
    rng = np.random.default_rng(11)
    C, H, Wd, G = 6, 3, 4, 3
    x, gamma, beta = rng.standard_normal((C, H, Wd)), rng.standard_normal(C), rng.standard_normal(C)
    y, sv = O.gn_forward(torch.from_numpy(x), torch.from_numpy(gamma), torch.from_numpy(beta), G)
    cpg = C // G
    y_ref = np.zeros_like(x)
    for g in range(G):
        blk = x[g * cpg:(g + 1) * cpg]
        n = blk.size
        mean = sum(blk.reshape(-1)) / n
        var = sum((v - mean) ** 2 for v in blk.reshape(-1)) / n       # biased
        for c in range(g * cpg, (g + 1) * cpg):
            y_ref[c] = (x[c] - mean) / math.sqrt(var + 1e-5) * gamma[c] + beta[c]
    assert np.allclose(y.numpy(), y_ref, rtol=1e-12, atol=1e-12)
    z = rng.standard_normal(7)
    loss, dz = O.softmax_ce(torch.from_numpy(z), 4)
    p = np.exp(z) / np.exp(z).sum()
    assert float(loss) == pytest.approx(-math.log(p[4]), rel=1e-12)
    onehot = np.zeros(7); onehot[4] = 1.0
    assert np.allclose(dz.numpy(), p - onehot, rtol=1e-12, atol=1e-15)


# --------------------------------------------------------------------------
# bf16 activation mode: the rounding itself and the places it is applied
# --------------------------------------------------------------------------
def _bf16_rne_bits(x32):
    """Round-to-nearest-even to bfloat16 by integer arithmetic on the float32 bit pattern."""
    u = np.asarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return ((u & 0xFFFF0000).astype(np.uint32)).view(np.float32)


def test_round_bf16_fixed_vectors():
    # 1 + 2^-8 lies exactly between 1 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 lies between 1 + 2^-7 (odd) and 1 + 2^-6 (even): goes up.  Truncation gets the
    # second and fourth wrong, round-half-up the first.
    cases = [(1.0 + 2.0 ** -8, 1.0), (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6), (-(1.0 + 2.0 ** -8), -1.0),
             (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7), (1.0 + 2.0 ** -7, 1.0 + 2.0 ** -7),
             (3.0e-3, float(_bf16_rne_bits([3.0e-3])[0])), (0.0, 0.0), (-2.5, -2.5),
             (255.0 + 0.5, 256.0), (1.0 - 2.0 ** -9, 1.0)]
    for x, want in cases:
        got = float(O._round_bf16(torch.tensor([x], dtype=O.DT))[0])
        assert got == want, (x, got, want)
    rng = np.random.default_rng(3)
    v = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    got = O._round_bf16(torch.from_numpy(v.astype(np.float64))).numpy()
    assert np.array_equal(got.astype(np.float32), _bf16_rne_bits(v))
    # a float64 value is first taken to float32 (what the library holds), then to bf16
    assert float(O._round_bf16(torch.tensor([1.0 + 2.0 ** -8 + 2.0 ** -40], dtype=O.DT))[0]) == 1.0


def _is_bf16(t):
    return torch.equal(t, t.float().bfloat16().double())


def test_bf16_rounding_sites_of_one_tick():
    """Every tensor that crosses a stage boundary or is kept for the backward pass is bf16 (network
    input, a conv output that feeds a GroupNorm of its own stage, stage outputs, every dX and skip
    gradient) and equals the nearest-even rounding of what the fp32-activation computation gives
    from the same inputs; statistics, normalised values, gradients, weights and velocities are not
    rounded."""
    net = dict(W.config("tiny_bottleneck"))
    net["act_dtype"] = "bf16"
    stages = net["stages"]
    S = len(stages)
    xs, ys = W.sample_pool(net)
    orc = O.PBOracle(net)
    for t in range(2 * S + 1):
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
    # state kept for the backward pass
    for s in range(S):
        for i, entry in orc.saved[s].items():
            assert _is_bf16(entry["x_in"]), (s, "stage input")
            for op, sv in zip(stages[s], entry["ops"]):
                if op["kind"] == "conv":
                    assert _is_bf16(sv["x"]) or any(o["kind"] == "gn" for o in stages[s][:stages[s].index(op)])
                if op["kind"] == "gn":
                    assert not _is_bf16(sv["xh"]) and not _is_bf16(sv["rstd"])
    for s, y in orc.fwd_mail.items():
        assert _is_bf16(y)
    for s, g in orc.grad_mail.items():
        assert _is_bf16(g)
    for s in range(S):
        for d in orc.skipgrad[s].values():
            assert _is_bf16(d)
    assert any(len(d) for d in orc.skipgrad)
    for s in range(S):
        for k in orc.w[s]:
            assert not _is_bf16(orc.last_grads[s][k]) or orc.last_grads[s][k].numel() < 3, (s, k)
        assert not _is_bf16(orc.w[s]["w"]) and not _is_bf16(orc.v[s]["w"])
    # values: stage forward in bf16 mode = rounding of the fp32-mode result at exactly the listed places
    x0 = O._round_bf16(torch.as_tensor(xs[0], dtype=O.DT))
    assert np.array_equal(x0.numpy().astype(np.float32), _bf16_rne_bits(xs[0]))
    P = orc.predicted(0)
    y_b, _, sv_b = O.stage_forward(stages[0], P, x0, None, None, bf16=True)      # conv, gn, relu, maxpool
    z = O.conv_forward(x0, P["w"], None, stages[0][0]["stride"], stages[0][0]["pad"])
    z_r = torch.from_numpy(_bf16_rne_bits(z.numpy().astype(np.float32)).astype(np.float64))
    rest, _, _ = O.stage_forward(stages[0][1:], P, z_r, None, None, bf16=False)
    want = _bf16_rne_bits(rest.numpy().astype(np.float32)).astype(np.float64)
    assert np.array_equal(y_b.numpy(), want)
    # a pre-norm stage: only the stage output is rounded
    P1 = orc.predicted(1)
    y1_b, _, _ = O.stage_forward(stages[1], P1, y_b, None, None, bf16=True)
    y1_f, _, sv1 = O.stage_forward(stages[1], P1, y_b, None, None, bf16=False)
    assert np.array_equal(y1_b.numpy(), _bf16_rne_bits(y1_f.numpy().astype(np.float32)).astype(np.float64))
    assert not _is_bf16(y1_f)
    # backward of that stage: the caller rounds dX, the stage routine itself leaves it alone
    dy = O._round_bf16(torch.randn(y1_f.shape, dtype=O.DT, generator=torch.Generator().manual_seed(4)))
    dx, grads, _ = O.stage_backward(stages[1], orc.w[1], sv1, dy, need_dx=True, bf16=True)
    assert not _is_bf16(dx) and not _is_bf16(grads["w"])


# --------------------------------------------------------------------------
# Update size above one (Appendix "Small Batch Size Training")
# --------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["tiny_mlp", "tiny_resnet"])
def test_update_size_one_is_the_default_path(name):
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    a, b = O.PBOracle(net), O.PBOracle(net, update_size=1)
    for t in range(40):
        a.tick(xs[t % len(ys)], ys[t % len(ys)])
        b.tick(xs[t % len(ys)], ys[t % len(ys)])
    assert np.array_equal(a.read_weights(), b.read_weights()) and np.array_equal(a.loss_history(), b.loss_history())


@pytest.mark.parametrize("name", NETS)
@pytest.mark.parametrize("N", [2, 3])
def test_zero_delay_with_update_size_n_is_minibatch_sgdm(name, N):
    """All delays zero and update size N: plain minibatch SGD with momentum on the mean loss of N
    samples (a library optimizer on an autograd model; the networks normalise per sample, so a batch
    is N independent samples), whatever the mitigation."""
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    n_upd = 5
    params = R.leaf_params(net, 42)
    opt = torch.optim.SGD([t for p in params for t in p.values()], lr=net["lr"], momentum=net["momentum"])
    for u in range(n_upd):
        opt.zero_grad()
        loss = sum(R.forward_loss(net, params, xs[u * N + j], ys[u * N + j]) for j in range(N)) / N
        loss.backward()
        opt.step()
    ref = R.flat(params)
    for mit in (0, 3):
        hist, _ = O.run_sample_indexed(net, n_upd * N, xs, ys, delays=[0] * S, mitigation=mit, update_size=N)
        assert all(len(hist[s]) == n_upd + 1 for s in range(S))
        got = torch.cat([t.reshape(-1) for s in range(S) for t in hist[s][n_upd][0].values()])
        assert torch.allclose(got, ref, rtol=1e-8, atol=1e-11)


@pytest.mark.parametrize("name", ["tiny_vgg", "tiny_resnet", "tiny_bottleneck"])
@pytest.mark.parametrize("N,mit", [(2, 3), (3, 3), (4, 0), (3, 1)])
def test_update_size_tick_form_equals_sample_indexed_form(name, N, mit):
    """Two independent book-keepings of the same rule: gradients added up per stage across ticks with
    an update every N-th backward pass, against versions indexed by floor(i / N)."""
    net = W.config(name)
    xs, ys = W.sample_pool(net)
    S = len(net["stages"])
    K = 5 * S + 7
    orc = O.PBOracle(net, mitigation=mit, update_size=N)
    for t in range(K):
        orc.tick(xs[t % len(ys)], ys[t % len(ys)])
    n = K - (S - 1)
    hist, losses = O.run_sample_indexed(net, n, xs, ys, mitigation=mit, update_size=N)
    assert np.allclose(orc.loss_history(), losses[:K - S + 1], rtol=1e-10)
    moved = False
    for s in range(S):
        n_bwd = max(0, K - 2 * (S - 1) + s)          # backward passes stage s has done
        wv, vv = hist[s][n_bwd // N]
        for name_, t_ in wv.items():
            assert torch.allclose(orc.w[s][name_], t_, rtol=1e-10, atol=1e-13), (s, name_)
            assert torch.allclose(orc.v[s][name_], vv[name_], rtol=1e-10, atol=1e-13)
        moved |= n_bwd // N > 0
    assert moved
    # the coefficients count the delay in updates
    for s in range(S):
        D = 2 * (S - 1 - s)
        a, b, T = orc.coef[s]
        if mit in (1, 3):
            assert a == pytest.approx(net["momentum"] ** (D / N), rel=1e-14)
        if mit in (2, 3):
            assert T == pytest.approx(D / N, rel=1e-15)


def test_update_size_with_scaled_hyperparameters_keeps_a_constant_gradient_trajectory(monkeypatch):
    """Eq. hpscale through the per-sample pipeline routine: a stream of samples that all have gradient
    1, plain momentum; update size 32 at the reference values and update size 1 at the scaled values
    move the weight by the same amount over the same number of samples."""
    def fwd(stage, P, x, skip_x, label, bf16=False, relu_shift=0.0):
        return None, P["w"].reshape(()), [dict()]

    def bwd(stage, Wb, saved, dy, need_dx=True, bf16=False):
        return None, {"w": torch.ones(1, 1, dtype=O.DT)}, None

    monkeypatch.setattr(O, "stage_forward", fwd)
    monkeypatch.setattr(O, "stage_backward", bwd)
    lr_r, m_r, n_r = 0.1, 0.9, 32
    lr, m = O.scale_hyperparameters(lr_r, m_r, n_r, 1)
    net = dict(name="const", stages=[[W.linear(1, 1, bias=0), W.ce()]], in_c=1, in_h=1, in_w=1, n_classes=1,
               lr=lr_r, momentum=m_r, n_pool=1, seed_data=1, ticks=0, act_dtype="fp32")
    x, y = np.zeros((1, 1, 1, 1), np.float32), np.zeros(1, np.int32)
    n_samples = n_r * 200
    h_r, _ = O.run_sample_indexed(net, n_samples, x, y, delays=[0], lr=lr_r, momentum=m_r, mitigation=0, update_size=n_r)
    h_1, _ = O.run_sample_indexed(net, n_samples, x, y, delays=[0], lr=lr, momentum=m, mitigation=0, update_size=1)
    assert len(h_r[0]) == 201 and len(h_1[0]) == n_samples + 1
    d_r = float(h_r[0][-1][0]["w"] - h_r[0][0][0]["w"])
    d_1 = float(h_1[0][-1][0]["w"] - h_1[0][0][0]["w"])
    assert d_1 == pytest.approx(d_r, rel=5e-3) and abs(d_r) > 1.0
