"""CPU oracle for batch-1 Pipelined Backpropagation with Spike Compensation
and Linear Weight Prediction.

TEST INFRASTRUCTURE ONLY.  This is the slow, plain reference that defines
what the HIP library must compute.  It shares no code with the HIP path and
must never be imported by it; only tests, the smoke check and the
``cpu_baseline`` leg of the benchmark call it.  Everything is float64 torch
CPU tensors; library primitives (conv2d, unfold/fold, matmul, max_pool2d)
serve as single steps, nothing is blocked, fused or reordered.

What it follows (paper sections / equations, by name):

* Pipeline schedule: Appendix "Pipelined Backpropagation".  S stages, each
  does one forward and one backward transformation per time step; a sample
  needs 2S-1 steps; the update is applied after every sample without
  draining (Eq. sgdpb).  The forward of sample i at stage s sees the stage's
  weights after max(0, i - 2(S-1-s)) updates, its backward sees them after i
  updates (Eqs. wi, wf).
* Optimizer: SGDM (Eqs. sgdmv, sgdm); Spike Compensation with a = m^D,
  b = (1-m^D)/(1-m) (Eqs. gscw, scd); Linear Weight Prediction in velocity
  form, w_hat = w - eta*T*v with T = D (Eq. lwp_v_form); combined update
  (Section "Combined Mitigation").
* Weight stashing (Eq. sgdpb_weight_stash) is available as bwd_weights=1.
* Learning rate and momentum for another update size (Appendix "Small
  Batch Size Training", Eq. hpscale): scale_hyperparameters.

Readings where the paper is silent or ambiguous (kept in step with the
library's documentation):
  R1  A tick's forward and backward passes both read the state as it stands
      at the start of the tick; all updates are applied at the end of it.
      (The last stage's forward and backward weights carry the same index in
      Eq. wf, i.e. zero delay means identical weights.)
  R2  D^s = 2(S-1-s) unless the caller passes delays explicitly.
  R3  The backward pass uses the current, unpredicted weights in every
      formula where a weight appears explicitly (dX = W^T dY, dxhat = gamma
      dy, projection transpose); every activation-derived quantity (saved
      inputs, normalised values, ReLU masks, pooling indices) is the one the
      forward pass produced with its predicted weights.
  R4  LWP uses the velocity as it stands at forward time (the one that
      produced the current weights).
  R5  T_s = D^s; all parameters of a stage (weights, bias, projection,
      GroupNorm scale/shift) share the stage's delay.
  R6  m = 1 gives b = D (limit); m = 0 gives a = 0^D with 0^0 = 1.
  R7  v_0 = 0; a stage without a gradient in a tick is not updated.
  R8  No weight decay, LR schedule, dropout or augmentation.
  R9  Loss = softmax cross-entropy of one sample, natural log, no averaging;
      dlogits = softmax - onehot.
  R10 GroupNorm: biased variance over (C/G)*H*W, eps 1e-5, per-channel affine
      initialised to (1, 0).  ReLU'(0) = 0.  Max-pool gradient goes to the
      first maximum in row-major window order.
  R11 Init: Kaiming normal, std = sqrt(2/fan_in), fan_in = cin*k*k, biases 0;
      counter-based generator documented at ``gauss_tensor``.
  R12 bf16 activation mode: round-to-nearest-even to bf16 of every tensor
      that crosses a stage boundary or is kept for the backward pass
      (stage outputs, a conv output that feeds a GroupNorm in the same
      stage, every dX and skip gradient); all sums stay in high precision.
  R13 Hyper-parameter scaling with the update size (Eq. hpscale) at a
      reference momentum of exactly 1, where the printed ratio is 0/0: the
      limit, lr = lr_ref (n/n_ref)^2.
  R14 Update size N above one (Appendix "Small Batch Size Training" defines it as
      the number of samples that contribute to the gradient of one update and
      sets it to one): the per-worker batch stays one sample per stage and
      tick; a stage adds up the gradients of N consecutive samples (samples
      kN .. kN+N-1 form update k) and applies ONE update with their mean when
      the last of them has passed its backward pass.  Delays are counted in
      updates: SC and LWP use D^s / N for the stage's delay (not rounded).
      Forward of sample i at stage s therefore sees floor((i - D^s) / N)
      updates, its backward floor(i / N).
  Canonical parameter order: stage-major; inside a stage: main weight
  [cout][cin][kh][kw], bias, projection weight, GroupNorm scale, shift.
"""
from __future__ import annotations

import math

import numpy as np
import torch
import torch.nn.functional as F

DT = torch.float64
GN_EPS = 1e-5

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


# --------------------------------------------------------------------------
# initial weights (reading R11)
# --------------------------------------------------------------------------
def _mix64(z):
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def gauss_tensor(seed, tensor_index, n):
    """n standard normals for parameter tensor ``tensor_index``.

    Element e uses outputs 2e and 2e+1 of a splitmix64 stream whose initial
    state is seed XOR (GOLD*(tensor_index+1)): r = mix64(state + GOLD*(c+1))
    for output counter c.  u1 = ((r1>>11)+1)*2^-53 in (0,1], u2 = (r2>>11)*2^-53
    in [0,1); value = sqrt(-2 ln u1) * cos(2 pi u2) (Box-Muller), in float64.
    """
    with np.errstate(over="ignore"):
        key = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) ^ (_GOLD * np.uint64(tensor_index + 1))
        e = np.arange(n, dtype=np.uint64)
        r1 = _mix64(key + _GOLD * (np.uint64(2) * e + np.uint64(1)))
        r2 = _mix64(key + _GOLD * (np.uint64(2) * e + np.uint64(2)))
    u1 = ((r1 >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)
    u2 = (r2 >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def stage_param_specs(stage):
    """[(name, shape, fan_in or None)] in canonical order for one stage."""
    main = [o for o in stage if o["kind"] in ("conv", "linear")]
    assert len(main) == 1, "one weight layer per stage"
    m = main[0]
    specs = []
    if m["kind"] == "conv":
        specs.append(("w", (m["cout"], m["cin"], m["k"], m["k"]), m["cin"] * m["k"] * m["k"]))
    else:
        specs.append(("w", (m["cout"], m["cin"]), m["cin"]))
    if m["bias"]:
        specs.append(("b", (m["cout"],), None))
    for o in stage:
        if o["kind"] == "add" and o["proj"]:
            specs.append(("wp", (o["cout"], o["cin"], 1, 1), o["cin"]))
    for o in stage:
        if o["kind"] == "gn":
            specs.append(("gamma", (o["cin"],), None))
            specs.append(("beta", (o["cin"],), None))
    return specs


def init_params(net, seed):
    """Per stage: dict name -> float64 tensor holding float32-representable
    values (the library stores float32 master weights)."""
    out = []
    tidx = 0
    for stage in net["stages"]:
        p = {}
        for name, shape, fan_in in stage_param_specs(stage):
            n = int(np.prod(shape))
            if fan_in is not None:
                std = math.sqrt(2.0 / fan_in)
                vals = (gauss_tensor(seed, tidx, n) * std).astype(np.float32)
            elif name == "gamma":
                vals = np.ones(n, dtype=np.float32)
            else:
                vals = np.zeros(n, dtype=np.float32)
            p[name] = torch.from_numpy(vals.astype(np.float64)).reshape(shape)
            tidx += 1
        out.append(p)
    return out


def flatten_params(params):
    """Canonical flat float64 vector of all stages' parameters."""
    return torch.cat([t.reshape(-1) for p in params for t in p.values()])


def stage_sizes(net):
    return [sum(int(np.prod(s)) for _, s, _ in stage_param_specs(st)) for st in net["stages"]]


# --------------------------------------------------------------------------
# optimizer pieces
# --------------------------------------------------------------------------
def natural_delays(S):
    """D^s = 2(S-1-s): update steps between a stage's forward and backward of
    the same sample (Eq. wf)."""
    return [2 * (S - 1 - s) for s in range(S)]


def sc_coefficients(m, D):
    """Spike Compensation default a = m^D, b = (1-m^D)/(1-m) (Eq. scd)."""
    a = 1.0 if D == 0 else float(m) ** D
    if m == 1.0:
        b = float(D)
    else:
        b = (1.0 - a) / (1.0 - m)
    return a, b


def scale_hyperparameters(lr_ref, m_ref, n_ref, n):
    """Learning rate and momentum for update size n from those of a reference
    update size n_ref (Appendix "Small Batch Size Training", Eq. hpscale):
    m = m_ref^(n/n_ref), lr = lr_ref (1-m) n / ((1-m_ref) n_ref).  Double
    arithmetic.  m_ref = 1 gives m = 1 and the limit of the ratio, (n/n_ref)^2."""
    m = float(m_ref) ** (float(n) / float(n_ref))
    if m_ref == 1.0:
        lr = float(lr_ref) * (float(n) / float(n_ref)) ** 2
    else:
        lr = (1.0 - m) * float(n) / ((1.0 - float(m_ref)) * float(n_ref)) * float(lr_ref)
    return lr, m


def gsc_update(w, v, g, lr, m, a, b):
    """v' = m v + g ; w' = w - lr (a v' + b g)  (Eqs. gscv, gscw)."""
    v_new = m * v + g
    w_new = w - lr * (a * v_new + b * g)
    return w_new, v_new


def lwp_predict(w, v, lr, T):
    """w_hat = w - lr T v  (Eq. lwp_v_form)."""
    return w - lr * T * v


def _round_bf16(x):
    return x.to(torch.float32).to(torch.bfloat16).to(DT)


# --------------------------------------------------------------------------
# layer routines: forward saves activation-derived state, backward takes the
# weights to use explicitly (reading R3)
# --------------------------------------------------------------------------
def gn_forward(x, gamma, beta, groups):
    C = x.shape[0]
    xg = x.reshape(groups, -1)
    mean = xg.mean(dim=1, keepdim=True)
    var = ((xg - mean) ** 2).mean(dim=1, keepdim=True)
    rstd = 1.0 / torch.sqrt(var + GN_EPS)
    xh = ((xg - mean) * rstd).reshape(x.shape)
    shp = (C,) + (1,) * (x.dim() - 1)
    y = xh * gamma.reshape(shp) + beta.reshape(shp)
    return y, dict(xh=xh, rstd=rstd, groups=groups)


def gn_backward(dy, sv, gamma_b):
    xh, rstd, groups = sv["xh"], sv["rstd"], sv["groups"]
    C = xh.shape[0]
    shp = (C,) + (1,) * (xh.dim() - 1)
    red = tuple(range(1, xh.dim()))
    dgamma = (dy * xh).sum(dim=red)
    dbeta = dy.sum(dim=red)
    dxh = (dy * gamma_b.reshape(shp)).reshape(groups, -1)
    xhg = xh.reshape(groups, -1)
    dx = rstd * (dxh - dxh.mean(dim=1, keepdim=True) - xhg * (dxh * xhg).mean(dim=1, keepdim=True))
    return dx.reshape(xh.shape), dgamma, dbeta


def conv_forward(x, w, b, stride, pad):
    y = F.conv2d(x.unsqueeze(0), w, b, stride=stride, padding=pad)[0]
    return y


def conv_backward(dy, x, w_b, stride, pad, need_dx=True):
    """dW[co,ci,kh,kw] = sum_{oh,ow} dy[co,oh,ow] x[ci,oh*s-p+kh,ow*s-p+kw];
    dX = transpose of the same linear map applied to dy."""
    cout, cin, k, _ = w_b.shape
    cols = F.unfold(x.unsqueeze(0), kernel_size=k, padding=pad, stride=stride)[0]  # [cin*k*k, L]
    dyf = dy.reshape(cout, -1)
    dw = (dyf @ cols.t()).reshape(w_b.shape)
    dx = None
    if need_dx:
        dcols = w_b.reshape(cout, -1).t() @ dyf
        dx = F.fold(dcols.unsqueeze(0), output_size=x.shape[1:], kernel_size=k, padding=pad,
                    stride=stride)[0]
    return dx, dw


def softmax_ce(logits, label):
    z = logits.reshape(-1)
    zmax = z.max()
    e = torch.exp(z - zmax)
    p = e / e.sum()
    loss = -(z[label] - zmax - torch.log(e.sum()))
    dz = p.clone()
    dz[label] -= 1.0
    return loss, dz.reshape(logits.shape)


def stage_forward(stage, P, x, skip_x, label, bf16=False, relu_shift=0.0):
    """Run one stage's op list.  P: parameters to use (predicted weights).
    Returns (output or None for the loss stage, loss or None, saved list).

    relu_shift is a conditioning probe for the tests, 0 everywhere else: the
    ReLU then passes x > relu_shift * rms(x) instead of x > 0, i.e. it takes
    the other decision for every element that lies within |relu_shift| * rms
    of zero on one side.  How far the trajectory of such a run departs from
    the reference run bounds what an implementation in lower precision may
    legitimately differ by when it rounds such an element to the other side."""
    saved = []
    loss = None
    n_ops = len(stage)
    for oi, op in enumerate(stage):
        kind = op["kind"]
        if kind == "gn":
            x, sv = gn_forward(x, P["gamma"], P["beta"], op["groups"])
        elif kind == "relu":
            if relu_shift == 0.0:
                sv = dict(mask=(x > 0))
            else:
                sv = dict(mask=(x > relu_shift * torch.sqrt((x * x).mean())))
            x = torch.where(sv["mask"], x, torch.zeros_like(x))
        elif kind == "conv":
            sv = dict(x=x)
            x = conv_forward(x, P["w"], P.get("b"), op["stride"], op["pad"])
            if bf16 and oi + 1 < n_ops and stage[oi + 1]["kind"] == "gn":
                x = _round_bf16(x)
        elif kind == "linear":
            sv = dict(x=x, shape=x.shape)
            y = P["w"] @ x.reshape(-1)
            if "b" in P:
                y = y + P["b"]
            x = y
            if bf16 and oi + 1 < n_ops and stage[oi + 1]["kind"] == "gn":
                x = _round_bf16(x)
        elif kind == "maxpool":
            y, idx = F.max_pool2d(x.unsqueeze(0), op["k"], op["stride"], op["pad"], return_indices=True)
            sv = dict(idx=idx[0], in_shape=x.shape)
            x = y[0]
        elif kind == "gap":
            sv = dict(in_shape=x.shape)
            x = x.mean(dim=(1, 2))
        elif kind == "add":
            sv = dict(skip=skip_x)
            if op["proj"]:
                x = x + conv_forward(skip_x, P["wp"], None, op["stride"], 0)
            else:
                x = x + skip_x
        elif kind == "ce":
            loss, dz = softmax_ce(x, label)
            sv = dict(dz=dz)
        else:
            raise ValueError(kind)
        saved.append(sv)
    if loss is None and bf16:
        x = _round_bf16(x)
    return (None if loss is not None else x), loss, saved


def stage_backward(stage, W, saved, dy, need_dx=True, bf16=False):
    """Backward through one stage with weights W.  Returns (dx, grads dict,
    dskip or None)."""
    grads = {}
    dskip = None
    first_param_op = min(i for i, o in enumerate(stage) if o["kind"] in ("conv", "linear"))
    for oi in range(len(stage) - 1, -1, -1):
        op, sv = stage[oi], saved[oi]
        kind = op["kind"]
        if kind == "ce":
            dy = sv["dz"]
        elif kind == "add":
            if op["proj"]:
                dskip, dwp = conv_backward(dy, sv["skip"], W["wp"], op["stride"], 0)
                grads["wp"] = dwp
            else:
                dskip = dy
        elif kind == "gap":
            C, H, Wd = sv["in_shape"]
            dy = (dy.reshape(C, 1, 1) / (H * Wd)).expand(C, H, Wd)
        elif kind == "maxpool":
            C, H, Wd = sv["in_shape"]
            du = torch.zeros(C, H * Wd, dtype=DT)
            du.scatter_add_(1, sv["idx"].reshape(C, -1), dy.reshape(C, -1))
            dy = du.reshape(C, H, Wd)
        elif kind == "linear":
            xin = sv["x"].reshape(-1)
            grads["w"] = torch.outer(dy.reshape(-1), xin)
            if "b" in W:
                grads["b"] = dy.reshape(-1).clone()
            last = (oi == first_param_op and oi == 0)
            if need_dx or not last:
                dy = (W["w"].t() @ dy.reshape(-1)).reshape(sv["shape"])
            else:
                dy = None
        elif kind == "conv":
            last = (oi == first_param_op and oi == 0)
            dx, dw = conv_backward(dy, sv["x"], W["w"], op["stride"], op["pad"],
                                   need_dx=(need_dx or not last))
            grads["w"] = dw
            if "b" in W:
                grads["b"] = dy.sum(dim=(1, 2))
            dy = dx
        elif kind == "relu":
            dy = torch.where(sv["mask"], dy, torch.zeros_like(dy))
        elif kind == "gn":
            dy, dg, db = gn_backward(dy, sv, W["gamma"])
            grads["gamma"], grads["beta"] = dg, db
        else:
            raise ValueError(kind)
    if bf16 and dskip is not None:
        dskip = _round_bf16(dskip)
    return dy, grads, dskip


def skip_source(stage):
    for o in stage:
        if o["kind"] == "add":
            return o["skip_from"]
    return -1


# --------------------------------------------------------------------------
# the pipeline, tick form
# --------------------------------------------------------------------------
class PBOracle:
    """pb_init / pb_tick / pb_read_weights / pb_loss_history on the CPU.

    mitigation: 0 plain delayed SGDM, 1 SC_D, 2 LWP^v_D, 3 both.
    bwd_weights: 0 current weights on the backward pass (paper default),
                 1 the forward's predicted weights (weight stashing).
    """

    def __init__(self, net, delays=None, lr=None, momentum=None, seed=42, mitigation=3,
                 bwd_weights=0, sc_scale=1.0, lwp_scale=1.0, lwp_form="v", update_size=1):
        self.net = net
        if int(update_size) < 1:
            raise ValueError("update_size must be >= 1")
        self.N = int(update_size)
        if lwp_form not in ("v", "w"):
            raise ValueError("lwp_form must be 'v' (velocity) or 'w' (weight difference)")
        self.lwp_form = lwp_form
        self.stages = net["stages"]
        self.S = S = len(self.stages)
        self.lr = float(net["lr"] if lr is None else lr)
        self.m = float(net["momentum"] if momentum is None else momentum)
        if not (0.0 <= self.m <= 1.0):
            raise ValueError("momentum must be in [0,1]")
        nat = natural_delays(S)
        self.delays = list(nat if delays is None else delays)
        if self.delays != nat:
            raise ValueError("tick form needs the pipeline's natural delays; "
                             "use run_sample_indexed for other delays")
        self.mitigation = mitigation
        self.bwd_weights = bwd_weights
        self.bf16 = (net.get("act_dtype", "fp32") == "bf16")
        self.w = init_params(net, seed)
        self.v = [{k: torch.zeros_like(t) for k, t in p.items()} for p in self.w]
        self.w_prev = [dict(p) for p in self.w]     # weights before the latest update (LWP weight-difference form)
        # over-compensation (Section "Combined Mitigation", appendix on extended horizons):
        # SC with the coefficients of delay sc_scale*D, LWP with horizon T = lwp_scale*D
        self.coef = []
        for D in self.delays:
            Du = D / self.N if self.N > 1 else D        # the stage's delay counted in updates (reading R14)
            a, b = sc_coefficients(self.m, sc_scale * Du) if mitigation in (1, 3) else (1.0, 0.0)
            T = float(lwp_scale * Du) if mitigation in (2, 3) else 0.0
            self.coef.append((a, b, T))
        self.gsum = [None] * S         # gradients added up since the stage's latest update
        self.gcount = [0] * S
        self.t = 0
        self.fwd_mail = {}      # stage -> activation produced for it last tick
        self.grad_mail = {}     # stage -> dY for its output, produced last tick
        self.saved = [dict() for _ in range(S)]     # stage -> sample -> saved state
        self.skipgrad = [dict() for _ in range(S)]  # tap stage -> sample -> dskip
        self.labels = {}
        self.losses = []
        self.last_grads = [None] * S   # gradients applied in the latest tick (for tests)
        self.relu_shift = 0.0          # conditioning probe for the tests, see stage_forward

    def predicted(self, s):
        a, b, T = self.coef[s]
        if self.lwp_form == "w":      # Eq. lwp_w_form: w_hat = w + T (w - w_prev)
            return {k: self.w[s][k] + T * (self.w[s][k] - self.w_prev[s][k]) for k in self.w[s]}
        return {k: lwp_predict(self.w[s][k], self.v[s][k], self.lr, T) for k in self.w[s]}

    def tick(self, sample, label):
        S, t = self.S, self.t
        x0 = torch.as_tensor(np.asarray(sample), dtype=DT).reshape(
            self.net["in_c"], self.net["in_h"], self.net["in_w"])
        if self.bf16:
            x0 = _round_bf16(x0)
        self.labels[t] = int(label)
        new_fwd, new_grad = {}, {}
        pending = {}
        dlogits_sample = None
        for s in range(S):
            stage = self.stages[s]
            i = t - s
            if i >= 0:
                xin = x0 if s == 0 else self.fwd_mail[s]
                what = self.predicted(s)
                src = skip_source(stage)
                skip_x = self.saved[src][i]["x_in"] if src >= 0 else None
                y, loss, sv = stage_forward(stage, what, xin, skip_x,
                                            self.labels[i] if s == S - 1 else None, self.bf16, self.relu_shift)
                self.saved[s][i] = dict(ops=sv, x_in=xin, what=what)
                if s < S - 1:
                    new_fwd[s + 1] = y
                else:
                    self.losses.append(float(loss))
                    dlogits_sample = i
            j = t - 2 * (S - 1) + s
            if j >= 0:
                entry = self.saved[s].pop(j)
                if s == S - 1:
                    assert dlogits_sample == j
                    dy = None                       # the ce op supplies dlogits
                else:
                    dy = self.grad_mail[s]
                W = entry["what"] if self.bwd_weights == 1 else self.w[s]
                dx, grads, dskip = stage_backward(stage, W, entry["ops"], dy,
                                                  need_dx=(s > 0), bf16=self.bf16)
                if s > 0:
                    if j in self.skipgrad[s]:
                        dx = dx + self.skipgrad[s].pop(j)
                    if self.bf16:
                        dx = _round_bf16(dx)
                    new_grad[s - 1] = dx
                src = skip_source(stage)
                if src >= 0:
                    self.skipgrad[src][j] = dskip
                pending[s] = grads
        # all reads done: apply the updates (reading R1)
        for s, grads in pending.items():
            a, b, T = self.coef[s]
            if self.N > 1:
                # update size N: one update with the mean gradient of N consecutive samples (reading R14)
                self.gsum[s] = grads if self.gsum[s] is None else {k: self.gsum[s][k] + grads[k] for k in grads}
                self.gcount[s] += 1
                self.last_grads[s] = grads
                if self.gcount[s] < self.N:
                    continue
                grads = {k: t_ / self.N for k, t_ in self.gsum[s].items()}
                self.gsum[s], self.gcount[s] = None, 0
            for k in self.w[s]:
                self.w_prev[s][k] = self.w[s][k]
                self.w[s][k], self.v[s][k] = gsc_update(self.w[s][k], self.v[s][k], grads[k],
                                                        self.lr, self.m, a, b)
            self.last_grads[s] = grads
        self.labels.pop(t - (S - 1), None)
        self.fwd_mail, self.grad_mail = new_fwd, new_grad
        self.t += 1

    def read_weights(self):
        return flatten_params(self.w).numpy().copy()

    def read_velocity(self):
        return flatten_params(self.v).numpy().copy()

    def loss_history(self):
        return np.asarray(self.losses, dtype=np.float64)


# --------------------------------------------------------------------------
# the same algorithm written per sample (Eqs. wi, sgdpb, wf; Appendix
# "Simulating Delayed Gradients"): defines arbitrary per-stage delays and
# cross-checks the tick form's bookkeeping
# --------------------------------------------------------------------------
def run_sample_indexed(net, n_samples, pool_x, pool_y, delays=None, lr=None, momentum=None,
                       seed=42, mitigation=3, bwd_weights=0, sc_scale=1.0, lwp_scale=1.0, lwp_form="v",
                       update_size=1):
    """Process samples one at a time.  Stage s's forward of sample i uses the
    stage's state after max(0, i - D^s) updates, the backward uses the state
    after i updates; then update i is applied to every stage.

    update_size N > 1 (reading R14): update k is applied after sample kN+N-1
    with the mean gradient of samples kN..kN+N-1; the forward pass of sample i
    sees floor(max(0, i - D^s) / N) updates, the backward pass floor(i / N).

    Returns (history, losses): history[s][k] = (params, velocity) of stage s
    after k updates, k = 0..n_samples // N.
    """
    N = int(update_size)
    stages = net["stages"]
    S = len(stages)
    lr = float(net["lr"] if lr is None else lr)
    m = float(net["momentum"] if momentum is None else momentum)
    delays = natural_delays(S) if delays is None else list(delays)
    bf16 = (net.get("act_dtype", "fp32") == "bf16")
    w0 = init_params(net, seed)
    hist = [[(w0[s], {k: torch.zeros_like(t) for k, t in w0[s].items()})] for s in range(S)]
    coef = []
    for D in delays:
        Du = D / N if N > 1 else D
        a, b = sc_coefficients(m, sc_scale * Du) if mitigation in (1, 3) else (1.0, 0.0)
        T = float(lwp_scale * Du) if mitigation in (2, 3) else 0.0
        coef.append((a, b, T))
    losses = []
    gsum = [None] * S
    n_pool = len(pool_y)
    for i in range(n_samples):
        x = torch.as_tensor(pool_x[i % n_pool], dtype=DT).reshape(net["in_c"], net["in_h"], net["in_w"])
        if bf16:
            x = _round_bf16(x)
        label = int(pool_y[i % n_pool])
        saved, inputs, whats = [], [], []
        for s in range(S):
            kf = max(0, i - delays[s]) // N            # updates the forward pass sees
            wv, vv = hist[s][kf]
            if lwp_form == "w":
                wp_, _ = hist[s][max(0, kf - 1)]
                what = {k: wv[k] + coef[s][2] * (wv[k] - wp_[k]) for k in wv}
            else:
                what = {k: lwp_predict(wv[k], vv[k], lr, coef[s][2]) for k in wv}
            src = skip_source(stages[s])
            inputs.append(x)
            y, loss, sv = stage_forward(stages[s], what, x, inputs[src] if src >= 0 else None,
                                        label if s == S - 1 else None, bf16)
            saved.append(sv)
            whats.append(what)
            x = y
        losses.append(float(loss))
        dy = None
        skipgrad = {}
        grads_all = [None] * S
        for s in range(S - 1, -1, -1):
            wcur, _ = hist[s][i // N]
            W = whats[s] if bwd_weights == 1 else wcur
            dx, grads, dskip = stage_backward(stages[s], W, saved[s], dy, need_dx=(s > 0), bf16=bf16)
            if s > 0:
                if s in skipgrad:
                    dx = dx + skipgrad.pop(s)
                if bf16:
                    dx = _round_bf16(dx)
            src = skip_source(stages[s])
            if src >= 0:
                skipgrad[src] = dskip
            grads_all[s] = grads
            dy = dx
        for s in range(S):
            g_upd = grads_all[s]
            if N > 1:
                gsum[s] = g_upd if gsum[s] is None else {k: gsum[s][k] + g_upd[k] for k in g_upd}
                if (i + 1) % N:
                    continue
                g_upd = {k: t_ / N for k, t_ in gsum[s].items()}
                gsum[s] = None
            wcur, vcur = hist[s][i // N]
            a, b, T = coef[s]
            wn, vn = {}, {}
            for k in wcur:
                wn[k], vn[k] = gsc_update(wcur[k], vcur[k], g_upd[k], lr, m, a, b)
            hist[s].append((wn, vn))
    return hist, np.asarray(losses)


def scalar_quadratic_run(lam, lr, m, D, a, b, T, steps, w_form=False, phi0=1.0):
    """Delayed optimisation of the scalar loss with gradient lam*phi
    (Section "Analysis for a Convex Quadratic"), driven through this module's
    own update and prediction routines.  g_t = lam * pred_t with pred_t built
    from the state D steps back (the state before step 0 is constant phi0 with
    zero velocity).  Velocity form: pred = lwp_predict(phi, v, lr, T);
    weight-difference form: pred = phi + T (phi - phi_prev).  Returns the
    trajectory phi_0..phi_steps."""
    phi = [phi0]
    v = [0.0]
    for t in range(steps):
        k = t - D
        ph = phi[k] if k >= 0 else phi0
        if w_form:
            ph_prev = phi[k - 1] if k - 1 >= 0 else phi0
            pred = ph + T * (ph - ph_prev)
        else:
            pred = lwp_predict(ph, v[k] if k >= 0 else 0.0, lr, T)
        w_new, v_new = gsc_update(phi[-1], v[-1], lam * pred, lr, m, a, b)
        phi.append(w_new)
        v.append(v_new)
    return np.asarray(phi)
