"""The stand-alone fused update kernel (pb_update_standalone) against the oracle's update and
prediction formulas, element by element (Section "Combined Mitigation": Eqs. gscv, gscw with the
default coefficients of Eq. scd; Eq. lwp_v_form)."""
import numpy as np
import pytest

from oracle import pb_oracle as O

pytestmark = pytest.mark.gpu

EPS = 2.0 ** -24   # half a unit in the last place of an fp32 result of magnitude 1


@pytest.mark.parametrize("n", [1024, 5 * 1024, 3 * 4096 + 1024, 64 * 4096 + 3 * 1024])
@pytest.mark.parametrize("with_what", [True, False])
@pytest.mark.parametrize("D,m,lr", [(0, 0.9, 0.01), (7, 0.9, 0.005), (38, 0.9, 0.005), (5, 0.0, 0.1), (3, 1.0, 0.01)])
def test_update_standalone_matches_oracle(n, with_what, D, m, lr):
    import torch
    from paper_2003_11666_amd import update_standalone
    rng = np.random.default_rng(1000 + n + D)
    w = rng.standard_normal(n).astype(np.float32)
    v = (rng.standard_normal(n) * 3).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    a, b = O.sc_coefficients(m, D)
    a32, b32, lrT32, lr32, m32 = (np.float32(x) for x in (a, b, lr * D, lr, m))
    wd, vd, gd = (torch.from_numpy(x).cuda() for x in (w, v, g))
    hd = torch.full((n,), 7.0, device="cuda") if with_what else None
    update_standalone(wd, vd, gd, hd, float(lr32), float(m32), float(a32), float(b32), float(lrT32))
    torch.cuda.synchronize()
    # the oracle's routines in float64 on the float32 inputs and the float32-rounded coefficients the kernel was handed
    w64, v64, g64 = (torch.from_numpy(x.astype(np.float64)) for x in (w, v, g))
    w_ref, v_ref = O.gsc_update(w64, v64, g64, float(lr32), float(m32), float(a32), float(b32))
    # (T enters the kernel as the single float lr*T)
    h_ref = w_ref - float(lrT32) * v_ref
    assert torch.equal(h_ref, O.lwp_predict(w_ref, v_ref, float(lrT32), 1.0))
    # fp32 evaluation with fused multiply-adds: v' has one rounding; w' = fma(-lr, fma(a, v', b*g), w) three
    # (b*g, the inner sum, the outer sum) plus the inherited error of v'; w_hat one more.  Bound every
    # element by 4 half-units in the last place of the magnitudes that enter it.
    av, ag, aw = np.abs(v_ref.numpy()), np.abs(g.astype(np.float64)), np.abs(w.astype(np.float64))
    v_bound = 4 * EPS * (abs(float(m32)) * np.abs(v.astype(np.float64)) + ag)
    w_bound = 4 * EPS * (aw + float(lr32) * (abs(float(a32)) * av + abs(float(b32)) * ag)) + float(lr32) * abs(float(a32)) * v_bound
    h_bound = w_bound + 4 * EPS * (np.abs(w_ref.numpy()) + float(lrT32) * av) + float(lrT32) * v_bound
    assert np.all(np.abs(vd.cpu().numpy() - v_ref.numpy()) <= v_bound)
    assert np.all(np.abs(wd.cpu().numpy() - w_ref.numpy()) <= w_bound)
    if with_what:
        assert np.all(np.abs(hd.cpu().numpy() - h_ref.numpy()) <= h_bound)
    # the gradient is an input: untouched
    assert np.array_equal(gd.cpu().numpy(), g)


def test_update_standalone_rejects_bad_arguments():
    import torch
    from paper_2003_11666_amd import update_standalone
    from paper_2003_11666_amd.binding import PBError
    w = torch.zeros(2048 + 4, device="cuda")
    v, g = torch.zeros_like(w), torch.zeros_like(w)
    with pytest.raises(PBError):     # not a multiple of 1024
        update_standalone(w[:1000], v[:1000], g[:1000], None, 0.1, 0.9, 1.0, 0.0, 0.0)
    with pytest.raises(PBError):     # 16-byte vector accesses need 16-byte aligned arrays
        update_standalone(w[1:1025], v[:1024], g[:1024], None, 0.1, 0.9, 1.0, 0.0, 0.0)
    with pytest.raises(PBError):
        update_standalone(w[:1024], v[:1024], g[:1024], w[2:1026], 0.1, 0.9, 1.0, 0.0, 0.0)
