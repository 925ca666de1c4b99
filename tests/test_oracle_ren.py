"""Pins of the oracle's Range-EvoNorm forward (Eq. "ren") and its derived backward."""
import os

import numpy as np
import pytest
import torch

import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _params(seed, C):
    g = wl.rng(seed)
    v = (1.0 + 0.3 * g.standard_normal(C)).astype(np.float32)
    gamma = (1.0 + 0.2 * g.standard_normal(C)).astype(np.float32)
    beta = (0.1 * g.standard_normal(C)).astype(np.float32)
    return v, gamma, beta


def test_constants_from_paper_formula(orc):
    rows = [l.split() for l in open(os.path.join(GOLD, "ren_constants.txt")) if l.strip() and l[0] != "#"]
    for m, cm in rows:
        m = int(m)
        # slab {0, 1} repeated: range 1, v=0 -> hs = 1/2 -> y = x / (2 C(m))
        x = np.zeros((1, 1, 2, m), np.float32)
        x[0, 0, 1, :] = 1.0
        y, rng_, _, _ = orc.range_evonorm_fwd(x, 1, np.zeros(m), np.ones(m), np.zeros(m), eps=0.0)
        assert rng_[0, 0] == 1.0
        assert abs(y[0, 0, 1, 0] - 0.5 / float(cm)) < 2e-6 * 0.5 / float(cm) + 1e-6


def test_hand_example(orc):
    # one group of m=2 channels over 3 pixels: slab {-3,-1,0,1,3,5}; R=8, D=0.849322*8
    x = np.array([-3, -1, 0, 1, 3, 5], np.float32).reshape(1, 1, 3, 2)
    y, rng_, amx, amn = orc.range_evonorm_fwd(x, 1, np.ones(2), np.ones(2), np.zeros(2), eps=0.0)
    assert rng_[0, 0] == 8.0 and amx[0, 0] == 5 and amn[0, 0] == 0
    yf = y.ravel()
    assert abs(yf[4] - 0.441529) < 1e-6       # x=3: hs=1
    assert yf[0] == 0.0                       # x=-3: hs=0
    assert abs(yf[3] - 0.098117) < 1e-6       # x=1: hs=4/6
    assert yf[2] == 0.0


def test_v_zero_and_relu_limit(orc):
    x = wl.images(11, 3, 5, 6, 8)
    C, groups = 8, 2
    _, gamma, beta = _params(12, C)
    y, rng_, _, _ = orc.range_evonorm_fwd(x, groups, np.zeros(C), gamma, beta, eps=0.0)
    m = C // groups
    Cm = 1 / np.sqrt(2 * np.log(m))
    xs = x.reshape(3, 30, groups, m).astype(np.float64)
    R = xs.max(axis=(1, 3)) - xs.min(axis=(1, 3))
    assert np.allclose(rng_, R, rtol=0, atol=0)
    ref = (xs * 0.5 / (Cm * R)[:, None, :, None]).reshape(x.shape) * gamma + beta
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
    # v -> large: x*hs(vx) -> relu(x)
    y2, _, _, _ = orc.range_evonorm_fwd(x, groups, np.full(C, 1e6), gamma, beta, eps=0.0)
    ref2 = (np.maximum(xs, 0) / (Cm * R)[:, None, :, None]).reshape(x.shape) * gamma + beta
    assert np.allclose(y2, ref2, rtol=1e-5, atol=1e-5)


def test_scale_invariance_and_eps(orc):
    x = wl.images(13, 2, 4, 4, 4)
    C = 4
    z, o = np.zeros(C), np.ones(C)
    y1, _, _, _ = orc.range_evonorm_fwd(x, 2, z, o, z, eps=0.0)
    y2, _, _, _ = orc.range_evonorm_fwd(x * np.float32(4.0), 2, z, o, z, eps=0.0)   # power of two: exact
    assert np.allclose(y1, y2, rtol=1e-14, atol=0)
    # eps adds to the denominator
    ya, r, _, _ = orc.range_evonorm_fwd(x, 2, z, o, z, eps=0.5)
    Cm = 1 / np.sqrt(2 * np.log(2))
    ratio = (Cm * r) / (Cm * r + 0.5)
    assert np.allclose(ya, y1 * np.repeat(ratio, 2, axis=1)[:, None, None, :], rtol=1e-12)


def test_first_index_tie_break(orc):
    x = np.zeros((1, 2, 2, 4), np.float32)      # groups=2, m=2; slab index = (h*W+w)*2+cc
    x[0, 0, 1, 0] = 2; x[0, 1, 0, 1] = 2        # two maxima in group 0 at idx 2 and 5
    x[0, 0, 0, 1] = -1; x[0, 1, 1, 0] = -1      # two minima in group 0 at idx 1 and 6
    _, r, amx, amn = orc.range_evonorm_fwd(x, 2, np.ones(4), np.ones(4), np.zeros(4))
    assert r[0, 0] == 3 and amx[0, 0] == 2 and amn[0, 0] == 1
    assert r[0, 1] == 0 and amx[0, 1] == 0 and amn[0, 1] == 0   # constant slab


def test_rejects_one_channel_per_group(orc):
    x = np.zeros((1, 2, 2, 4), np.float32)
    with pytest.raises(orc.OracleError):
        orc.range_evonorm_fwd(x, 4, np.ones(4), np.ones(4), np.zeros(4))
    with pytest.raises(orc.OracleError):
        orc.range_evonorm_fwd(x, 3, np.ones(4), np.ones(4), np.zeros(4))


def _torch_ren(x, groups, v, gamma, beta, eps):
    N, H, W, C = x.shape
    m = C // groups
    xs = x.reshape(N, H * W, groups, m)
    R = xs.amax(dim=(1, 3)) - xs.amin(dim=(1, 3))
    D = (R / np.sqrt(2 * np.log(m)) + eps)[:, None, :, None]
    hs = torch.clamp((xs * v.reshape(groups, m) + 3) / 6, 0, 1)
    return ((xs * hs / D) * gamma.reshape(groups, m) + beta.reshape(groups, m)).reshape(N, H, W, C)


@pytest.mark.parametrize("shape,groups", [((2, 4, 5, 8), 2), ((3, 3, 3, 16), 8), ((1, 6, 6, 4), 1)])
def test_bwd_against_float64_autograd(orc, shape, groups):
    x = wl.images(21, *shape)
    C = shape[3]
    v, gamma, beta = _params(22, C)
    dy = wl.rng(23).standard_normal(shape)
    eps = 1e-5
    xt = torch.from_numpy(x.astype(np.float64)).requires_grad_()
    vt, gt, bt = (torch.from_numpy(t.astype(np.float64)).requires_grad_() for t in (v, gamma, beta))
    yt = _torch_ren(xt, groups, vt, gt, bt, eps)
    y, _, _, _ = orc.range_evonorm_fwd(x, groups, v, gamma, beta, eps)
    assert np.allclose(y, yt.detach().numpy(), rtol=1e-12, atol=1e-13)
    yt.backward(torch.from_numpy(dy))
    dx, dv, dg, db = orc.range_evonorm_bwd(dy, x, groups, v, gamma, eps)
    assert np.allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dv, vt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dg, gt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(db, bt.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_bwd_finite_differences(orc):
    # the oracle forward takes fp32 x: use a dyadic step so perturbed inputs stay exact in fp32
    shape, groups, C = (1, 3, 3, 4), 2, 4
    x = (np.rint(wl.images(31, *shape) * 64) / 64).astype(np.float32)
    v, gamma, beta = _params(32, C)
    dy = wl.rng(33).standard_normal(shape)
    dx, dv, dg, db = orc.range_evonorm_bwd(dy, x, groups, v, gamma, eps=1e-5)
    h = 2.0 ** -12
    z = x.astype(np.float64) * v
    assert np.abs(np.abs(z) - 3).min() > 10 * h      # away from hard-sigmoid kinks
    L = lambda xx, vv=v, gg=gamma, bb=beta: (orc.range_evonorm_fwd(xx, groups, vv, gg, bb, eps=1e-5)[0] * dy).sum()
    for i in range(x.size):
        e = np.zeros(x.size, np.float32); e[i] = h
        e = e.reshape(shape)
        fd = (L(x + e) - L(x - e)) / (2 * h)
        assert abs(fd - dx.ravel()[i]) < 1e-5 * max(1.0, abs(fd)), i


def test_bwd_scale_invariance_identity(orc):
    # v=0, eps=0, beta=0: y is invariant to x -> a*x, hence sum_slab x*dx = 0
    shape, groups, C = (2, 4, 4, 8), 2, 8
    x = wl.images(41, *shape)
    dy = wl.rng(42).standard_normal(shape)
    dx, _, _, _ = orc.range_evonorm_bwd(dy, x, groups, np.zeros(C), np.ones(C), eps=0.0)
    s = (dx * x).reshape(2, 16, groups, 4).sum(axis=(1, 3))
    assert np.abs(s).max() < 1e-10
