"""Pins of the oracle's two full-precision comparison layers: EvoNorm-S0 (Eq. "en") and range batch-norm (Eq. "rbn"),
forward against closed forms and library statistics, backward against float64 autograd and finite differences."""
import numpy as np
import torch

import workloads as wl


def _params(seed, C):
    g = wl.rng(seed)
    v = (1.0 + 0.3 * g.standard_normal(C)).astype(np.float32)
    gamma = (1.0 + 0.2 * g.standard_normal(C)).astype(np.float32)
    beta = (0.1 * g.standard_normal(C)).astype(np.float32)
    return v, gamma, beta


# ---------------------------------------------------------------- EvoNorm-S0
def test_evonorm_hand_example(orc):
    # one sample, one group of 2 channels over 2 pixels: slab {1, 3, 5, 7}: mean 4, population variance 5
    x = np.array([1, 3, 5, 7], np.float32).reshape(1, 1, 2, 2)
    y, mean, var = orc.evonorm_s0_fwd(x, 1, np.zeros(2), np.ones(2), np.zeros(2), eps=0.0)
    assert mean[0, 0] == 4.0 and var[0, 0] == 5.0
    # v = 0: sigmoid = 1/2, y = x / (2 sqrt 5)
    assert np.allclose(y.ravel(), np.array([1, 3, 5, 7]) / (2 * np.sqrt(5.0)), rtol=1e-15)
    # v = ln 3 at x = 1: sigmoid = 3/4
    y2, _, _ = orc.evonorm_s0_fwd(x, 1, np.full(2, np.float32(np.log(3.0))), np.ones(2), np.zeros(2), eps=0.0)
    assert abs(y2.ravel()[0] - 0.75 / np.sqrt(5.0)) < 1e-7


def test_evonorm_v_zero_is_half_x_over_library_std(orc):
    x = wl.images(21, 3, 5, 6, 8) * 2.0 + 0.7
    C, groups = 8, 2
    _, gamma, beta = _params(22, C)
    y, mean, var = orc.evonorm_s0_fwd(x, groups, np.zeros(C), gamma, beta, eps=0.0)
    xs = x.reshape(3, 30, groups, C // groups).astype(np.float64)
    assert np.allclose(mean, xs.mean(axis=(1, 3)), rtol=1e-13, atol=1e-13)
    assert np.allclose(var, xs.var(axis=(1, 3)), rtol=1e-12)            # numpy's default: the population variance
    ref = (0.5 * xs / xs.std(axis=(1, 3))[:, None, :, None]).reshape(x.shape) * gamma + beta
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_evonorm_large_v_is_relu_over_std_and_eps_enters_under_the_root(orc):
    x = wl.images(23, 2, 4, 4, 4)
    y, _, var = orc.evonorm_s0_fwd(x, 1, np.full(4, 1e6), np.ones(4), np.zeros(4), eps=0.0)
    ref = np.maximum(x.astype(np.float64), 0) / np.sqrt(var)[:, None, None, :]
    assert np.allclose(y, ref, rtol=1e-5, atol=1e-6)
    y2, _, var2 = orc.evonorm_s0_fwd(x, 1, np.zeros(4), np.ones(4), np.zeros(4), eps=0.25)
    assert np.allclose(y2, 0.5 * x.astype(np.float64) / np.sqrt(var2 + 0.25)[:, None, None, :], rtol=1e-12)


def test_evonorm_scale_invariance(orc):
    x = wl.images(24, 2, 5, 5, 6)
    v, gamma, beta = _params(25, 6)
    y1, _, _ = orc.evonorm_s0_fwd(x, 3, v, gamma, beta, eps=0.0)
    y2, _, _ = orc.evonorm_s0_fwd(x * np.float32(4.0), 3, v * np.float32(0.25), gamma, beta, eps=0.0)   # exact scalings
    assert np.allclose(y1, y2, rtol=1e-12, atol=1e-12)


def _torch_evonorm(x, groups, v, gamma, beta, eps):
    N, H, W, C = x.shape
    xs = x.reshape(N, H * W, groups, C // groups)
    var = xs.var(dim=(1, 3), unbiased=False, keepdim=True)
    u = x * torch.sigmoid(v * x)
    return (u.reshape(xs.shape) / torch.sqrt(var + eps)).reshape(x.shape) * gamma + beta


def test_evonorm_backward_matches_float64_autograd(orc):
    N, H, W, C, groups = 2, 3, 4, 8, 4
    x = wl.images(26, N, H, W, C)
    v, gamma, beta = _params(27, C)
    dy = wl.rng(28).standard_normal(x.shape)
    dx, dv, dg, db = orc.evonorm_s0_bwd(dy, x, groups, v, gamma, eps=1e-3)
    tx, tv, tg, tb = (torch.tensor(t.astype(np.float64), requires_grad=True) for t in (x, v, gamma, beta))
    y = _torch_evonorm(tx, groups, tv, tg, tb, 1e-3)
    yo, _, _ = orc.evonorm_s0_fwd(x, groups, v, gamma, beta, eps=1e-3)
    assert np.allclose(yo, y.detach().numpy(), rtol=1e-12, atol=1e-12)
    y.backward(torch.tensor(dy))
    for got, ref in ((dx, tx.grad), (dv, tv.grad), (dg, tg.grad), (db, tb.grad)):
        assert np.allclose(got, ref.numpy(), rtol=1e-10, atol=1e-12)


def test_evonorm_backward_finite_difference_of_the_forward(orc):
    N, H, W, C, groups = 1, 2, 3, 4, 2
    x = wl.images(29, N, H, W, C)
    v, gamma, beta = _params(30, C)
    dy = wl.rng(31).standard_normal(x.shape)
    dx, _, _, _ = orc.evonorm_s0_bwd(dy, x, groups, v, gamma, eps=1e-2)
    h = np.float32(2.0 ** -10)
    for at in [(0, 0, 0, 0), (0, 1, 2, 3), (0, 0, 1, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[at] += h; xm[at] -= h
        yp, _, _ = orc.evonorm_s0_fwd(xp, groups, v, gamma, beta, eps=1e-2)
        ym, _, _ = orc.evonorm_s0_fwd(xm, groups, v, gamma, beta, eps=1e-2)
        num = ((yp - ym) * dy).sum() / float(xp[at] - xm[at])
        assert abs(num - dx[at]) < 1e-4 * max(1.0, abs(dx[at]))


# ---------------------------------------------------------------- range batch-norm
def test_range_bn_hand_example(orc):
    # one channel, batch 2, one pixel each... plus a second channel: values {-1, 3} and {2, 2.5}
    x = np.array([[-1, 2], [3, 2.5]], np.float32).reshape(2, 1, 1, 2)
    y, mean, rng_, amx, amn = orc.range_bn_fwd(x, np.ones(2), np.zeros(2), eps=0.0)
    Cb = 1 / np.sqrt(2 * np.log(2.0))
    assert list(mean) == [1.0, 2.25] and list(rng_) == [4.0, 0.5]
    assert list(amx) == [1, 1] and list(amn) == [0, 0]
    assert np.allclose(y[:, 0, 0, 0], np.array([-2.0, 2.0]) / (Cb * 4.0), rtol=1e-15)
    assert np.allclose(y[:, 0, 0, 1], np.array([-0.25, 0.25]) / (Cb * 0.5), rtol=1e-15)


def test_range_bn_against_library_statistics_shift_and_first_index(orc):
    N, H, W, C = 4, 3, 5, 6
    x = wl.images(41, N, H, W, C)
    _, gamma, beta = _params(42, C)
    y, mean, rng_, amx, amn = orc.range_bn_fwd(x, gamma, beta, eps=0.0)
    xs = x.reshape(-1, C).astype(np.float64)
    assert np.allclose(mean, xs.mean(0), rtol=1e-13, atol=1e-14)
    assert np.array_equal(rng_, xs.max(0) - xs.min(0))
    assert np.array_equal(amx, xs.argmax(0)) and np.array_equal(amn, xs.argmin(0))     # numpy: first occurrence
    Cb = 1 / np.sqrt(2 * np.log(N))
    assert np.allclose(y.reshape(-1, C), (xs - xs.mean(0)) / (Cb * rng_) * gamma + beta, rtol=1e-12, atol=1e-12)
    # a per-channel shift changes nothing (exactly representable shifts keep x + s exact here)
    y2, _, _, _, _ = orc.range_bn_fwd((x.astype(np.float64) + 8.0).astype(np.float32), gamma, beta, eps=0.0)
    assert np.allclose(y, y2, rtol=0, atol=2e-5)
    # ties: the first position wins
    xt = np.zeros((2, 1, 3, 1), np.float32)
    xt[0, 0, 1, 0] = xt[1, 0, 0, 0] = 2.0
    xt[0, 0, 2, 0] = xt[1, 0, 2, 0] = -1.0
    _, _, _, a, b = orc.range_bn_fwd(xt, np.ones(1), np.zeros(1))
    assert a[0] == 1 and b[0] == 2


def _torch_range_bn(x, gamma, beta, eps, N):
    C = x.shape[-1]
    xs = x.reshape(-1, C)
    mu = xs.mean(0)
    R = xs.max(0).values - xs.min(0).values
    D = R / np.sqrt(2 * np.log(N)) + eps
    return ((xs - mu) / D * gamma + beta).reshape(x.shape)


def test_range_bn_backward_matches_float64_autograd(orc):
    N, H, W, C = 3, 2, 4, 5
    x = wl.images(43, N, H, W, C)         # continuous data: no ties, the extrema are unique
    _, gamma, beta = _params(44, C)
    dy = wl.rng(45).standard_normal(x.shape)
    dx, dg, db = orc.range_bn_bwd(dy, x, gamma, eps=1e-3)
    tx, tg, tb = (torch.tensor(t.astype(np.float64), requires_grad=True) for t in (x, gamma, beta))
    y = _torch_range_bn(tx, tg, tb, 1e-3, N)
    yo, _, _, _, _ = orc.range_bn_fwd(x, gamma, beta, eps=1e-3)
    assert np.allclose(yo, y.detach().numpy(), rtol=1e-12, atol=1e-12)
    y.backward(torch.tensor(dy))
    for got, ref in ((dx, tx.grad), (dg, tg.grad), (db, tb.grad)):
        assert np.allclose(got, ref.numpy(), rtol=1e-10, atol=1e-12)
    assert np.abs(dx.reshape(-1, C).sum(0)).max() < 1e-10      # shift invariance of the forward: gradients sum to 0


def test_range_bn_rejects_batch_of_one(orc):
    import pytest
    with pytest.raises(Exception):
        orc.range_bn_fwd(np.zeros((1, 2, 2, 4), np.float32), np.ones(4), np.zeros(4))
