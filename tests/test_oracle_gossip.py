"""Pins of the oracle's gossip step (Algorithm 1 step 7; supplement Algorithms 2 and 3) and of
the glue layers (Table "hardware_training": skip connection, average pool)."""
import numpy as np
import torch

import workloads as wl


def test_plain_mix_is_W_times_X(orc):
    n, d = 8, 1000
    x = wl.agent_params(1, n, d)
    for Wm in (wl.ring_matrix(n), wl.torus_matrix(2, 4)):
        out, _ = orc.gossip_mix(x, None, Wm, eta=1.0)
        assert np.allclose(out, Wm.astype(np.float64) @ x.astype(np.float64), rtol=1e-12, atol=1e-14)
        # doubly stochastic W preserves the agent average, for any averaging rate
        out2, _ = orc.gossip_mix(x, None, Wm, eta=0.37)
        assert np.allclose(out2.mean(0), x.astype(np.float64).mean(0), rtol=0, atol=1e-7)
    out, _ = orc.gossip_mix(x, None, np.eye(n, dtype=np.float32), eta=1.0)
    assert np.array_equal(out, x.astype(np.float64))
    out, _ = orc.gossip_mix(x, None, wl.ring_matrix(n), eta=0.0)
    assert np.array_equal(out, x.astype(np.float64))


def test_ring_fourier_mode_closed_form(orc):
    # ring(1/3,1/3,1/3) is circulant: mode k scales by (1 + 2cos(2 pi k/n))/3 ; n=16,k=1 -> 0.949253
    n, d = 16, 5
    Wm = wl.ring_matrix(n)
    for k in (1, 2, 5, 8):
        lam = (1 + 2 * np.cos(2 * np.pi * k / n)) / 3
        x = (np.cos(2 * np.pi * k * np.arange(n) / n)[:, None] * np.arange(1, d + 1)[None, :]).astype(np.float32)
        out, _ = orc.gossip_mix(x, None, Wm, eta=1.0)
        assert np.allclose(out, lam * x.astype(np.float64), atol=2e-7 * d)
    assert abs((1 + 2 * np.cos(2 * np.pi / 16)) / 3 - 0.949253) < 1e-6


def _brute_topk(v, k):
    order = sorted(range(len(v)), key=lambda i: (-abs(float(v[i])), i))
    return sorted(order[:k])


def test_choco_topk_against_sort_with_ties(orc):
    n, d = 3, 64
    g = wl.rng(5)
    x = (g.integers(-4, 5, size=(n, d)) * 0.25).astype(np.float32)      # many exact ties, zeros
    xhat = (g.integers(-2, 3, size=(n, d)) * 0.25).astype(np.float32)
    seg = [0, 10, 11, 40, 64]
    rho = 0.2
    Wm = wl.ring_matrix(n)
    out, xh = orc.gossip_mix(x, xhat, Wm, eta=0.5, keep_ratio=rho, seg_offsets=seg)
    ref_xh = xhat.copy()
    for i in range(n):
        for a, b in zip(seg[:-1], seg[1:]):
            v = x[i, a:b] - xhat[i, a:b]
            k = max(1, int(np.ceil(rho * (b - a))))
            for e in _brute_topk(v, k):
                ref_xh[i, a + e] = xhat[i, a + e] + v[e]
    assert np.array_equal(xh, ref_xh)
    W64 = Wm.astype(np.float64)          # fp32 thirds do not sum to exactly 1: keep the row sum explicit
    ref = x.astype(np.float64) + 0.5 * (W64 @ ref_xh.astype(np.float64) - W64.sum(1, keepdims=True) * ref_xh)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-14)
    # xhat moves on at most k positions per segment (a selected v may be exactly 0)
    changed = (xh != xhat)
    for i in range(n):
        for a, b in zip(seg[:-1], seg[1:]):
            assert changed[i, a:b].sum() <= max(1, int(np.ceil(rho * (b - a))))


def test_choco_counts_and_average(orc):
    n, d = 16, 4000
    x = wl.agent_params(7, n, d)
    xhat = wl.agent_params(8, n, d, spread=1e-3)
    seg = [0, 1500, 1564, 4000]
    Wm = wl.ring_matrix(n)
    out, xh = orc.gossip_mix(x, xhat, Wm, eta=0.3, keep_ratio=0.01, seg_offsets=seg)
    for a, b in zip(seg[:-1], seg[1:]):
        k = int(np.ceil(0.01 * (b - a)))
        assert ((xh[:, a:b] != xhat[:, a:b]).sum(1) == k).all()      # continuous data: no ties, no zeros
    sel = xh != xhat
    assert np.array_equal(xh[sel], (xhat + (x - xhat))[sel])
    # selected magnitudes dominate unselected ones, per agent and segment
    v = np.abs(x - xhat)
    for i in range(n):
        for a, b in zip(seg[:-1], seg[1:]):
            s = sel[i, a:b]
            assert v[i, a:b][s].min() >= v[i, a:b][~s].max()
    assert np.allclose(out.mean(0), x.astype(np.float64).mean(0), atol=1e-9)   # columns of W-I sum to 0


def test_choco_no_compression_reduces_to_plain(orc):
    n, d = 8, 300
    x = wl.agent_params(9, n, d)
    xhat = np.zeros((n, d), np.float32)          # xhat + (x - xhat) = x exactly when xhat = 0
    Wm = wl.ring_matrix(n, self_w=0.5)           # dyadic weights: fp32 row sums are exactly 1
    out, xh = orc.gossip_mix(x, xhat, Wm, eta=1.0, keep_ratio=1.0)
    plain, _ = orc.gossip_mix(x, None, Wm, eta=1.0)
    assert np.array_equal(xh, x)
    assert np.allclose(out, plain, rtol=1e-13, atol=1e-15)


def test_glue_against_library(orc):
    x = wl.images(3, 2, 9, 9, 5)
    for k, st, pd in [(2, 2, 0), (3, 2, 1)]:
        y, idx = orc.maxpool_fwd(x, k, st, pd)
        xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2).contiguous().requires_grad_()
        yt = torch.nn.functional.max_pool2d(xt, k, st, pd)
        assert np.array_equal(y, yt.detach().permute(0, 2, 3, 1).numpy().astype(np.float32))
        dy = wl.rng(4).standard_normal(y.shape)
        yt.backward(torch.from_numpy(dy).permute(0, 3, 1, 2))
        dx = orc.maxpool_bwd(dy, idx, x.shape)
        assert np.allclose(dx, xt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-13, atol=0)
    ya = orc.avgpool_fwd(x)
    assert np.allclose(ya, x.astype(np.float64).mean(axis=(1, 2)), rtol=1e-13)
    dya = wl.rng(5).standard_normal(ya.shape)
    assert np.allclose(orc.avgpool_bwd(dya, x.shape), np.broadcast_to(dya[:, None, None, :] / 81, x.shape))
    lg = wl.rng(6).standard_normal((7, 10)).astype(np.float32) * 3
    lb = wl.labels_uniform(7, 7, 10)
    loss, dl = orc.softmax_xent(lg, lb)
    lt = torch.from_numpy(lg.astype(np.float64)).requires_grad_()
    lo = torch.nn.functional.cross_entropy(lt, torch.from_numpy(lb.astype(np.int64)))
    lo.backward()
    assert abs(loss - lo.item()) < 1e-12 and np.allclose(dl, lt.grad.numpy(), rtol=1e-11, atol=1e-14)
    a, b = wl.rng(8).standard_normal(50), wl.rng(9).standard_normal(50)
    assert np.array_equal(orc.add(a, b), a + b)
    xs, gs = a.astype(np.float32), b.astype(np.float32)
    assert np.allclose(orc.sgd(xs, gs, 0.1), xs.astype(np.float64) - float(np.float32(0.1)) * gs.astype(np.float64))
