"""Pins of the oracle's three integer convolutions (Table "hardware_training", row Conv:
forward, gradient w.r.t. the layer input, gradient w.r.t. the filter)."""
import numpy as np
import pytest
import torch

import workloads as wl

CASES = [
    # N C H W K R S stride pad
    (2, 3, 7, 7, 4, 3, 3, 1, 1),
    (1, 5, 9, 8, 3, 3, 3, 2, 1),
    (2, 4, 11, 11, 6, 7, 7, 2, 3),
    (3, 8, 6, 5, 5, 1, 1, 1, 0),
    (2, 6, 8, 8, 4, 1, 1, 2, 0),
    (1, 2, 5, 5, 2, 3, 3, 1, 0),
    (2, 16, 6, 6, 16, 3, 3, 1, 1),
]


def _case(orc, shp, seed, kind="uniform"):
    N, C, H, W, K, R, S, st, pd = shp
    d = orc.conv_desc(N, C, H, W, K, R, S, st, pd)
    x = wl.int8_codes(seed, (N, H, W, C), kind)
    w = wl.int8_codes(seed + 1, (K, R, S, C), kind)
    g = wl.int8_codes(seed + 2, (N, d.P, d.Q, K), kind)
    return d, x, w, g


def _torch_ref(d, x, w, g):
    """float64 library convolution on integer-valued tensors is exact (|acc| << 2^53)."""
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2).contiguous().requires_grad_()
    wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2).contiguous().requires_grad_()
    y = torch.nn.functional.conv2d(xt, wt, stride=d.stride_h, padding=d.pad_h)
    gt = torch.from_numpy(g.astype(np.float64)).permute(0, 3, 1, 2)
    y.backward(gt)
    f = lambda t: np.rint(t.detach().permute(0, 2, 3, 1).numpy()).astype(np.int64)
    return f(y), f(xt.grad), f(wt.grad)


@pytest.mark.parametrize("shp", CASES)
@pytest.mark.parametrize("kind", ["uniform", "extreme"])
def test_against_float64_library_conv(orc, shp, kind):
    d, x, w, g = _case(orc, shp, 100, kind)
    y, dx, dw = _torch_ref(d, x, w, g)
    assert np.array_equal(orc.qconv_fwd(d, x, w), y)
    assert np.array_equal(orc.qconv_bwd_data(d, g, w), dx)
    assert np.array_equal(orc.qconv_bwd_weight(d, g, x), dw)


def _brute_fwd(d, x, w):
    acc = np.zeros((d.N, d.P, d.Q, d.K), np.int64)
    for n in range(d.N):
        for p in range(d.P):
            for q in range(d.Q):
                for k in range(d.K):
                    s = 0
                    for r in range(d.R):
                        for t in range(d.S):
                            h, ww = p * d.stride_h + r - d.pad_h, q * d.stride_w + t - d.pad_w
                            if 0 <= h < d.H and 0 <= ww < d.W:
                                s += int(np.dot(x[n, h, ww].astype(np.int64), w[k, r, t].astype(np.int64)))
                    acc[n, p, q, k] = s
    return acc


def test_brute_force_tiny(orc):
    for shp in [(1, 2, 4, 5, 3, 3, 3, 1, 1), (2, 3, 5, 5, 2, 3, 3, 2, 1), (1, 1, 7, 7, 1, 7, 7, 2, 3)]:
        d, x, w, g = _case(orc, shp, 7)
        assert np.array_equal(orc.qconv_fwd(d, x, w), _brute_fwd(d, x, w))


@pytest.mark.parametrize("shp", CASES)
def test_adjoint_identities(orc, shp):
    # <G, fwd(X,W)> = <bwd_data(G,W), X> = <bwd_weight(G,X), W> in exact integers
    d, x, w, g = _case(orc, shp, 200)
    i64 = lambda a: a.astype(np.int64)
    a = (i64(g) * i64(orc.qconv_fwd(d, x, w))).sum()
    b = (i64(orc.qconv_bwd_data(d, g, w)) * i64(x)).sum()
    c = (i64(orc.qconv_bwd_weight(d, g, x)) * i64(w)).sum()
    assert a == b == c


def test_1x1_is_integer_matmul(orc):
    N, C, K = 37, 24, 11
    d = orc.conv_desc(N, C, 1, 1, K, 1, 1, 1, 0)
    x = wl.int8_codes(5, (N, 1, 1, C), "uniform")
    w = wl.int8_codes(6, (K, 1, 1, C), "uniform")
    g = wl.int8_codes(7, (N, 1, 1, K), "uniform")
    X, Wm, G = (t.reshape(t.shape[0], -1).astype(np.int64) for t in (x, w, g))
    assert np.array_equal(orc.qconv_fwd(d, x, w).reshape(N, K), X @ Wm.T)
    assert np.array_equal(orc.qconv_bwd_data(d, g, w).reshape(N, C), G @ Wm)
    assert np.array_equal(orc.qconv_bwd_weight(d, g, x).reshape(K, C), G.T @ X)


def test_delta_filter_shifts(orc):
    # filter = 1 at tap (r0,s0), channel c->k identity: output is the input shifted, zero padded
    N, C, H, W = 1, 3, 6, 7
    d = orc.conv_desc(N, C, H, W, C, 3, 3, 1, 1)
    x = wl.int8_codes(9, (N, H, W, C), "uniform")
    for r0, s0 in [(0, 0), (1, 1), (2, 0), (1, 2)]:
        w = np.zeros((C, 3, 3, C), np.int8)
        for c in range(C):
            w[c, r0, s0, c] = 1
        y = orc.qconv_fwd(d, x, w)
        ref = np.zeros_like(y)
        for p in range(H):
            for q in range(W):
                h, ww = p + r0 - 1, q + s0 - 1
                if 0 <= h < H and 0 <= ww < W:
                    ref[0, p, q] = x[0, h, ww]
        assert np.array_equal(y, ref)


def test_overflow_is_reported(orc):
    # 127*127*L exceeds int32 once L > 133144: the oracle refuses rather than wrap
    L = 133145
    d = orc.conv_desc(1, L, 1, 1, 1, 1, 1, 1, 0)
    x = np.full((1, 1, 1, L), 127, np.int8)
    w = np.full((1, 1, 1, L), 127, np.int8)
    with pytest.raises(orc.OracleError):
        orc.qconv_fwd(d, x, w)
    d2 = orc.conv_desc(1, L - 1, 1, 1, 1, 1, 1, 1, 0)
    assert orc.qconv_fwd(d2, x[..., :-1], w[..., :-1])[0, 0, 0, 0] == 127 * 127 * (L - 1)
