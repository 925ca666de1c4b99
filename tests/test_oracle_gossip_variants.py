"""Pins of the oracle's Deep-Squeeze, Sparse-Push and Quant-SGP steps (supplement, Algorithms "Deep-Squeeze",
"Sparse-Push", "Quant-SGP"): identities the algorithms fix, brute-force selection, and the textbook behaviour of
push-sum averaging on a directed graph."""
import math

import numpy as np

import workloads as wl


def _brute_topk(v, k):
    order = sorted(range(len(v)), key=lambda i: (-abs(float(v[i])), i))
    return sorted(order[:k])


def test_variants_without_state_reduce_to_the_pinned_mixes(orc):
    n, d = 8, 700
    x, xh = wl.agent_params(31, n, d), wl.agent_params(32, n, d, spread=2e-3)
    Wm = wl.ring_matrix(n)
    a, _ = orc.gossip_mix(x, None, Wm, eta=0.6)
    b, _, _, _ = orc.gossip_mix_ex(x, None, Wm, eta=0.6, mode=orc.MIX_PLAIN)
    assert np.allclose(a, b, rtol=0, atol=1e-15)
    a, ah = orc.gossip_mix(x, xh, Wm, eta=0.4, keep_ratio=0.05, seg_offsets=[0, 300, 700])
    b, bh, _, _ = orc.gossip_mix_ex(x, xh, Wm, eta=0.4, keep_ratio=0.05, seg_offsets=[0, 300, 700], mode=orc.MIX_CHOCO)
    assert np.array_equal(ah, bh) and np.allclose(a, b, rtol=0, atol=1e-12)


def test_deepsqueeze_selection_error_memory_and_update(orc):
    n, d, seg, rho, eta = 5, 240, [0, 7, 100, 240], 0.1, 0.3
    g = wl.rng(41)
    x = (g.integers(-9, 10, size=(n, d)) * 0.25).astype(np.float32)        # many exact ties
    delta = (g.integers(-3, 4, size=(n, d)) * 0.125).astype(np.float32)
    Wm = wl.ring_matrix(n)
    out, dnew, _, _ = orc.gossip_mix_ex(x, delta, Wm, eta=eta, keep_ratio=rho, seg_offsets=seg, mode=orc.MIX_DEEPSQUEEZE)
    v = (x + delta).astype(np.float32)                                      # one fp32 addition, as the algorithm states it
    C = np.zeros_like(v)
    for i in range(n):
        for lo, hi in zip(seg[:-1], seg[1:]):
            k = max(1, math.ceil(rho * (hi - lo)))
            for e in _brute_topk(v[i, lo:hi], k):
                C[i, lo + e] = v[i, lo + e]
    # error memory: delta + C[v] = v, bit for bit (the error-update step of the algorithm)
    assert np.array_equal(dnew + C, v) and np.array_equal(dnew, v - C)
    assert np.array_equal(dnew[C != 0], np.zeros_like(dnew[C != 0]))
    # gossip update: x + eta * (W - I) C[v]
    ref = x.astype(np.float64) + float(np.float32(eta)) * ((Wm.astype(np.float64) - np.eye(n)) @ C.astype(np.float64))
    assert np.allclose(out, ref, rtol=0, atol=1e-12)
    # a doubly stochastic W keeps the agent average, whatever is dropped
    assert np.allclose(out.mean(0), x.astype(np.float64).mean(0), rtol=0, atol=1e-6)   # fp32 thirds sum to 1 + 2e-8


def test_deepsqueeze_without_compression(orc):
    n, d = 6, 300
    x, delta = wl.agent_params(51, n, d), wl.agent_params(52, n, d, spread=1e-3) * np.float32(0.01)
    Wm = wl.ring_matrix(n)
    out, dnew, _, _ = orc.gossip_mix_ex(x, delta, Wm, eta=1.0, keep_ratio=1.0, mode=orc.MIX_DEEPSQUEEZE)
    assert not dnew.any()                                                   # everything was sent: nothing left over
    v = (x + delta).astype(np.float32).astype(np.float64)
    assert np.allclose(out, x + (Wm.astype(np.float64) - np.eye(n)) @ v, rtol=0, atol=1e-12)
    out0, _, _, _ = orc.gossip_mix_ex(x, np.zeros_like(x), Wm, eta=1.0, keep_ratio=1.0, mode=orc.MIX_DEEPSQUEEZE)
    plain, _ = orc.gossip_mix(x, None, Wm, eta=1.0)
    assert np.allclose(out0, plain, rtol=0, atol=1e-12)


def test_push_sum_weights_stay_one_on_a_doubly_stochastic_graph(orc):
    n, d = 8, 50
    x = wl.agent_params(61, n, d)
    out, _, u, z = orc.gossip_mix_ex(x, None, wl.ring_matrix(n, self_w=0.5), eta=0.7, mode=orc.MIX_PLAIN, u=np.ones(n, np.float32))
    assert np.array_equal(u, np.ones(n)) and np.array_equal(z, out)


def test_push_sum_conserves_mass_and_reaches_the_average(orc):
    """Column-stochastic W on a directed graph with unequal in-degrees: sum_i x_i and sum_i u_i are invariant, and
    repeated steps without gradients drive every de-biased model z_i = x_i/u_i to the average of the initial models
    (push-sum averaging), although the x_i themselves converge to unequal multiples of it."""
    n, d = 9, 6
    Wm = wl.directed_matrix(n)
    assert np.allclose(Wm.sum(0), 1.0, atol=1e-6) and np.abs(Wm.sum(1) - 1.0).max() > 0.1
    x0 = wl.agent_params(71, n, d, spread=0.5)
    x, u = x0.copy(), np.ones(n, np.float32)
    for it in range(120):
        out, _, un, z = orc.gossip_mix_ex(x, None, Wm, eta=1.0, mode=orc.MIX_PLAIN, u=u)
        if it == 0:
            Wd = Wm.astype(np.float64)
            assert np.allclose(out, Wd @ x0.astype(np.float64), rtol=0, atol=1e-12)
            assert np.allclose(un, Wd @ np.ones(n), rtol=0, atol=1e-12)
            assert np.allclose(z, out / un[:, None], rtol=1e-15, atol=0)
        assert abs(un.sum() - n) < 1e-4 and np.abs(out.sum(0) - x0.astype(np.float64).sum(0)).max() < 1e-4
        x, u = out.astype(np.float32), un.astype(np.float32)
    mean = x0.astype(np.float64).mean(0)
    assert np.abs(z - mean[None, :]).max() < 1e-5
    assert np.abs(x - mean[None, :]).max() > 1e-2          # the biased models do NOT agree with the average


def test_sparse_push_and_quant_sgp_compose(orc):
    """Compression and push-sum act on different things: x and the state follow the compressed algorithm on the same
    W, u follows the weight recursion, z is their quotient."""
    n, d, seg = 7, 180, [0, 60, 180]
    Wm = wl.directed_matrix(n)
    x, st = wl.agent_params(81, n, d), wl.agent_params(82, n, d, spread=2e-3)
    u = (1.0 + 0.1 * wl.rng(83).standard_normal(n)).astype(np.float32)
    for mode in (orc.MIX_CHOCO, orc.MIX_DEEPSQUEEZE):
        a, sa, _, _ = orc.gossip_mix_ex(x, st, Wm, eta=0.5, keep_ratio=0.1, seg_offsets=seg, mode=mode)
        b, sb, un, z = orc.gossip_mix_ex(x, st, Wm, eta=0.5, keep_ratio=0.1, seg_offsets=seg, mode=mode, u=u)
        assert np.array_equal(sa, sb)
        if mode == orc.MIX_DEEPSQUEEZE:
            assert np.array_equal(a, b)
        else:   # Quant-SGP mixes xhat with the operator that mixes u: x + eta (W - I) xhat_new
            ref = x.astype(np.float64) + 0.5 * ((Wm.astype(np.float64) - np.eye(n)) @ sb.astype(np.float64))
            assert np.allclose(b, ref, rtol=0, atol=1e-12)
        uref = u.astype(np.float64) + 0.5 * ((Wm.astype(np.float64) - np.eye(n)) @ u.astype(np.float64))
        assert np.allclose(un, uref, rtol=0, atol=1e-14)
        assert np.allclose(z, b / un[:, None], rtol=1e-15, atol=0)
        # column-stochastic W: the sum over agents of x is preserved by both compressed updates
        assert np.allclose(b.sum(0), x.astype(np.float64).sum(0), rtol=0, atol=1e-6)
