"""The numpy one-by-one evaluators (used where the full sizes make the C oracle's loops too slow) against the C oracle
and against brute force."""
import numpy as np

import workloads as wl
from oracle import sampled


def test_sampled_conv_outputs_match_the_oracle(orc):
    for shp in [(2, 16, 9, 11, 24, 3, 3, 1, 1), (2, 8, 15, 14, 16, 3, 3, 2, 1), (1, 3, 20, 20, 8, 7, 7, 2, 3), (3, 32, 6, 6, 16, 1, 1, 2, 0)]:
        N, C, H, W, K, R, S, st, pd = shp
        P, Q = wl.conv_out(H, pd, R, st), wl.conv_out(W, pd, S, st)
        x, w, g = wl.int8_codes(1, (N, H, W, C), "uniform"), wl.int8_codes(2, (K, R, S, C), "uniform"), wl.int8_codes(3, (N, P, Q, K), "uniform")
        d = orc.conv_desc(*shp)
        rng = wl.rng(9)
        co = [(rng.integers(N), rng.integers(P), rng.integers(Q), rng.integers(K)) for _ in range(60)] + [(0, 0, 0, 0), (N - 1, P - 1, Q - 1, K - 1)]
        full = orc.qconv_fwd(d, x, w)
        assert np.array_equal(sampled.qconv_fwd_at(x, w, st, pd, co), [full[c] for c in co])
        ci = [(rng.integers(N), rng.integers(H), rng.integers(W), rng.integers(C)) for _ in range(60)] + [(0, 0, 0, 0), (N - 1, H - 1, W - 1, C - 1)]
        full = orc.qconv_bwd_data(d, g, w)
        assert np.array_equal(sampled.qconv_bwd_data_at(g, w, H, W, st, pd, ci), [full[c] for c in ci])
        cw = [(rng.integers(K), rng.integers(R), rng.integers(S), rng.integers(C)) for _ in range(40)] + [(0, 0, 0, 0), (K - 1, R - 1, S - 1, C - 1)]
        full = orc.qconv_bwd_weight(d, g, x)
        assert np.array_equal(sampled.qconv_bwd_weight_at(g, x, R, S, st, pd, cw), [full[c] for c in cw])


def test_topk_mask_is_the_sorted_rule(orc):
    g = wl.rng(4)
    for n, k in [(1, 1), (10, 3), (1000, 10), (1000, 1000), (5000, 4999)]:
        v = (g.integers(-5, 6, size=n) * 0.25).astype(np.float32)          # heavy ties, zeros, both signs
        order = sorted(range(n), key=lambda i: (-abs(float(v[i])), i))
        ref = np.zeros(n, bool)
        ref[order[:k]] = True
        assert np.array_equal(sampled.topk_mask(v, k), ref)
    # and it is the selection the C oracle makes
    x, xh = wl.agent_params(5, 3, 4000), wl.agent_params(6, 3, 4000, spread=2e-3)
    _, xh_new = orc.gossip_mix(x, xh, wl.ring_matrix(3), eta=0.5, keep_ratio=0.02, seg_offsets=[0, 1500, 4000])
    for i in range(3):
        for lo, hi in ((0, 1500), (1500, 4000)):
            m = sampled.topk_mask((x[i, lo:hi] - xh[i, lo:hi]).astype(np.float32), int(np.ceil(0.02 * (hi - lo))))
            assert np.array_equal(xh_new[i, lo:hi] != xh[i, lo:hi], m & ((x[i, lo:hi] - xh[i, lo:hi]) != 0))
