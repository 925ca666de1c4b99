"""GPU parity of the Deep-Squeeze, Sparse-Push and Quant-SGP gossip steps against the oracle: the state matrix (error
memory / xhat) bit-exact, models, push-sum weights and de-biased models to fp32 rounding."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import assert_close, dev, host

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)


def _case(orc, mode, n, d, seg, rho, rate, seed, Wm, push, ties=False):
    if ties:
        g = wl.rng(seed)
        x = (g.integers(-6, 7, size=(n, d)) * 0.125).astype(np.float32)
        st = (g.integers(-2, 3, size=(n, d)) * 0.125).astype(np.float32)
    else:
        x = wl.agent_params(seed, n, d)
        st = wl.agent_params(seed + 1, n, d, spread=2e-3)
        if mode == orc.MIX_DEEPSQUEEZE:
            st = (st * np.float32(0.05)).astype(np.float32)       # an error memory is small next to the model
    if mode == orc.MIX_PLAIN:
        st = None
    u = (1.0 + 0.2 * wl.rng(seed + 2).random(n)).astype(np.float32) if push else None
    rx, rs, ru, rz = orc.gossip_mix_ex(x, st, Wm, eta=rate, keep_ratio=rho, seg_offsets=seg, mode=mode, u=u)
    xd, sd = dev(x), (None if st is None else dev(st))
    ud = None if u is None else dev(u)
    zd = torch.empty_like(xd) if push else None
    lpdt.gossip_mix_ex(xd, sd, Wm, rate=rate, keep_ratio=rho, seg_offsets=seg, mode=mode, u=ud, z=zd)
    if st is not None:
        assert np.array_equal(host(sd), rs), "state (selection and update) must be bit-exact"
    floor = float(np.abs(x).max())
    assert_close(host(xd), rx, 1e-5, floor, "mixed models")
    if push:
        assert_close(host(ud), ru, 1e-6, 1.0, "push-sum weights")
        assert_close(host(zd), rz, 1e-5, floor, "de-biased models")


SEG = [0, 432, 448, 464, 2784, 2800, 20000, 20001, 20001, 20010, 30000]


@pytest.mark.parametrize("n,topo", [(16, "ring"), (9, "directed"), (33, "ring")])
def test_deepsqueeze(orc, n, topo):
    Wm = wl.ring_matrix(n) if topo == "ring" else wl.directed_matrix(n)
    push = topo == "directed"
    _case(orc, orc.MIX_DEEPSQUEEZE, n, 30000, SEG, 0.01, 0.3, 900 + n, Wm, push)
    _case(orc, orc.MIX_DEEPSQUEEZE, n, 30000, SEG, 0.1, 0.5, 910 + n, Wm, push)
    _case(orc, orc.MIX_DEEPSQUEEZE, n, 5001, None, 1.0, 1.0, 920 + n, Wm, push)            # nothing dropped
    _case(orc, orc.MIX_DEEPSQUEEZE, n, 9000, [0, 100, 4500, 9000], 0.05, 0.4, 930 + n, Wm, push, ties=True)


@pytest.mark.parametrize("stride", [1, 2])
def test_deepsqueeze_one_pass_selection(orc, stride):
    # the top-k window guessed from a sample of the tiles (forced here at a small size); exact like the two-pass form
    lpdt.gossip_set_sample_stride(stride)
    try:
        _case(orc, orc.MIX_DEEPSQUEEZE, 16, 30000, SEG, 0.01, 0.3, 916, wl.ring_matrix(16), False)
        _case(orc, orc.MIX_DEEPSQUEEZE, 9, 30000, SEG, 0.1, 0.5, 919, wl.directed_matrix(9), True)
        _case(orc, orc.MIX_DEEPSQUEEZE, 5, 9000, [0, 100, 4500, 9000], 0.05, 0.4, 935, wl.ring_matrix(5), False, ties=True)
    finally:
        lpdt.gossip_set_sample_stride(-1)


@pytest.mark.parametrize("n", [7, 16])
def test_quant_sgp_and_sparse_push_on_a_directed_graph(orc, n):
    Wm = wl.directed_matrix(n)
    assert np.abs(Wm.sum(1) - 1).max() > 0.1                          # rows do not sum to 1: push-sum is needed
    for mode in (orc.MIX_CHOCO, orc.MIX_DEEPSQUEEZE, orc.MIX_PLAIN):
        _case(orc, mode, n, 30000, SEG if mode != orc.MIX_PLAIN else None, 0.02, 0.4, 940 + n + mode, Wm, True)


def test_push_sum_with_doubly_stochastic_graph_keeps_weights(orc):
    n, d = 16, 10000
    x = wl.agent_params(960, n, d)
    xd, ud, zd = dev(x), dev(np.ones(n, np.float32)), torch.empty(n, d, device="cuda")
    lpdt.gossip_mix_ex(xd, None, wl.ring_matrix(n, self_w=0.5), rate=1.0, mode=lpdt.MIX_PLAIN, u=ud, z=zd)
    assert np.array_equal(host(ud), np.ones(n, np.float32)) and torch.equal(zd, xd)


def test_ex_modes_equal_the_plain_entry_point(orc):
    n, d = 16, 30000
    x, xh = wl.agent_params(970, n, d), wl.agent_params(971, n, d, spread=2e-3)
    Wm = wl.ring_matrix(n)
    a, ah = dev(x), dev(xh)
    b, bh = dev(x), dev(xh)
    lpdt.gossip_mix(a, ah, Wm, rate=0.3, keep_ratio=0.01, seg_offsets=SEG)
    lpdt.gossip_mix_ex(b, bh, Wm, rate=0.3, keep_ratio=0.01, seg_offsets=SEG, mode=lpdt.MIX_CHOCO)
    assert torch.equal(a, b) and torch.equal(ah, bh)
    a, b = dev(x), dev(x)
    lpdt.gossip_mix(a, None, Wm, rate=0.7)
    lpdt.gossip_mix_ex(b, None, Wm, rate=0.7, mode=lpdt.MIX_PLAIN)
    assert torch.equal(a, b)
