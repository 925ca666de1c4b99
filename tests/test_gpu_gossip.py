"""GPU parity of the gossip step (plain and CHOCO top-k) and of the glue layers against the oracle."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import assert_close, dev, host

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)


@pytest.mark.parametrize("n,d,topo", [(16, 272_474, "ring"), (8, 1000, "ring"), (16, 5003, "torus"), (3, 17, "ring"),
                                      (33, 2049, "ring"), (64, 300, "ring")])
@pytest.mark.parametrize("rate", [1.0, 0.37])
def test_plain_mix(orc, n, d, topo, rate):
    x = wl.agent_params(800, n, d)
    Wm = wl.ring_matrix(n) if topo == "ring" else wl.torus_matrix(4, 4)
    ref, _ = orc.gossip_mix(x, None, Wm, eta=rate)
    xd = dev(x)
    lpdt.gossip_mix(xd, None, Wm, rate=rate)
    # x + rate*(sum_j W_ij x_j - x_i): a few fp32 roundings of terms of size max|x|
    assert_close(host(xd), ref, 1e-5, float(np.abs(x).max()), "plain mix")
    assert np.abs(host(xd).astype(np.float64).mean(0) - x.astype(np.float64).mean(0)).max() < 1e-6


def _choco_case(orc, n, d, seg, rho, rate, seed, ties=False):
    if ties:
        g = wl.rng(seed)
        x = (g.integers(-6, 7, size=(n, d)) * 0.125).astype(np.float32)
        xhat = (g.integers(-2, 3, size=(n, d)) * 0.125).astype(np.float32)
    else:
        x = wl.agent_params(seed, n, d)
        xhat = wl.agent_params(seed + 1, n, d, spread=2e-3)
    Wm = wl.ring_matrix(n)
    ref_x, ref_h = orc.gossip_mix(x, xhat, Wm, eta=rate, keep_ratio=rho, seg_offsets=seg)
    xd, hd = dev(x), dev(xhat)
    lpdt.gossip_mix(xd, hd, Wm, rate=rate, keep_ratio=rho, seg_offsets=seg)
    assert np.array_equal(host(hd), ref_h), "xhat (top-k membership and update) must be bit-exact"
    assert_close(host(xd), ref_x, 1e-5, float(np.abs(x).max()), "choco mix")


def test_choco_layerwise_topk(orc):
    # segments shaped like a small conv net's parameter tensors, including tiny ones
    seg = [0, 432, 448, 464, 480, 2784, 2800, 2816, 2832, 20000, 20001, 20001, 20010, 60000]
    _choco_case(orc, 16, 60000, seg, 0.01, 0.3, 810)
    _choco_case(orc, 16, 60000, seg, 0.1, 0.5, 812)


def test_choco_global_topk_and_ties(orc):
    _choco_case(orc, 8, 100_003, None, 0.01, 0.2, 820)
    _choco_case(orc, 5, 9000, [0, 100, 4500, 9000], 0.05, 0.4, 822, ties=True)   # massive exact ties, zeros
    _choco_case(orc, 4, 3000, [0, 3000], 0.999, 1.0, 824, ties=True)
    # thousands of equal magnitudes around the threshold: more survivors than the refinement keeps on chip
    _choco_case(orc, 3, 60000, [0, 60000], 0.3, 0.5, 826, ties=True)
    _choco_case(orc, 2, 50000, [0, 10, 50000], 0.5, 0.5, 828, ties=True)


@pytest.fixture
def sample_stride():
    """Forces the one-pass top-k (window of bins guessed from every s-th 4096-element tile) at any size; back to the
    library's own choice afterwards."""
    yield lpdt.gossip_set_sample_stride
    lpdt.gossip_set_sample_stride(-1)


@pytest.mark.parametrize("stride", [1, 3, 16])
def test_choco_one_pass_selection(orc, sample_stride, stride):
    # the same cases as the two-pass form: the selection is exact whichever path finds it
    sample_stride(stride)
    seg = [0, 432, 448, 464, 480, 2784, 2800, 2816, 2832, 20000, 20001, 20001, 20010, 60000]
    _choco_case(orc, 16, 60000, seg, 0.01, 0.3, 810)
    _choco_case(orc, 8, 100_003, None, 0.01, 0.2, 820)
    _choco_case(orc, 5, 9000, [0, 100, 4500, 9000], 0.05, 0.4, 822, ties=True)
    _choco_case(orc, 3, 60000, [0, 60000], 0.3, 0.5, 826, ties=True)
    _choco_case(orc, 2, 50000, [0, 10, 50000], 0.5, 0.5, 828, ties=True)
    _choco_case(orc, 6, 300_000, [0, 150_000, 150_064, 300_000], 0.01, 0.7, 832)
    _choco_case(orc, 4, 200_000, [0, 200_000], 0.002, 1.0, 834)


@pytest.mark.parametrize("stride", [0, 1, 8])
def test_choco_many_tiny_segments_in_one_tile(orc, sample_stride, stride):
    """More segment boundaries inside a 4096-element tile than the kernels keep at hand (32): the rest is walked from
    memory; empty segments in between; then long segments again."""
    sample_stride(stride)
    g = wl.rng(850)
    lens = [5000] + [int(v) for v in g.integers(1, 60, size=90)] + [0, 0, 7] + [int(v) for v in g.integers(1, 40, size=70)] + [9000, 3, 12000]
    seg = [0]
    for n_ in lens:
        seg.append(seg[-1] + n_)
    d = seg[-1]
    _choco_case(orc, 5, d, seg, 0.1, 0.4, 852)
    _choco_case(orc, 3, d, seg, 0.01, 0.9, 854)
    _choco_case(orc, 2, d, seg, 0.5, 0.5, 856, ties=True)


@pytest.mark.parametrize("stride", [0, 2])
def test_choco_more_segments_than_one_set_up_launch_carries(orc, sample_stride, stride):
    """The segment table, the per-segment k and the sampled tiles normally travel in one kernel-argument chunk (384 values)
    with the set-up launch; 260 segments do not fit, and the tables go up in launches of their own."""
    sample_stride(stride)
    g = wl.rng(860)
    lens = [int(v) for v in g.integers(1, 400, size=257)] + [9000, 0, 6000]
    seg = [0]
    for n_ in lens:
        seg.append(seg[-1] + n_)
    d = seg[-1]
    _choco_case(orc, 4, d, seg, 0.05, 0.4, 862)
    _choco_case(orc, 2, d, seg, 0.3, 0.8, 864, ties=True)


@pytest.mark.parametrize("loud", ["unsampled", "sampled"])
def test_choco_one_pass_window_misses(orc, sample_stride, loud):
    """Sampled tiles that say nothing about the rest: the guessed window misses the threshold bin and the pair is
    collected a second time; other pairs of the same call keep their first collection."""
    sample_stride(4)
    n, tile, ntiles = 3, 4096, 24
    d = tile * ntiles + 1000
    seg = [0, tile * 12, d]
    g = wl.rng(840)
    x = (g.standard_normal((n, d)) * 1e-3).astype(np.float32)
    xhat = np.zeros((n, d), np.float32)
    big = np.zeros(d, bool)
    for t in range(12):   # first segment only: tiles 0, 4, 8 are the sampled ones
        if (t % 4 == 0) == (loud == "sampled"):
            big[t * tile:(t + 1) * tile] = True
    x[:, big] *= 1000.0
    Wm = wl.ring_matrix(n)
    for rho in (0.01, 0.2, 0.6):
        ref_x, ref_h = orc.gossip_mix(x, xhat, Wm, eta=0.5, keep_ratio=rho, seg_offsets=seg)
        xd, hd = dev(x), dev(xhat)
        lpdt.gossip_mix(xd, hd, Wm, rate=0.5, keep_ratio=rho, seg_offsets=seg)
        assert np.array_equal(host(hd), ref_h), f"rho={rho}: xhat must be bit-exact"
        assert_close(host(xd), ref_x, 1e-5, float(np.abs(x).max()), "choco mix")


def test_choco_no_compression(orc):
    _choco_case(orc, 8, 5000, [0, 1200, 5000], 1.0, 1.0, 830)


def test_glue(orc):
    for C in (20, 7):   # 16-byte path (4 channels per thread) and the any-shape path
        xp = wl.images(840 + C, 3, 9, 9, C)
        xp[0, 2:5, 2:5, :] = 0.5   # ties inside windows: the first position in window order wins
        for k, st, pd in [(2, 2, 0), (3, 2, 1), (3, 1, 1)]:
            y_ref, idx_ref = orc.maxpool_fwd(xp, k, st, pd)
            y, idx = lpdt.maxpool_fwd(dev(xp), k, st, pd)
            assert np.array_equal(host(y), y_ref) and np.array_equal(host(idx), idx_ref)
            dy = wl.upstream_grad(841, y_ref.shape)
            dx = lpdt.maxpool_bwd(dev(dy), idx, xp.shape, k, st, pd)
            # a position can win several windows: its gradient is a short fp32 sum, so the floor is the size of a summand
            assert_close(host(dx), orc.maxpool_bwd(dy.astype(np.float64), idx_ref, xp.shape), 1e-6, float(np.abs(dy).max()),
                         "maxpool bwd")
    x = wl.images(840, 3, 9, 9, 20)
    assert_close(host(lpdt.avgpool_fwd(dev(x))), orc.avgpool_fwd(x), 1e-5, 1e-2, "avgpool fwd")
    dya = wl.upstream_grad(842, (3, 20))
    assert_close(host(lpdt.avgpool_bwd(dev(dya), x.shape)), orc.avgpool_bwd(dya.astype(np.float64), x.shape), 1e-6, 0.0, "avgpool bwd")
    for N, classes in [(7, 10), (64, 100)]:
        lg = (wl.rng(843).standard_normal((N, classes)) * 3).astype(np.float32)
        lb = wl.labels_uniform(844, N, classes)
        loss_ref, dl_ref = orc.softmax_xent(lg, lb)
        loss, dl = lpdt.softmax_xent(dev(lg), dev(lb))
        assert abs(host(loss)[0] - loss_ref) < 1e-5 * max(1.0, abs(loss_ref))
        assert_close(host(dl), dl_ref, 1e-4, 1e-3 / N, "dlogits")
        # labels outside [0, classes) are not dereferenced: NaN loss for those samples, gradient rows without a target term,
        # every other sample as before
        bad = lb.copy()
        bad[0], bad[N - 1] = -1, classes
        loss_b, dl_b = lpdt.softmax_xent(dev(lg), dev(bad))
        loss_b, dl_b = host(loss_b), host(dl_b)
        assert np.isnan(loss_b[0]) and np.isnan(loss_b[1]) and np.isnan(loss_b[N])
        assert np.array_equal(loss_b[2:N], host(loss)[2:N]) and np.array_equal(dl_b[1:N - 1], host(dl)[1:N - 1])
        sm = np.exp(lg[0].astype(np.float64) - lg[0].max()); sm /= sm.sum()
        assert_close(dl_b[0], sm / N, 1e-4, 1e-3 / N, "dlogits of a sample without a valid label")
    a, b = wl.images(845, 2, 5, 5, 7), wl.images(846, 2, 5, 5, 7)
    # 350 elements: exercises the scalar tail
    assert np.array_equal(host(lpdt.add(dev(a), dev(b))), (a + b))
    p = dev(a.copy())
    lpdt.sgd(p, dev(b), 0.1)
    assert_close(host(p), orc.sgd(a, b, 0.1), 1e-6, 1e-2, "sgd")
