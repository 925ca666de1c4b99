"""GPU parity of the full-precision comparison layers (EvoNorm-S0, range batch-norm) against the oracle: 1e-4 relative
(|a-b| <= 1e-4 * max(|a|,|b|,floor)), saved positions bit-exact, results identical from run to run."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import assert_close, dev, host

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)

# N H W C groups
CASES = [
    (8, 32, 32, 16, 8),
    (4, 16, 16, 32, 8),
    (2, 28, 28, 128, 32),
    (2, 7, 7, 512, 32),
    (5, 1, 1, 512, 32),
    (2, 9, 7, 48, 6),         # C/4 = 12 does not divide 256
    (3, 70, 70, 64, 32),      # several blocks per sample with a ragged last block
    (2, 6, 6, 1024, 1),       # the widest tensor taken, one group
]


def _params(seed, C):
    g = wl.rng(seed)
    return ((1.0 + 0.3 * g.standard_normal(C)).astype(np.float32), (1.0 + 0.2 * g.standard_normal(C)).astype(np.float32),
            (0.1 * g.standard_normal(C)).astype(np.float32))


def _sum_floor(ref, count):
    # channel sums of `count` signed terms: floor at the size of their random walk
    return max(float(np.abs(ref).max()) * 1e-2, 1e-3 * np.sqrt(count) * float(np.abs(ref).max()) / max(count, 1))


@pytest.mark.parametrize("shape", CASES)
def test_evonorm_s0(orc, shape):
    N, H, W, C, groups = shape
    print("case", shape, flush=True)
    x = wl.images(1100, N, H, W, C) * np.float32(2.0) + np.float32(0.3)
    v, gamma, beta = _params(1101, C)
    dy = wl.upstream_grad(1102, (N, H, W, C))
    y_ref, m_ref, var_ref = orc.evonorm_s0_fwd(x, groups, v, gamma, beta, 1e-5)
    y, mean, var = lpdt.evonorm_s0_fwd(dev(x), groups, dev(v), dev(gamma), dev(beta), 1e-5)
    assert_close(host(mean), m_ref, 1e-5, float(np.abs(x).max()) * 1e-2, "mean")
    assert_close(host(var), var_ref, 1e-5, 0.0, "var")
    assert_close(host(y), y_ref, 1e-4, float(np.abs(y_ref).max()) * 1e-2, "y")
    dx_ref, dv_ref, dg_ref, db_ref = orc.evonorm_s0_bwd(dy.astype(np.float64), x, groups, v, gamma, 1e-5)
    dx, dv, dg, db = lpdt.evonorm_s0_bwd(dev(dy), dev(x), groups, dev(v), dev(gamma), mean, var, 1e-5)
    assert_close(host(dx), dx_ref, 1e-4, float(np.abs(dx_ref).max()) * 1e-2, "dx")
    for got, ref, name in ((dv, dv_ref, "dv"), (dg, dg_ref, "dgamma"), (db, db_ref, "dbeta")):
        assert_close(host(got), ref, 1e-4, _sum_floor(ref, N * H * W), name)
    again = lpdt.evonorm_s0_bwd(dev(dy), dev(x), groups, dev(v), dev(gamma), mean, var, 1e-5)
    assert all(torch.equal(a, b) for a, b in zip((dx, dv, dg, db), again)), "fixed-order reductions: identical bits"


@pytest.mark.parametrize("shape", [c for c in CASES if c[0] >= 2])
def test_range_bn(orc, shape):
    N, H, W, C, _ = shape
    print("case", shape, flush=True)
    x = wl.images(1110, N, H, W, C) * np.float32(2.0) - np.float32(0.4)
    _, gamma, beta = _params(1111, C)
    dy = wl.upstream_grad(1112, (N, H, W, C))
    y_ref, m_ref, r_ref, amx_ref, amn_ref = orc.range_bn_fwd(x, gamma, beta, 1e-5)
    y, mean, rng, amx, amn = lpdt.range_bn_fwd(dev(x), dev(gamma), dev(beta), 1e-5)
    assert np.array_equal(host(amx), amx_ref) and np.array_equal(host(amn), amn_ref)
    assert_close(host(rng), r_ref, 1e-6, 0.0, "range")
    assert_close(host(mean), m_ref, 1e-5, float(np.abs(x).max()) * 1e-2, "mean")
    assert_close(host(y), y_ref, 1e-4, float(np.abs(y_ref).max()) * 1e-2, "y")
    dx_ref, dg_ref, db_ref = orc.range_bn_bwd(dy.astype(np.float64), x, gamma, 1e-5)
    dx, dg, db = lpdt.range_bn_bwd(dev(dy), dev(x), dev(gamma), mean, rng, amx, amn, 1e-5)
    assert_close(host(dx), dx_ref, 1e-4, float(np.abs(dx_ref).max()) * 1e-2, "dx")
    for got, ref, name in ((dg, dg_ref, "dgamma"), (db, db_ref, "dbeta")):
        assert_close(host(got), ref, 1e-4, _sum_floor(ref, N * H * W), name)
    again = lpdt.range_bn_bwd(dev(dy), dev(x), dev(gamma), mean, rng, amx, amn, 1e-5)
    assert all(torch.equal(a, b) for a, b in zip((dx, dg, db), again))


def test_range_bn_ties_take_first_position(orc):
    # values on a coarse grid: many equal extrema per channel, spread over samples and blocks
    N, H, W, C = 3, 40, 40, 8
    x = (wl.rng(1120).integers(-3, 4, size=(N, H, W, C)) * 0.5).astype(np.float32)
    _, _, r_ref, amx_ref, amn_ref = orc.range_bn_fwd(x, np.ones(C), np.zeros(C), 0.0)
    _, _, rng, amx, amn = lpdt.range_bn_fwd(dev(x), dev(np.ones(C, np.float32)), dev(np.zeros(C, np.float32)), 0.0)
    assert np.array_equal(host(amx), amx_ref) and np.array_equal(host(amn), amn_ref)
    assert np.array_equal(host(rng).astype(np.float64), r_ref)


def test_limits_and_errors():
    z = torch.zeros((2, 4, 4, 8), dtype=torch.float32, device="cuda")
    p = torch.ones(8, dtype=torch.float32, device="cuda")
    # a constant tensor: variance 0; with eps > 0 everything stays finite
    y, mean, var = lpdt.evonorm_s0_fwd(z + 1.5, 2, p, p, p, 1e-3)
    assert torch.isfinite(y).all() and float(var.abs().max()) < 1e-6 and abs(float(mean[0, 0]) - 1.5) < 1e-6
    for bad in (lambda: lpdt.evonorm_s0_fwd(torch.zeros((2, 4, 4, 6), device="cuda"), 2, p, p, p),        # C % 4
                lambda: lpdt.evonorm_s0_fwd(z, 3, p, p, p),                                                 # groups
                lambda: lpdt.range_bn_fwd(z[:1].contiguous(), p, p)):                                       # batch of one
        with pytest.raises(lpdt.LpdtError):
            bad()
