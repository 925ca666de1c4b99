"""lpdt_qconv_ren_fwd_q, the chain convolution -> Range-EvoNorm -> quantizer in one call, against the calls it stands
for (bit for bit: y, codes, scale, range, first arg-max / arg-min) and against the oracle's Range-EvoNorm on the same y."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev, host

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)

# shape, groups, expected lpdt_qconv_kernel_id(d, 3): 41 / 42 / 43 / 44 = the statistics ride in the epilogue of the 128x128
# (8 waves), 128x128 (4 waves, tile staged in two runs), 64x128 and 256x128 (staged in four runs) tiles; anything else runs
# the two calls
CASES = [
    ((16, 128, 28, 28, 256, 3, 3, 1, 1), 32, 41),    # 784 pixels per sample: a tile touches up to 2 samples
    ((16, 64, 56, 56, 128, 3, 3, 1, 1), 32, 42),
    ((16, 256, 14, 14, 512, 3, 3, 1, 1), 32, 43),    # 196 pixels per sample, 64-pixel tiles
    ((64, 512, 7, 7, 512, 3, 3, 1, 1), 32, 43),      # 49 pixels per sample: up to 3 samples per tile
    ((64, 512, 7, 7, 512, 3, 3, 1, 1), 256, 43),     # two channels per group
    ((8, 64, 56, 56, 512, 3, 3, 1, 1), 32, 44),      # GEMM-like launch with a short reduction
    ((40, 128, 28, 28, 512, 1, 1, 1, 0), 64, 44),    # 784 pixels per sample on 256-pixel tiles: up to 2 samples per tile
    ((16, 128, 28, 28, 256, 3, 3, 2, 1), 32, 12),    # too few tiles for the fused form at this batch: the two calls
    ((2, 64, 14, 14, 64, 3, 3, 1, 1), 8, 11),
    ((3, 384, 5, 5, 64, 3, 3, 1, 1), 8, 112),        # the two calls, the product with a split reduction
    ((3, 3, 20, 20, 16, 3, 3, 1, 1), 4, 1),          # first-layer kernel
]


@pytest.mark.parametrize("shp,groups,kid", CASES)
@pytest.mark.parametrize("accumulate", [False, True])
def test_chain_equals_the_separate_calls(orc, shp, groups, kid, accumulate):
    N, C, H, W, K, R, S, st, pd = shp
    ld = lpdt.ConvDesc.make(*shp)
    assert lpdt.qconv_kernel_id(ld, 3) == kid, "the planner changed: update CASES"
    seed = 4000 + sum(shp) + groups
    x, w = wl.int8_codes(seed, (N, H, W, C), "gauss"), wl.int8_codes(seed + 1, (K, R, S, C), "gauss")
    g = wl.rng(seed + 2)
    v, gamma, beta = ((1.0 + 0.3 * g.standard_normal(K)).astype(np.float32), (1.0 + 0.2 * g.standard_normal(K)).astype(np.float32),
                      (0.1 * g.standard_normal(K)).astype(np.float32))
    sx, sw = dev(np.array([0.021], np.float32)), dev(np.array([0.0037], np.float32))
    xd, wd, vd, gd, bd = dev(x), dev(w), dev(v), dev(gamma), dev(beta)
    base = dev(wl.images(seed + 3, N, ld.P, ld.Q, K)) if accumulate else None
    # the calls it stands for
    if accumulate:
        y_ref = lpdt.qconv_fwd_f32_add(ld, xd, wd, sx, sw, base.clone())
    else:
        y_ref = lpdt.qconv_fwd_f32(ld, xd, wd, sx, sw)
    z_ref = torch.empty_like(y_ref)
    q_ref, s_ref, r_ref, amx_ref, amn_ref = lpdt.range_evonorm_fwd_q(y_ref, groups, vd, gd, bd, 1e-5, y=z_ref)
    print("chain", shp, groups, accumulate, flush=True)
    z = torch.empty_like(y_ref) if accumulate else None      # the normalised fp32 output is optional
    y, q, s, r, amx, amn = lpdt.qconv_ren_fwd_q(ld, xd, wd, sx, sw, groups, vd, gd, bd, 1e-5,
                                                y=base.clone() if accumulate else None, accumulate=accumulate, z=z)
    assert torch.equal(y, y_ref), "conv output"
    assert z is None or torch.equal(z, z_ref), "normalised output"
    assert torch.equal(r, r_ref), "range"
    assert torch.equal(amx, amx_ref) and torch.equal(amn, amn_ref), "positions of the extremes"
    assert torch.equal(s, s_ref) and torch.equal(q, q_ref), "codes and scale"
    # and the oracle's statistics of the same y: quantized conv outputs tie massively, the first position must win
    if N * ld.P * ld.Q * K <= 4_000_000:
        _, r_o, amx_o, amn_o = orc.range_evonorm_fwd(host(y), groups, v, gamma, beta, 1e-5)
        assert np.array_equal(host(amx), amx_o) and np.array_equal(host(amn), amn_o)
        assert np.allclose(host(r), r_o, rtol=1e-6, atol=0)


def test_chain_twice_in_a_row_reuses_its_workspace():
    # the statistics array in the workspace is cleared by every call
    shp, groups = (16, 128, 28, 28, 256, 3, 3, 1, 1), 32
    ld = lpdt.ConvDesc.make(*shp)
    ws = lpdt.Workspace("cuda")
    g = wl.rng(77)
    vd, gd, bd = (dev((1.0 + 0.1 * g.standard_normal(256)).astype(np.float32)) for _ in range(3))
    sx, sw = dev(np.array([0.5], np.float32)), dev(np.array([0.25], np.float32))
    outs = []
    for seed, amp in ((1, "extreme"), (2, "gauss")):      # large values first: stale maxima would show in the second call
        xd, wd = dev(wl.int8_codes(seed, (16, 28, 28, 128), amp)), dev(wl.int8_codes(seed + 10, (256, 3, 3, 128), amp))
        got = lpdt.qconv_ren_fwd_q(ld, xd, wd, sx, sw, groups, vd, gd, bd, 1e-5, ws=ws)
        ref_y = lpdt.qconv_fwd_f32(ld, xd, wd, sx, sw)
        ref = lpdt.range_evonorm_fwd_q(ref_y, groups, vd, gd, bd, 1e-5)
        assert torch.equal(got[0], ref_y)
        for a, b in zip(got[1:], ref):
            assert torch.equal(a, b)
        outs.append(got)
