"""GPU parity of the 16-bit weight-gradient product (gradient bifurcation as the paper states it) against the oracle:
bfloat16 conversion bit-exact; fp32-accumulated sums within 2e-6 of the sum of |terms| (the kernel adds a few
thousand fp32 terms per accumulator before the partial tiles are combined; the exact sum comes from the oracle)."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev, host

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)

CASES = [
    (8, 16, 32, 32, 16, 3, 3, 1, 1),
    (2, 64, 14, 14, 64, 3, 3, 1, 1),
    (3, 32, 9, 11, 48, 3, 3, 1, 1),       # ragged
    (2, 64, 15, 15, 128, 3, 3, 2, 1),     # stride 2
    (2, 64, 16, 16, 128, 1, 1, 2, 0),     # 1x1 stride-2 projection
    (5, 48, 7, 7, 80, 1, 1, 1, 0),        # pointwise, flattened
    (70, 64, 1, 1, 24, 1, 1, 1, 0),       # linear layer
    (2, 3, 32, 32, 16, 3, 3, 1, 1),       # 3 input channels: any-shape kernel
    (1, 20, 6, 6, 20, 3, 3, 1, 1),        # channel counts outside the tiled kernel's reach
    (4, 128, 28, 28, 64, 3, 3, 1, 1),     # several pixel splits
]


def test_to_bf16_bit_exact(orc):
    g = wl.rng(5)
    x = (g.standard_normal(300_001) * np.exp(g.uniform(-30, 30, 300_001))).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.00390625, 1.01171875]            # exact ties
    got = host(lpdt.to_bf16(dev(x))).view(np.uint16)
    assert np.array_equal(got, orc.to_bf16(x))


@pytest.mark.parametrize("shp", CASES)
def test_weight_gradient_from_bf16_gradient(orc, shp):
    N, C, H, W, K, R, S, st, pd = shp
    P, Q = wl.conv_out(H, pd, R, st), wl.conv_out(W, pd, S, st)
    g = wl.upstream_grad(600 + sum(shp), (N, P, Q, K))
    xq = wl.int8_codes(601 + sum(shp), (N, H, W, C))
    sx = np.float32(0.0173)
    g16 = orc.to_bf16(g)
    ref, mag = orc.qconv_bwd_weight_bf16(orc.conv_desc(*shp), g16, xq, sx)
    g16d = lpdt.to_bf16(dev(g))
    assert np.array_equal(host(g16d).view(np.uint16), g16)
    dw = host(lpdt.qconv_bwd_weight_bf16(lpdt.ConvDesc.make(*shp), g16d, dev(xq), dev(np.array([sx]))))
    err = np.abs(dw.astype(np.float64) - ref)
    bound = 2e-6 * mag + 1e-30
    assert (err <= bound).all(), f"worst {float((err / bound).max()):.2f} x the bound at {np.unravel_index(np.argmax(err / bound), err.shape)}"
    # twice the same call: the same bits
    dw2 = host(lpdt.qconv_bwd_weight_bf16(lpdt.ConvDesc.make(*shp), g16d, dev(xq), dev(np.array([sx]))))
    assert np.array_equal(dw, dw2)


def test_full_size_layer_on_sampled_outputs(orc):
    """ResNet-18 layer1 at batch 64: sampled filter elements summed one by one in double."""
    shp = (64, 64, 56, 56, 64, 3, 3, 1, 1)
    N, C, H, W, K, R, S, st, pd = shp
    g = wl.upstream_grad(650, (N, H, W, K))
    xq = wl.int8_codes(651, (N, H, W, C))
    sx = np.float32(0.0173)
    g16 = orc.to_bf16(g)
    gv = (g16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    dw = host(lpdt.qconv_bwd_weight_bf16(lpdt.ConvDesc.make(*shp), dev(g16.view(np.int16)), dev(xq), dev(np.array([sx]))))
    rng = wl.rng(652)
    for _ in range(40):
        k, r, s, c = int(rng.integers(K)), int(rng.integers(R)), int(rng.integers(S)), int(rng.integers(C))
        ps, qs = np.arange(H), np.arange(W)
        pv, qv = ps[(ps + r - pd >= 0) & (ps + r - pd < H)], qs[(qs + s - pd >= 0) & (qs + s - pd < W)]
        terms = gv[:, pv][:, :, qv, k] * xq[:, pv + r - pd][:, :, qv + s - pd, c].astype(np.float64)
        assert abs(float(dw[k, r, s, c]) - float(sx) * terms.sum()) <= 2e-6 * float(sx) * np.abs(terms).sum()
