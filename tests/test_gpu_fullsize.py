"""Parity at the benchmark's full sizes (config 5: ResNet-18 shapes at batch 64 and 224x224, 16 agents x 11.2 M
parameters), in the launch configurations bench.py times.  Inputs are seeded and synthetic.  The three convolution
products of every layer are compared with the C oracle element by element over the WHOLE result
(test_conv_products_at_full_size_whole_tensors, which also pins the kernel and tile each product takes), and, as a
quick check that also covers the fused-scale and packed-filter entry points, on sampled coordinates that the oracle
computes one by one (oracle/sampled.py); the O(n) parts (quantizer, Range-EvoNorm) against the full C oracle; the CHOCO
mix against the top-k rule written out in numpy."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from workloads import nets
from gpu_util import assert_close, dev, host
from oracle import sampled

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)

B = 64
LAYERS = {   # N C H W K R S stride pad
    # config 5: every distinct layer shape of ResNet-18 at batch 64, 224x224
    "stem 7x7 s2": (B, 3, 224, 224, 64, 7, 7, 2, 3),
    "layer1 3x3": (B, 64, 56, 56, 64, 3, 3, 1, 1),
    "layer2 3x3 s2": (B, 64, 56, 56, 128, 3, 3, 2, 1),
    "layer2 1x1 s2": (B, 64, 56, 56, 128, 1, 1, 2, 0),
    "layer2 3x3": (B, 128, 28, 28, 128, 3, 3, 1, 1),
    "layer3 3x3 s2": (B, 128, 28, 28, 256, 3, 3, 2, 1),
    "layer3 1x1 s2": (B, 128, 28, 28, 256, 1, 1, 2, 0),
    "layer3 3x3": (B, 256, 14, 14, 256, 3, 3, 1, 1),
    "layer4 3x3 s2": (B, 256, 14, 14, 512, 3, 3, 2, 1),
    "layer4 1x1 s2": (B, 256, 14, 14, 512, 1, 1, 2, 0),
    "layer4 3x3": (B, 512, 7, 7, 512, 3, 3, 1, 1),
    "classifier": (B, 512, 1, 1, 100, 1, 1, 1, 0),
    # configs 2 and 4: first and widest layers of ResNet-20 at batch 128 and VGG-11 at batch 256
    "resnet20 first": (128, 3, 32, 32, 16, 3, 3, 1, 1),
    "resnet20 16": (128, 16, 32, 32, 16, 3, 3, 1, 1),
    "resnet20 64": (128, 64, 8, 8, 64, 3, 3, 1, 1),
    "vgg11 first": (256, 3, 32, 32, 64, 3, 3, 1, 1),
    "vgg11 128": (256, 64, 16, 16, 128, 3, 3, 1, 1),
    "vgg11 512": (256, 512, 2, 2, 512, 3, 3, 1, 1),
}


# lpdt_qconv_kernel_id of (forward, backward-data, backward-weight) at these sizes: the kernels and tiles bench.py times.
# 1: first-layer kernels (narrow_fwd_kernel / narrow_wgrad_kernel); 10..14 (+100: split reduction): igemm_kernel
# <128,32,4>, <64,64,4>, <64,64,8>, <128,64,4>, <128,64,8>; 20..24: igemm_dma_kernel 256x256, 128x128 (8 waves), 128x128
# (4 waves), 64x128, 256x128 (3 stages); 50: patch_conv_kernel (filter resident in LDS, row tiles); 30 + t + 4*[64-pixel steps] + 8*[two wave groups]: wgrad_rect_kernel with tile t (0: 32x64, 1: 64x64);
# 60: wgrad_rows_kernel (row tiles of a stride-1 layer, operands straight into LDS); 62: wgrad_gemm_kernel (pointwise, 256x256 tiles);
# 2: wgrad_kernel; 3: linear_small_kernel; 0: the any-shape kernels.
KERNELS = {
    "stem 7x7 s2": (1, 10, 1), "layer1 3x3": (50, 50, 60), "layer2 3x3 s2": (22, 13, 38), "layer2 1x1 s2": (22, 13, 31),
    "layer2 3x3": (22, 22, 60), "layer3 3x3 s2": (21, 22, 38), "layer3 1x1 s2": (21, 22, 31), "layer3 3x3": (21, 21, 60),
    "layer4 3x3 s2": (23, 21, 38), "layer4 1x1 s2": (23, 21, 31), "layer4 3x3": (23, 23, 60), "classifier": (3, 3, 3),
    "resnet20 first": (1, 10, 1), "resnet20 16": (10, 10, 42), "resnet20 64": (11, 11, 60), "vgg11 first": (1, 10, 1),
    "vgg11 128": (22, 14, 60), "vgg11 512": (112, 112, 63),
    "gemm 256x128 tile": (24, 12, 60), "gemm 256x256 tile": (20, 24, 62),
}
# the two direct-to-LDS tiles no benchmark layer takes at batch 64, and the GEMM-shaped weight gradient
LAYERS["gemm 256x128 tile"] = (8, 64, 56, 56, 512, 3, 3, 1, 1)
LAYERS["gemm 256x256 tile"] = (10240, 2304, 1, 1, 1024, 1, 1, 1, 0)


@pytest.mark.parametrize("name", list(LAYERS))
def test_conv_products_at_full_size_whole_tensors(orc, name):
    shp = LAYERS[name]
    N, C, H, W, K, R, S, st, pd = shp
    P, Q = wl.conv_out(H, pd, R, st), wl.conv_out(W, pd, S, st)
    seed = 9000 + sum(shp)
    x, w, g = wl.int8_codes(seed, (N, H, W, C)), wl.int8_codes(seed + 1, (K, R, S, C)), wl.int8_codes(seed + 2, (N, P, Q, K))
    xd, wd, gd = dev(x), dev(w), dev(g)
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    assert tuple(lpdt.qconv_kernel_id(ld, i) for i in range(3)) == KERNELS[name], "the planner changed: update KERNELS"
    print(name, "forward", flush=True)
    got = host(lpdt.qconv_fwd(ld, xd, wd))
    assert np.array_equal(got, orc.qconv_fwd(od, x, w)), name + " forward"
    if name != "stem 7x7 s2":   # nothing upstream of the image; its backward-data is covered at small sizes
        print(name, "backward-data", flush=True)
        got = host(lpdt.qconv_bwd_data(ld, gd, wd))
        assert np.array_equal(got, orc.qconv_bwd_data(od, g, w)), name + " backward-data"
    print(name, "backward-weight", flush=True)
    got = host(lpdt.qconv_bwd_weight(ld, gd, xd))
    assert np.array_equal(got, orc.qconv_bwd_weight(od, g, x)), name + " backward-weight"


def _coords(rng, dims, count):
    pts = {tuple(0 for _ in dims), tuple(d - 1 for d in dims)}
    for axis in range(len(dims)):          # one point on every face
        for edge in (0, dims[axis] - 1):
            p = [int(rng.integers(d)) for d in dims]
            p[axis] = edge
            pts.add(tuple(p))
    while len(pts) < count:
        pts.add(tuple(int(rng.integers(d)) for d in dims))
    return sorted(pts)


@pytest.mark.parametrize("name", list(LAYERS))
def test_conv_products_at_full_size_on_sampled_outputs(name):
    # the fused-scale (fp32) and packed-filter entry points on top of the int32 ones, on sampled coordinates
    shp = LAYERS[name]
    N, C, H, W, K, R, S, st, pd = shp
    P, Q = wl.conv_out(H, pd, R, st), wl.conv_out(W, pd, S, st)
    seed = 7000 + sum(shp)
    x, w, g = wl.int8_codes(seed, (N, H, W, C)), wl.int8_codes(seed + 1, (K, R, S, C)), wl.int8_codes(seed + 2, (N, P, Q, K))
    xd, wd, gd = dev(x), dev(w), dev(g)
    ld = lpdt.ConvDesc.make(*shp)
    rng = wl.rng(seed + 3)
    sa = torch.tensor([0.0131], device="cuda")
    sb = torch.tensor([0.00217], device="cuda")
    scale = float(np.float32(0.0131) * np.float32(0.00217))

    co = _coords(rng, (N, P, Q, K), 160)
    ref = sampled.qconv_fwd_at(x, w, st, pd, co)
    acc = host(lpdt.qconv_fwd(ld, xd, wd))
    assert np.array_equal(np.array([acc[c] for c in co], np.int64), ref), name + " forward"
    y = host(lpdt.qconv_fwd_f32(ld, xd, wd, sa, sb))
    assert_close(np.array([y[c] for c in co]), scale * ref.astype(np.float64), 1e-5, 0.0, name + " forward, fused scale")
    del acc, y

    ci = _coords(rng, (N, H, W, C), 160)
    ref = sampled.qconv_bwd_data_at(g, w, H, W, st, pd, ci)
    dx = host(lpdt.qconv_bwd_data(ld, gd, wd))
    assert np.array_equal(np.array([dx[c] for c in ci], np.int64), ref), name + " backward-data"
    dxf = host(lpdt.qconv_bwd_data_f32(ld, gd, wd, sa, sb))
    assert_close(np.array([dxf[c] for c in ci]), scale * ref.astype(np.float64), 1e-5, 0.0, name + " backward-data, fused scale")
    packed = lpdt.qconv_bwd_data_pack_filter(ld, wd)       # the filter transposed ahead of time: the same bits
    if packed is not None:
        assert np.array_equal(host(lpdt.qconv_bwd_data_f32_packed(ld, gd, packed, sa, sb)), dxf), name + " backward-data, packed filter"
    del dx, dxf

    cw = _coords(rng, (K, R, S, C), 60)
    ref = sampled.qconv_bwd_weight_at(g, x, R, S, st, pd, cw)
    dw = host(lpdt.qconv_bwd_weight(ld, gd, xd))
    assert np.array_equal(np.array([dw[c] for c in cw], np.int64), ref), name + " backward-weight"
    dwf = host(lpdt.qconv_bwd_weight_f32(ld, gd, xd, sa, sb))
    assert_close(np.array([dwf[c] for c in cw]), scale * ref.astype(np.float64), 1e-5, 0.0, name + " backward-weight, fused scale")


def test_quantizer_at_the_largest_activation(orc):
    n = B * 112 * 112 * 64                                     # the stem's output: 51.4 M elements
    x = wl.rng(7100).standard_normal(n, dtype=np.float32) * np.float32(0.8)
    xd = dev(x)
    for rounding in (0, 1):
        q_ref, s_ref = orc.quantize(x, rounding, wl.PHILOX_SEED, (3 << 32) + (5 << 24))
        q, s = lpdt.quantize(xd, rounding, wl.PHILOX_SEED, (3 << 32) + (5 << 24))
        assert host(s)[0] == s_ref and np.array_equal(host(q), q_ref)


def test_range_evonorm_at_the_largest_activation(orc):
    N, H, W, C, groups = B, 112, 112, 64, 32
    g = wl.rng(7200)
    x = g.standard_normal((N, H, W, C), dtype=np.float32)
    dy = g.standard_normal((N, H, W, C), dtype=np.float32) * np.float32(0.1)
    v = (1.0 + 0.1 * g.standard_normal(C)).astype(np.float32)
    gamma = (1.0 + 0.1 * g.standard_normal(C)).astype(np.float32)
    beta = (0.1 * g.standard_normal(C)).astype(np.float32)
    z_ref, rng_ref, amx_ref, amn_ref = orc.range_evonorm_fwd(x, groups, v, gamma, beta, 1e-5)
    xd = dev(x)
    z, rng_d, amx, amn = lpdt.range_evonorm_fwd(xd, groups, dev(v), dev(gamma), dev(beta), 1e-5)
    assert np.array_equal(host(amx), amx_ref) and np.array_equal(host(amn), amn_ref)
    assert_close(host(z), z_ref, 1e-4, float(np.abs(z_ref).max()) * 1e-2, "Range-EvoNorm forward")
    del z_ref
    dx_ref, dv_ref, dg_ref, db_ref = orc.range_evonorm_bwd(dy, x, groups, v, gamma, 1e-5)
    dx, dv, dg, db = lpdt.range_evonorm_bwd(dev(dy), xd, groups, dev(v), dev(gamma), rng_d, amx, amn, 1e-5)
    assert_close(host(dx), dx_ref, 1e-4, float(np.abs(dx_ref).max()) * 1e-2, "Range-EvoNorm dx")
    for got, r, nm in ((dv, dv_ref, "dv"), (dg, dg_ref, "dgamma"), (db, db_ref, "dbeta")):
        # sums of 0.8 M terms of either sign per channel in fp32 (fixed order): a few 1e-6 of the sum of magnitudes
        assert_close(host(got), r, 1e-4, float(np.abs(r).max()), nm)
    # the int8-output forward on the same 51 M elements: the codes and scale of forward + quantizer, bit for bit
    import torch
    z2, _, _, _, absmax = lpdt.range_evonorm_fwd(xd, groups, dev(v), dev(gamma), dev(beta), 1e-5, want_absmax=True)
    q_ref, s_ref = lpdt.quantize_with_absmax(z2, absmax, lpdt.ROUND_NEAREST)
    q, s, r2, amx2, amn2 = lpdt.range_evonorm_fwd_q(xd, groups, dev(v), dev(gamma), dev(beta), 1e-5)
    assert torch.equal(s, s_ref) and torch.equal(q, q_ref)
    assert torch.equal(r2, rng_d) and torch.equal(amx2, amx) and torch.equal(amn2, amn)


def test_choco_mix_at_full_size():
    net = nets.resnet18()
    n, d, rho, rate = 16, net.num_params(), 0.01, 0.1
    seg = net.param_offsets()
    x = wl.agent_params(7300, n, d)
    xh = wl.agent_params(7301, n, d, spread=2e-3)
    Wm = wl.ring_matrix(n)
    xd, hd = dev(x), dev(xh)
    lpdt.gossip_mix(xd, hd, Wm, rate=rate, keep_ratio=rho, seg_offsets=seg)
    got_h, got_x = host(hd), host(xd)
    # xhat: the top-k rule per agent and layer, written out
    ref_h = xh.copy()
    for i in range(n):
        v = (x[i] - xh[i]).astype(np.float32)
        for lo, hi in zip(seg[:-1], seg[1:]):
            if hi == lo:
                continue
            m = sampled.topk_mask(v[lo:hi], max(1, math.ceil(rho * (hi - lo))))
            ref_h[i, lo:hi][m] = (xh[i, lo:hi][m] + v[lo:hi][m]).astype(np.float32)
        assert np.array_equal(got_h[i], ref_h[i]), f"xhat of agent {i}"
    # x on sampled columns: x_i + rate * sum_j W_ij (xhat_j - xhat_i) in double
    cols = np.unique(np.concatenate([wl.rng(7302).integers(0, d, size=4000), [0, d - 1], np.array(seg[1:-1]) - 1, np.array(seg[1:-1])]))
    hc = ref_h[:, cols].astype(np.float64)
    mix = Wm.astype(np.float64) @ hc - Wm.astype(np.float64).sum(1, keepdims=True) * hc
    ref_x = x[:, cols].astype(np.float64) + float(np.float32(rate)) * mix
    assert_close(got_x[:, cols], ref_x, 1e-5, float(np.abs(x).max()), "mixed models")
    # untouched where nothing is mixed in: the agent average is preserved (columns of W - I sum to zero)
    assert np.abs(got_x[:, cols].astype(np.float64).mean(0) - x[:, cols].astype(np.float64).mean(0)).max() < 1e-6
