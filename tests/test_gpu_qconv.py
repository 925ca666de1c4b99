"""GPU parity of the three int8 convolutions against the oracle: int32 results bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev, host

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)

# N C H W K R S stride pad -- sizes the oracle finishes in seconds, spanning several tiles with ragged tails
CASES = [
    (8, 16, 32, 32, 16, 3, 3, 1, 1),      # the single-layer benchmark configuration
    (2, 64, 14, 14, 64, 3, 3, 1, 1),
    (3, 32, 9, 11, 48, 3, 3, 1, 1),       # ragged: M = 297, Cout = 48
    (2, 64, 15, 15, 128, 3, 3, 2, 1),     # stride 2
    (2, 128, 8, 8, 256, 3, 3, 1, 1),      # few tiles, 9 reduction steps: not worth a split
    (2, 64, 16, 16, 128, 1, 1, 2, 0),     # 1x1 stride-2 projection shortcut
    (5, 48, 7, 7, 80, 1, 1, 1, 0),
    (70, 64, 1, 1, 10, 1, 1, 1, 0),       # linear layer 64 -> 10
    (33, 512, 1, 1, 512, 1, 1, 1, 0),     # linear layer
    (2, 3, 32, 32, 16, 3, 3, 1, 1),       # first layer, 3 input channels
    (1, 3, 37, 37, 64, 7, 7, 2, 3),       # stem-like 7x7 stride 2
    (2, 16, 12, 12, 32, 7, 7, 2, 3),      # 49 taps with channel-multiple-of-16
    (1, 20, 6, 6, 24, 3, 3, 1, 1),        # channel counts that are not multiples of 16
    (1, 256, 4, 4, 512, 3, 3, 1, 1),
    (257, 768, 1, 1, 768, 1, 1, 1, 0),    # transformer-shaped linear layers (tokens x 768 -> 768 / 3072 -> 768), ragged token count
    (130, 3072, 1, 1, 768, 1, 1, 1, 0),
    (2, 144, 7, 7, 80, 3, 3, 1, 1),       # 81 granules of reduction: the forward's 8-granule steps end in a ragged one
    (1, 80, 5, 5, 144, 3, 3, 1, 1),       # the same for backward-data (reduction over 144 output channels x 9 taps)
    (2, 512, 4, 4, 256, 3, 3, 1, 1),      # few tiles, 36 steps: split reduction (zero fill, atomic adds, scale pass)
    (3, 384, 5, 5, 64, 3, 3, 1, 1),       # the same on 64 x 64 tiles
]


def _data(shp, seed, kind):
    N, C, H, W, K, R, S, st, pd = shp
    P, Q = wl.conv_out(H, pd, R, st), wl.conv_out(W, pd, S, st)
    return (wl.int8_codes(seed, (N, H, W, C), kind), wl.int8_codes(seed + 1, (K, R, S, C), kind),
            wl.int8_codes(seed + 2, (N, P, Q, K), kind))


@pytest.mark.parametrize("shp", CASES)
@pytest.mark.parametrize("kind", ["gauss", "uniform"])
def test_three_convs_bit_exact(orc, shp, kind):
    x, w, g = _data(shp, 300, kind)
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    print("case", shp, kind, flush=True)
    acc = lpdt.qconv_fwd(ld, dev(x), dev(w))
    assert np.array_equal(host(acc), orc.qconv_fwd(od, x, w)), "forward"
    dx = lpdt.qconv_bwd_data(ld, dev(g), dev(w))
    assert np.array_equal(host(dx), orc.qconv_bwd_data(od, g, w)), "backward-data"
    dw = lpdt.qconv_bwd_weight(ld, dev(g), dev(x))
    assert np.array_equal(host(dw), orc.qconv_bwd_weight(od, g, x)), "backward-weight"


# stride-1 layers with 64 reduction channels and at most 64 result channels, enough row tiles to fill the chip: the
# filter-resident row-tile kernel (lpdt_qconv_kernel_id 50) -- paddings 0/1/2, ragged last tiles, maps from 14 to 120 wide,
# 2x2 / 3x1 / 3x3 filters, fewer than 64 result channels
ROW_TILE_CASES = [(10, 64, 56, 56, 64, 3, 3, 1, 1), (40, 64, 30, 30, 64, 3, 3, 1, 0), (14, 64, 57, 41, 48, 3, 3, 1, 1),
                  (40, 64, 28, 28, 64, 3, 3, 1, 1), (130, 64, 14, 14, 64, 3, 3, 1, 1), (9, 64, 64, 64, 32, 3, 1, 1, 0),
                  (3, 64, 100, 120, 64, 2, 2, 1, 0), (11, 64, 50, 50, 64, 3, 3, 1, 2)]


@pytest.mark.parametrize("shp", ROW_TILE_CASES)
def test_row_tile_kernel_bit_exact(orc, shp):
    x, w, g = _data(shp, 700, "uniform")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    assert lpdt.qconv_kernel_id(ld, 0) == 50, "the planner changed: pick shapes that reach the row-tile kernel"
    print("row tiles", shp, flush=True)
    assert np.array_equal(host(lpdt.qconv_fwd(ld, dev(x), dev(w))), orc.qconv_fwd(od, x, w)), "forward"
    if shp[4] == 64:
        assert lpdt.qconv_kernel_id(ld, 1) == 50
        ref = orc.qconv_bwd_data(od, g, w)
        assert np.array_equal(host(lpdt.qconv_bwd_data(ld, dev(g), dev(w))), ref), "backward-data"
        # fused scale and accumulation into an existing gradient
        sa, sb = dev(np.array([0.017], np.float32)), dev(np.array([0.0021], np.float32))
        base = dev(wl.images(701, *ref.shape))
        want = lpdt.dequantize(dev(ref.astype(np.int32)), sa, sb, y=base.clone(), accumulate=True)
        got = lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), sa, sb, dx=base.clone(), accumulate=True)
        assert torch.equal(got, want), "backward-data, fused scale, accumulated"


# backward-weight through wgrad_rows_kernel (kernel id 60): ragged last row tile of an image (57 rows in tiles of 2),
# a single row per tile (80 columns), tiles that span the whole image (7x7, 8x8: 2 and 2 reduction groups), no padding,
# padding 2, 2x2 / 3x1 / 1x3 / 2x3 filters, one and several channel tiles, a pixel share that ends inside an image
WGRAD_ROWS_CASES = [(5, 64, 57, 41, 32, 3, 3, 1, 1), (3, 64, 6, 80, 64, 3, 3, 1, 1), (37, 128, 7, 7, 96, 3, 3, 1, 1),
                    (9, 64, 8, 8, 32, 3, 3, 1, 1), (6, 64, 30, 30, 64, 3, 3, 1, 0), (4, 64, 20, 22, 32, 3, 3, 1, 2),
                    (3, 64, 33, 17, 32, 2, 2, 1, 0), (5, 128, 14, 14, 64, 3, 1, 1, 0), (5, 64, 14, 16, 160, 1, 3, 1, 0),
                    (2, 192, 12, 28, 64, 2, 3, 1, 1), (67, 64, 28, 28, 32, 3, 3, 1, 1),
                    (3, 512, 7, 7, 512, 3, 3, 1, 1)]   # the last: 128 output tiles, one pixel share -> results stored by the product kernel itself


@pytest.mark.parametrize("shp", WGRAD_ROWS_CASES)
def test_wgrad_rows_kernel_bit_exact(orc, shp):
    x, w, g = _data(shp, 800, "uniform")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    assert lpdt.qconv_kernel_id(ld, 2) == 60, "the planner changed: pick shapes that reach the row-tile weight-gradient kernel"
    print("wgrad rows", shp, flush=True)
    ref = orc.qconv_bwd_weight(od, g, x)
    assert np.array_equal(host(lpdt.qconv_bwd_weight(ld, dev(g), dev(x))), ref), "backward-weight"
    sa, sb = dev(np.array([0.013], np.float32)), dev(np.array([0.0037], np.float32))
    want = lpdt.dequantize(dev(ref.astype(np.int32)), sa, sb)
    assert torch.equal(lpdt.qconv_bwd_weight_f32(ld, dev(g), dev(x), sa, sb), want), "backward-weight, fused scale"


# backward-weight of first-layer shapes (few input channels; kernel id 1): 1, 3, 4, 5 and 6 input channels, windows of exactly
# 32 bytes, strides 1 and 2, 4- and 8-row filters, fewer than 64 output channels, pixel counts that leave ragged last steps
# and idle waves
NARROW_WGRAD_CASES = [((3, 3, 37, 41, 64, 7, 7, 2, 3), 1), ((5, 3, 32, 32, 16, 3, 3, 1, 1), 1), ((2, 1, 28, 28, 32, 5, 5, 1, 2), 1),
                      ((2, 5, 20, 20, 48, 3, 3, 2, 1), 1), ((70, 3, 24, 24, 64, 7, 7, 2, 3), 1), ((2, 4, 18, 18, 64, 8, 8, 1, 0), 1),
                      ((16, 3, 224, 224, 64, 7, 7, 2, 3), 1), ((2, 6, 12, 12, 32, 5, 5, 1, 2), 1), ((2, 3, 20, 24, 32, 3, 9, 1, 1), 1)]


@pytest.mark.parametrize("shp,kid", NARROW_WGRAD_CASES)
def test_first_layer_weight_gradient_bit_exact(orc, shp, kid):
    x, w, g = _data(shp, 1300, "uniform")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    assert lpdt.qconv_kernel_id(ld, 2) == kid, "the planner changed: pick shapes that reach the first-layer weight-gradient kernel"
    print("first-layer wgrad", shp, flush=True)
    ref = orc.qconv_bwd_weight(od, g, x)
    assert np.array_equal(host(lpdt.qconv_bwd_weight(ld, dev(g), dev(x))), ref), "backward-weight"
    sa, sb = dev(np.array([0.013], np.float32)), dev(np.array([0.0037], np.float32))
    want = lpdt.dequantize(dev(ref.astype(np.int32)), sa, sb)
    assert torch.equal(lpdt.qconv_bwd_weight_f32(ld, dev(g), dev(x), sa, sb), want), "backward-weight, fused scale"


@pytest.mark.parametrize("shp", [(67, 64, 28, 28, 32, 3, 3, 1, 1), (37, 128, 7, 7, 96, 3, 3, 1, 1), (40, 64, 28, 28, 128, 3, 3, 2, 1),
                                 (40, 64, 28, 28, 128, 1, 1, 2, 0)])
def test_weight_gradient_sized_for_running_beside_other_kernels(orc, shp):
    """lpdt_qconv_set_wgrad_beside: fewer blocks (other pixel shares, other partial tiles), the same sums bit for bit -- row-tile
    and rectangle kernels; the workspace query covers both settings."""
    x, w, g = _data(shp, 1400, "uniform")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    ref = orc.qconv_bwd_weight(od, g, x)
    try:
        for beside in (True, False, True):
            lpdt.qconv_set_wgrad_beside(beside)
            assert np.array_equal(host(lpdt.qconv_bwd_weight(ld, dev(g), dev(x))), ref), f"beside={beside}"
    finally:
        lpdt.qconv_set_wgrad_beside(False)


# backward-weight of pointwise products through wgrad_gemm_kernel (kernel id 62): token counts that are no multiple of the
# 64-token step or of a block's share, 3 x 3 / 3 x 12 / 12 x 3 / 4 x 4 tiles, a spatial 1x1 layer
WGRAD_GEMM_CASES = [(8200, 768, 1, 1, 768, 1, 1, 1, 0), (3001, 768, 1, 1, 3072, 1, 1, 1, 0), (2987, 3072, 1, 1, 768, 1, 1, 1, 0),
                    (9, 1024, 24, 25, 1024, 1, 1, 1, 0)]


# the same kernel with one filter tap per block (kernel id 63): VGG's 4 x 4 and 2 x 2 maps at 512 channels, a ragged last
# 64-pixel step on a 5 x 3 map, a 2 x 3 filter without padding, 512 -> 256 and 256 -> 512 channels
WGRAD_GEMM_TAPS_CASES = [(64, 512, 4, 4, 512, 3, 3, 1, 1), (256, 512, 2, 2, 512, 3, 3, 1, 1), (100, 256, 5, 3, 512, 3, 3, 1, 1),
                         (120, 512, 4, 4, 512, 2, 3, 1, 0), (77, 512, 4, 4, 256, 3, 3, 1, 1)]


@pytest.mark.parametrize("shp", WGRAD_GEMM_TAPS_CASES)
def test_wgrad_gemm_kernel_with_taps_bit_exact(orc, shp):
    x, w, g = _data(shp, 950, "uniform")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    assert lpdt.qconv_kernel_id(ld, 2) == 63, "the planner changed: pick shapes that reach the one-tap-per-block GEMM weight gradient"
    print("wgrad gemm taps", shp, flush=True)
    ref = orc.qconv_bwd_weight(od, g, x)
    assert np.array_equal(host(lpdt.qconv_bwd_weight(ld, dev(g), dev(x))), ref), "backward-weight"
    sa, sb = dev(np.array([0.013], np.float32)), dev(np.array([0.0037], np.float32))
    want = lpdt.dequantize(dev(ref.astype(np.int32)), sa, sb)
    assert torch.equal(lpdt.qconv_bwd_weight_f32(ld, dev(g), dev(x), sa, sb), want), "backward-weight, fused scale"


@pytest.mark.parametrize("shp", WGRAD_GEMM_CASES)
def test_wgrad_gemm_kernel_bit_exact(orc, shp):
    x, w, g = _data(shp, 900, "uniform")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    assert lpdt.qconv_kernel_id(ld, 2) == 62, "the planner changed: pick shapes that reach the GEMM-shaped weight-gradient kernel"
    print("wgrad gemm", shp, flush=True)
    ref = orc.qconv_bwd_weight(od, g, x)
    assert np.array_equal(host(lpdt.qconv_bwd_weight(ld, dev(g), dev(x))), ref), "backward-weight"
    sa, sb = dev(np.array([0.013], np.float32)), dev(np.array([0.0037], np.float32))
    want = lpdt.dequantize(dev(ref.astype(np.int32)), sa, sb)
    assert torch.equal(lpdt.qconv_bwd_weight_f32(ld, dev(g), dev(x), sa, sb), want), "backward-weight, fused scale"


def test_extreme_codes_no_overflow_in_range(orc):
    # all +-127 with reduction length 4608 (fwd) / 1152 (wgrad): the largest magnitudes the path can see here
    shp = (2, 512, 6, 6, 64, 3, 3, 1, 1)
    x, w, g = _data(shp, 400, "extreme")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    assert np.array_equal(host(lpdt.qconv_fwd(ld, dev(x), dev(w))), orc.qconv_fwd(od, x, w))
    assert np.array_equal(host(lpdt.qconv_bwd_data(ld, dev(g), dev(w))), orc.qconv_bwd_data(od, g, w))
    assert np.array_equal(host(lpdt.qconv_bwd_weight(ld, dev(g), dev(x))), orc.qconv_bwd_weight(od, g, x))


def test_output_buffers_are_overwritten_and_deterministic():
    shp = (2, 128, 8, 8, 256, 3, 3, 1, 1)
    x, w, g = _data(shp, 500, "gauss")
    ld = lpdt.ConvDesc.make(*shp)
    junk = torch.full((2, 8, 8, 256), 12345, dtype=torch.int32, device="cuda")
    a = lpdt.qconv_fwd(ld, dev(x), dev(w), acc=junk)
    b = lpdt.qconv_fwd(ld, dev(x), dev(w))
    assert torch.equal(a, b)
    junk = torch.full((256, 3, 3, 128), -7, dtype=torch.int32, device="cuda")
    a = lpdt.qconv_bwd_weight(ld, dev(g), dev(x), dw=junk)
    b = lpdt.qconv_bwd_weight(ld, dev(g), dev(x))
    assert torch.equal(a, b)


# CASES[5]: three of the four residue classes of a 1x1 stride-2 filter have no taps (accumulating calls leave their pixels
# alone); CASES[6], CASES[7]: small linear layers (the one-launch kernel with every output mode)
@pytest.mark.parametrize("shp", [CASES[0], CASES[2], CASES[3], CASES[4], CASES[5], CASES[6], CASES[7], CASES[9], CASES[10], CASES[12]])
def test_fused_fp32_epilogue_equals_int32_then_dequantize(orc, shp):
    """The *_f32 entry points must give exactly the bits of the int32 call followed by lpdt_dequantize,
    and stay within 1e-5 of the oracle's real-valued result."""
    x, w, g = _data(shp, 600, "gauss")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    sa, sb = np.float32(0.0123), np.float32(3.3e-3)
    dsa, dsb = dev(np.array([sa])), dev(np.array([sb]))
    y = lpdt.qconv_fwd_f32(ld, dev(x), dev(w), dsa, dsb)
    assert torch.equal(y, lpdt.dequantize(lpdt.qconv_fwd(ld, dev(x), dev(w)), dsa, dsb))
    ref = orc.dequantize(orc.qconv_fwd(od, x, w), sa, sb)
    assert np.abs(host(y) - ref).max() <= 1e-5 * np.abs(ref).max()
    # the skip connection's addition in the epilogue: the bits of the product into a temporary + lpdt_add
    addend = dev(wl.images(602, *host(y).shape))
    want = lpdt.add(addend, y)
    got = lpdt.qconv_fwd_f32_add(ld, dev(x), dev(w), dsa, dsb, addend.clone())
    assert torch.equal(got, want)
    dx = lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), dsa, dsb)
    assert torch.equal(dx, lpdt.dequantize(lpdt.qconv_bwd_data(ld, dev(g), dev(w)), dsa, dsb))
    base = wl.images(601, *host(dx).shape)
    acc = dev(base)
    lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), dsa, dsb, dx=acc, accumulate=True)
    ref = orc.dequantize(orc.qconv_bwd_data(od, g, w), sa, sb) + base
    assert np.abs(host(acc) - ref).max() <= 1e-5 * max(np.abs(ref).max(), 1.0)
    dw = lpdt.qconv_bwd_weight_f32(ld, dev(g), dev(x), dsa, dsb)
    assert torch.equal(dw, lpdt.dequantize(lpdt.qconv_bwd_weight(ld, dev(g), dev(x)), dsa, dsb))


def _random_shapes(seed, count):
    """Seeded shapes across the kernels' decision boundaries: channel counts around multiples of 16, maps around the
    tile and rectangle sizes, filters 1/3/5, strides 1/2, paddings 0..2, batch sizes that leave ragged tiles."""
    g = wl.rng(seed)
    out = []
    while len(out) < count:
        R = int(g.choice([1, 3, 3, 5]))
        st, pd = int(g.choice([1, 1, 2])), int(g.integers(0, R // 2 + 2))
        C = int(g.choice([16, 32, 48, 64, 80, 96, 128, 12, 40]))
        K = int(g.choice([16, 32, 48, 64, 96, 128, 144, 24, 100]))
        H, W = int(g.integers(R, 23)), int(g.integers(R, 23))
        N = int(g.integers(1, 6))
        if H + 2 * pd < R or W + 2 * pd < R or pd >= R:
            continue
        out.append((N, C, H, W, K, R, R, st, pd))
    return out


@pytest.mark.parametrize("shp", _random_shapes(4242, 28))
def test_random_shapes_bit_exact_and_fused_epilogues(orc, shp):
    print("case", shp, flush=True)
    x, w, g = _data(shp, 900, "gauss")
    od, ld = orc.conv_desc(*shp), lpdt.ConvDesc.make(*shp)
    ref_f, ref_d, ref_w = orc.qconv_fwd(od, x, w), orc.qconv_bwd_data(od, g, w), orc.qconv_bwd_weight(od, g, x)
    acc, dx, dw = lpdt.qconv_fwd(ld, dev(x), dev(w)), lpdt.qconv_bwd_data(ld, dev(g), dev(w)), lpdt.qconv_bwd_weight(ld, dev(g), dev(x))
    assert np.array_equal(host(acc), ref_f), "forward"
    assert np.array_equal(host(dx), ref_d), "backward-data"
    assert np.array_equal(host(dw), ref_w), "backward-weight"
    sa, sb = dev(np.array([0.0123], np.float32)), dev(np.array([3.3e-3], np.float32))
    assert torch.equal(lpdt.qconv_fwd_f32(ld, dev(x), dev(w), sa, sb), lpdt.dequantize(acc, sa, sb))
    assert torch.equal(lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), sa, sb), lpdt.dequantize(dx, sa, sb))
    assert torch.equal(lpdt.qconv_bwd_weight_f32(ld, dev(g), dev(x), sa, sb), lpdt.dequantize(dw, sa, sb))


@pytest.mark.parametrize("shp", [CASES[1], CASES[3], CASES[4], CASES[5], CASES[13], CASES[15]])
def test_backward_data_with_prepacked_filter_equals_the_plain_call(shp):
    """lpdt_qconv_bwd_data_pack_filter + lpdt_qconv_bwd_data_f32_packed: the bits of lpdt_qconv_bwd_data_f32, overwrite and
    accumulate; the packed copy stays valid over several calls."""
    x, w, g = _data(shp, 900, "gauss")
    ld = lpdt.ConvDesc.make(*shp)
    sg = torch.tensor([0.031], dtype=torch.float32, device="cuda")
    sw = torch.tensor([0.0042], dtype=torch.float32, device="cuda")
    packed = lpdt.qconv_bwd_data_pack_filter(ld, dev(w))
    assert packed is not None
    ref = lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), sg, sw)
    got = lpdt.qconv_bwd_data_f32_packed(ld, dev(g), packed, sg, sw)
    assert torch.equal(got, ref)
    base = dev(wl.upstream_grad(901, tuple(ref.shape)))
    ref2 = lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), sg, sw, dx=base.clone(), accumulate=True)
    got2 = lpdt.qconv_bwd_data_f32_packed(ld, dev(g), packed, sg, sw, dx=base.clone(), accumulate=True)
    assert torch.equal(got2, ref2)


def test_filters_prepacked_in_one_launch_equal_the_single_calls():
    """lpdt_qconv_bwd_data_pack_filters: the bytes of lpdt_qconv_bwd_data_pack_filter for every filter, with more filters
    than one launch's table holds (24), stride 1 and 2, 1x1 and 3x3; a shape without a prepared form is refused."""
    shapes = [CASES[1], CASES[3], CASES[4], CASES[5], CASES[13], CASES[15]] * 5
    descs = [lpdt.ConvDesc.make(*shp) for shp in shapes]
    ws = [dev(_data(shp, 1200 + i, "gauss")[1]) for i, shp in enumerate(shapes)]
    got = lpdt.qconv_bwd_data_pack_filters(descs, ws)
    for d, w, t in zip(descs, ws, got):
        ref = lpdt.qconv_bwd_data_pack_filter(d, w)
        assert torch.equal(t[:ref.numel()], ref)
    bad = lpdt.ConvDesc.make(1, 20, 6, 6, 24, 3, 3, 1, 1)
    with pytest.raises(lpdt.LpdtError):
        lpdt.qconv_bwd_data_pack_filters([descs[0], bad], [ws[0], torch.zeros((24, 3, 3, 20), dtype=torch.int8, device="cuda")])


def test_prepacked_filter_is_refused_where_backward_data_has_no_packed_form():
    ld = lpdt.ConvDesc.make(1, 20, 6, 6, 24, 3, 3, 1, 1)     # channel counts that are not multiples of 16
    w = torch.zeros((24, 3, 3, 20), dtype=torch.int8, device="cuda")
    assert lpdt.qconv_bwd_data_pack_filter(ld, w) is None


# the last three: launches on the 256x256, 256x128 and 128x128 tiles of the direct-to-LDS kernel (kernel ids 20, 24, 22)
@pytest.mark.parametrize("shp", [CASES[1], CASES[2], CASES[3], CASES[4], CASES[9], CASES[12], CASES[14], CASES[15],
                                 (16384, 768, 1, 1, 3072, 1, 1, 1, 0), (8, 64, 56, 56, 512, 3, 3, 1, 1), (8200, 768, 1, 1, 768, 1, 1, 1, 0)])
def test_products_with_absmax_output(shp):
    """lpdt_qconv_fwd_f32_absmax / lpdt_qconv_bwd_data_f32_absmax: the results of the plain calls, bit for bit, and the exact
    largest magnitude of what was stored (epilogue path, split reductions, first layer, odd channel counts)."""
    x, w, g = _data(shp, 950, "gauss")
    ld = lpdt.ConvDesc.make(*shp)
    s1 = torch.tensor([0.027], dtype=torch.float32, device="cuda")
    s2 = torch.tensor([0.0031], dtype=torch.float32, device="cuda")
    ref = lpdt.qconv_fwd_f32(ld, dev(x), dev(w), s1, s2)
    y, am = lpdt.qconv_fwd_f32_absmax(ld, dev(x), dev(w), s1, s2)
    assert torch.equal(y, ref) and float(am[0]) == float(ref.abs().max())
    ref = lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), s1, s2)
    dx, am = lpdt.qconv_bwd_data_f32_absmax(ld, dev(g), dev(w), s1, s2)
    assert torch.equal(dx, ref) and float(am[0]) == float(ref.abs().max())
    base = dev(wl.upstream_grad(951, tuple(ref.shape)))
    ref2 = lpdt.qconv_bwd_data_f32(ld, dev(g), dev(w), s1, s2, dx=base.clone(), accumulate=True)
    packed = lpdt.qconv_bwd_data_pack_filter(ld, dev(w))
    dx2, am2 = lpdt.qconv_bwd_data_f32_absmax(ld, dev(g), None if packed is not None else dev(w), s1, s2, packed=packed, dx=base.clone(),
                                              accumulate=True)
    assert torch.equal(dx2, ref2) and float(am2[0]) == float(ref2.abs().max())
