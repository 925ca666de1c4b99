"""Pins of the oracle's 16-bit weight-gradient product (Section 3, gradient bifurcation: the weight gradient is
computed from a 16-bit floating-point copy of the layer gradient)."""
import numpy as np
import torch

import workloads as wl


def test_bf16_rounding_known_values_and_library(orc):
    f = lambda bits: np.array([bits], np.uint32).view(np.float32)[0]
    cases = {1.0: 0x3F80, -2.5: 0xC020, 0.0: 0x0000, float(f(0x3F808000)): 0x3F80,   # tie, even stays
             float(f(0x3F818000)): 0x3F82,                                            # tie, odd goes up to even
             float(f(0x3F808001)): 0x3F81, float(f(0x3F80FFFF)): 0x3F81, float(f(0x3F7FFFFF)): 0x3F80,
             3.0e38: 0x7F62}
    for x, bits in cases.items():
        assert orc.to_bf16(np.array([x], np.float32))[0] == bits, (x, hex(bits))
    x = (wl.rng(3).standard_normal(100_000) * np.exp(wl.rng(4).uniform(-20, 20, 100_000))).astype(np.float32)
    lib_bits = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.to_bf16(x), lib_bits)


def test_bf16_weight_gradient_against_library_autograd(orc):
    for shp in [(2, 16, 9, 8, 16, 3, 3, 1, 1), (3, 8, 11, 11, 12, 3, 3, 2, 1), (4, 32, 1, 1, 10, 1, 1, 1, 0), (1, 3, 19, 19, 8, 7, 7, 2, 3)]:
        N, C, H, W, K, R, S, st, pd = shp
        P, Q = wl.conv_out(H, pd, R, st), wl.conv_out(W, pd, S, st)
        g = wl.upstream_grad(11, (N, P, Q, K))
        xq = wl.int8_codes(12, (N, H, W, C))
        sx = np.float32(0.0123)
        g16 = orc.to_bf16(g)
        dw, da = orc.qconv_bwd_weight_bf16(orc.conv_desc(*shp), g16, xq, sx)
        gb = torch.from_numpy(g).to(torch.bfloat16).to(torch.float64)                      # the library's bf16 copy
        xt = torch.from_numpy(xq.astype(np.float64)).permute(0, 3, 1, 2)
        wt = torch.zeros((K, C, R, S), dtype=torch.float64, requires_grad=True)
        y = torch.nn.functional.conv2d(xt, wt, stride=st, padding=pd)
        y.backward(gb.permute(0, 3, 1, 2))
        ref = float(sx) * wt.grad.permute(0, 2, 3, 1).numpy()
        assert np.allclose(dw, ref, rtol=1e-12, atol=1e-12 * float(da.max()))
        assert (da >= np.abs(dw) - 1e-12).all()
        # exact 16-bit values: with a gradient already representable in bf16 the product equals the int8 path's sum
        gi = wl.int8_codes(13, (N, P, Q, K))
        dwi, _ = orc.qconv_bwd_weight_bf16(orc.conv_desc(*shp), orc.to_bf16(gi.astype(np.float32)), xq, np.float32(1.0))
        assert np.array_equal(dwi, orc.qconv_bwd_weight(orc.conv_desc(*shp), gi, xq).astype(np.float64))
