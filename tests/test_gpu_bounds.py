"""No entry point writes outside what it was given: results and workspaces sit between guard bytes, the workspace has
exactly the size its query returned, and the guards are intact after the call.  (Values are checked by the parity tests;
the shapes here are theirs, one or more per kernel.)"""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)

GUARD = 4096
FILL = 0xA5


class Guards:
    """Hands out device tensors and workspaces with GUARD bytes of FILL on both sides; check() looks at all of them."""

    def __init__(self):
        self.bufs = []

    def _make(self, nbytes):
        buf = torch.full((GUARD + nbytes + GUARD,), FILL, dtype=torch.uint8, device="cuda")
        self.bufs.append((buf, nbytes))
        return buf[GUARD:GUARD + nbytes]

    def tensor(self, shape, dtype):
        n = int(np.prod(shape))
        return self._make(n * torch.empty((), dtype=dtype).element_size()).view(dtype).view(*shape)

    def get(self, nbytes):          # the binding's workspace protocol: exactly the size asked for
        nbytes = int(nbytes)
        if nbytes == 0:
            return None, 0
        return self._make(nbytes), nbytes

    def check(self, what):
        torch.cuda.synchronize()
        for i, (buf, nbytes) in enumerate(self.bufs):
            lo, hi = buf[:GUARD], buf[GUARD + nbytes:]
            assert bool((lo == FILL).all()) and bool((hi == FILL).all()), f"{what}: buffer {i} ({nbytes} bytes) was overrun"
        self.bufs.clear()


# N C H W K R S stride pad: every convolution kernel of the library (tile-at-a-time and direct-to-LDS implicit GEMM with and
# without a split reduction, row tiles, first layer, small linear, weight gradients by rows / rectangles / GEMM / taps)
CONV_CASES = [
    (8, 16, 32, 32, 16, 3, 3, 1, 1), (3, 32, 9, 11, 48, 3, 3, 1, 1), (2, 64, 15, 15, 128, 3, 3, 2, 1), (2, 64, 16, 16, 128, 1, 1, 2, 0),
    (70, 64, 1, 1, 10, 1, 1, 1, 0), (33, 512, 1, 1, 512, 1, 1, 1, 0), (1, 3, 37, 37, 64, 7, 7, 2, 3), (1, 20, 6, 6, 24, 3, 3, 1, 1),
    (257, 768, 1, 1, 768, 1, 1, 1, 0), (2, 144, 7, 7, 80, 3, 3, 1, 1), (2, 512, 4, 4, 256, 3, 3, 1, 1), (3, 384, 5, 5, 64, 3, 3, 1, 1),
    (10, 64, 56, 56, 64, 3, 3, 1, 1), (14, 64, 57, 41, 48, 3, 3, 1, 1), (5, 64, 57, 41, 32, 3, 3, 1, 1), (37, 128, 7, 7, 96, 3, 3, 1, 1),
    (3, 512, 7, 7, 512, 3, 3, 1, 1), (2, 1, 28, 28, 32, 5, 5, 1, 2), (3001, 768, 1, 1, 3072, 1, 1, 1, 0), (64, 512, 4, 4, 512, 3, 3, 1, 1),
    (100, 256, 5, 3, 512, 3, 3, 1, 1), (16, 128, 28, 28, 128, 3, 3, 1, 1), (16, 128, 28, 28, 256, 3, 3, 2, 1),
]


@pytest.mark.parametrize("shp", CONV_CASES)
def test_convolutions_stay_inside_results_and_workspaces(shp):
    N, C, H, W, K, R, S, st, pd = shp
    print("case", shp, flush=True)
    P, Q = wl.conv_out(H, pd, R, st), wl.conv_out(W, pd, S, st)
    x, w, g = (dev(wl.int8_codes(300, (N, H, W, C), "gauss")), dev(wl.int8_codes(301, (K, R, S, C), "gauss")),
               dev(wl.int8_codes(302, (N, P, Q, K), "gauss")))
    d = lpdt.ConvDesc.make(*shp)
    G = Guards()
    s1, s2 = dev(np.float32([0.01])), dev(np.float32([0.02]))
    lpdt.qconv_fwd(d, x, w, acc=G.tensor((N, P, Q, K), torch.int32), ws=G)
    G.check("qconv_fwd")
    lpdt.qconv_bwd_data(d, g, w, dx=G.tensor((N, H, W, C), torch.int32), ws=G)
    G.check("qconv_bwd_data")
    lpdt.qconv_bwd_weight(d, g, x, dw=G.tensor((K, R, S, C), torch.int32), ws=G)
    G.check("qconv_bwd_weight")
    y = G.tensor((N, P, Q, K), torch.float32)
    lpdt.qconv_fwd_f32(d, x, w, s1, s2, y=y, ws=G)
    G.check("qconv_fwd_f32")
    y2 = G.tensor((N, P, Q, K), torch.float32)
    y2.zero_()
    lpdt.qconv_fwd_f32_add(d, x, w, s1, s2, y2, ws=G)
    G.check("qconv_fwd_f32_add")
    lpdt.qconv_fwd_f32_absmax(d, x, w, s1, s2, y=G.tensor((N, P, Q, K), torch.float32), ws=G)
    G.check("qconv_fwd_f32_absmax")
    for accumulate in (False, True):
        dx = G.tensor((N, H, W, C), torch.float32)
        dx.zero_()
        lpdt.qconv_bwd_data_f32(d, g, w, s1, s2, dx=dx, accumulate=accumulate, ws=G)
        G.check("qconv_bwd_data_f32")
    lpdt.qconv_bwd_data_f32_absmax(d, g, w, s1, s2, dx=G.tensor((N, H, W, C), torch.float32), ws=G)
    G.check("qconv_bwd_data_f32_absmax")
    for beside in (0, 1):
        lpdt.qconv_set_wgrad_beside(beside)
        try:
            lpdt.qconv_bwd_weight_f32(d, g, x, s1, s2, dw=G.tensor((K, R, S, C), torch.float32), ws=G)
        finally:
            lpdt.qconv_set_wgrad_beside(0)
        G.check("qconv_bwd_weight_f32")


# N H W C groups
NORM_CASES = [(8, 32, 32, 16, 8), (2, 28, 28, 128, 32), (2, 7, 7, 512, 32), (5, 1, 1, 512, 32), (2, 9, 7, 48, 6), (2, 5, 5, 6, 3),
              (1, 70, 70, 64, 32), (3, 56, 56, 64, 32)]


@pytest.mark.parametrize("shape", NORM_CASES)
def test_normalisation_stays_inside_results_and_workspaces(shape):
    N, H, W, C, groups = shape
    print("case", shape, flush=True)
    g = wl.rng(701)
    v, gamma, beta = (dev((1.0 + 0.3 * g.standard_normal(C)).astype(np.float32)), dev((1.0 + 0.2 * g.standard_normal(C)).astype(np.float32)),
                      dev((0.1 * g.standard_normal(C)).astype(np.float32)))
    x, dy = dev(wl.images(700, N, H, W, C) * np.float32(2.0)), dev(wl.upstream_grad(702, (N, H, W, C)))
    G = Guards()
    y, r, amx, amn, _ = lpdt.range_evonorm_fwd(x, groups, v, gamma, beta, 1e-5, y=G.tensor((N, H, W, C), torch.float32),
                                               want_absmax=True, ws=G)
    G.check("range_evonorm_fwd")
    lpdt.range_evonorm_bwd(dy, x, groups, v, gamma, r, amx, amn, 1e-5, dx=G.tensor((N, H, W, C), torch.float32), want_absmax=True, ws=G)
    G.check("range_evonorm_bwd")
    if C % 4 == 0:
        lpdt.range_evonorm_fwd_q(x, groups, v, gamma, beta, 1e-5, q=G.tensor((N, H, W, C), torch.int8),
                                 y=G.tensor((N, H, W, C), torch.float32), ws=G)
        G.check("range_evonorm_fwd_q")
        if H >= 3 and W >= 3:
            out = lpdt.range_evonorm_maxpool_fwd(x, groups, v, gamma, beta, 3, 2, 1, 1e-5, want_absmax=True, ws=G)
            G.check("range_evonorm_maxpool_fwd")
            z, idx, r2, amx2, amn2 = out[:5]
            dz = dev(wl.upstream_grad(703, tuple(z.shape)))
            lpdt.range_evonorm_maxpool_bwd(dz, idx, x, groups, v, gamma, r2, amx2, amn2, 3, 2, 1, 1e-5, want_absmax=True, ws=G)
            G.check("range_evonorm_maxpool_bwd")


@pytest.mark.parametrize("n", [1, 7, 4096, 70001, 1 << 20, (1 << 22) + 3])
def test_quantizers_stay_inside_results_and_workspaces(n):
    x = dev(wl.rng(11).standard_normal(n).astype(np.float32))
    G = Guards()
    for rounding in (lpdt.ROUND_NEAREST, lpdt.ROUND_STOCHASTIC):
        lpdt.quantize(x, rounding, 5, 0, q=G.tensor((n,), torch.int8), scale=G.tensor((1,), torch.float32), ws=G)
        G.check("quantize")
    if n >= 64:
        cuts = [0, 16 * (n // 48), 16 * (n // 24), n]
        lpdt.quantize_segments(x, cuts[:-1], cuts[1:], lpdt.ROUND_NEAREST, 5, 0, q=G.tensor((n,), torch.int8),
                               scales=G.tensor((3,), torch.float32), ws=G)
        G.check("quantize_segments")


@pytest.mark.parametrize("agents,d", [(4, 1000), (16, 70001), (8, 1 << 18)])
def test_gossip_mix_stays_inside_its_workspace(agents, d):
    W = wl.ring_matrix(agents)
    X = dev(wl.rng(21).standard_normal((agents, d)).astype(np.float32))
    Xhat = X.clone()
    G = Guards()
    lpdt.gossip_mix(X, None, W, rate=1.0, ws=G)
    G.check("plain mix")
    offs = [0, d // 3, d]
    for keep in (0.01, 0.3):
        lpdt.gossip_mix(X, Xhat, W, rate=0.5, keep_ratio=keep, seg_offsets=offs, ws=G)
        G.check("choco mix")
