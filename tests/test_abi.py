"""Host-side checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before enqueueing any device work."""
import ctypes
import os
import re

import pytest

import paper_2111_09389_amd as lpdt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x10000)      # aligned, never dereferenced: every call below fails validation first
sz = ctypes.c_size_t


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(lpdt.library_path()):
        from paper_2111_09389_amd import build
        build.build(verbose=False)
    return lpdt.lib()


def test_header_symbols_are_exported(L):
    text = open(os.path.join(ROOT, "include", "lpdt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(lpdt_[a-z0-9_]+)\s*\(", text)))
    assert len(declared) >= 25
    for name in declared:
        assert hasattr(L, name), f"{name} declared in lpdt.h but not exported"
    assert sorted(lpdt.EXPORTS) == declared
    assert L.lpdt_version() >= 100


def test_no_cuda_or_torch_symbols_in_signatures():
    text = open(os.path.join(ROOT, "include", "lpdt.h")).read()
    assert "torch" not in text and "at::" not in text and "hipStream_t stream" not in text


def _err(L):
    return L.lpdt_last_error().decode()


def test_quantize_argument_errors(L):
    u64 = ctypes.c_uint64
    assert L.lpdt_quantize(None, sz(4), 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(4096), None) == -1
    assert L.lpdt_quantize(FAKE, sz(0), 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(4096), None) == -2
    assert L.lpdt_quantize(FAKE, sz(4), 7, u64(0), u64(0), FAKE, FAKE, FAKE, sz(4096), None) == -1
    assert "rounding" in _err(L)
    assert L.lpdt_quantize(ctypes.c_void_p(0x10004), sz(4), 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(4096), None) == -1
    assert L.lpdt_quantize(FAKE, sz(4), 0, u64(0), u64(0), FAKE, FAKE, None, sz(0), None) == -3
    assert L.lpdt_quantize(FAKE, sz(4), 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(16), None) == -3
    assert "workspace" in _err(L)
    assert L.lpdt_quantize(FAKE, sz(4), 0, u64(0), u64(0), FAKE, FAKE, ctypes.c_void_p(0x10010), sz(8192), None) == -3


def test_quantize_segments_argument_errors(L):
    u64, i64 = ctypes.c_uint64, ctypes.c_int64
    b, e = (i64 * 2)(0, 16), (i64 * 2)(16, 40)
    need = L.lpdt_quantize_segments_workspace_bytes(2)
    assert need >= 2 * 16 + 2 * 4
    assert L.lpdt_quantize_segments(FAKE, b, e, 0, 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(need), None) == -2
    assert L.lpdt_quantize_segments(None, b, e, 2, 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(need), None) == -1
    assert L.lpdt_quantize_segments(FAKE, b, e, 2, 3, u64(0), u64(0), FAKE, FAKE, FAKE, sz(need), None) == -1
    assert L.lpdt_quantize_segments(FAKE, b, e, 2, 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(8), None) == -3
    empty = (i64 * 2)(16, 16)
    assert L.lpdt_quantize_segments(FAKE, b, empty, 2, 0, u64(0), u64(0), FAKE, FAKE, FAKE, sz(need), None) == -2
    assert "slice 1" in _err(L)
    huge = (i64 * 2)(16, (1 << 26) + 1 + 16)
    assert L.lpdt_quantize_segments(FAKE, b, huge, 2, 1, u64(0), u64(0), FAKE, FAKE, FAKE, sz(need), None) == -2


def test_conv_argument_errors(L):
    good = lpdt.ConvDesc.make(2, 16, 8, 8, 16, 3, 3, 1, 1)
    assert L.lpdt_qconv_fwd(None, FAKE, FAKE, FAKE, None, sz(0), None) == -1
    assert L.lpdt_qconv_fwd(ctypes.byref(good), None, FAKE, FAKE, None, sz(0), None) == -1
    bad = lpdt.ConvDesc.make(2, 16, 8, 8, 16, 3, 3, 0, 1)
    assert L.lpdt_qconv_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, sz(0), None) == -1
    bad = lpdt.ConvDesc.make(2, 16, 2, 2, 16, 7, 7, 1, 0)
    assert L.lpdt_qconv_bwd_weight(ctypes.byref(bad), FAKE, FAKE, FAKE, None, sz(0), None) == -1
    assert "filter larger" in _err(L)
    bad = lpdt.ConvDesc.make(2, 16, 8, 8, 16, 3, 3, 1, 3)
    assert L.lpdt_qconv_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, sz(0), None) == -2
    # backward-data needs room for the transposed filter
    need = L.lpdt_qconv_bwd_data_workspace_bytes(ctypes.byref(good))
    assert need >= 16 * 9 * 16
    assert L.lpdt_qconv_bwd_data(ctypes.byref(good), FAKE, FAKE, FAKE, None, sz(0), None) == -3
    assert L.lpdt_qconv_bwd_data(ctypes.byref(good), FAKE, FAKE, FAKE, FAKE, sz(need - 1), None) == -3
    huge = lpdt.ConvDesc.make(1 << 20, 64, 64, 64, 64, 3, 3, 1, 1)
    assert L.lpdt_qconv_fwd(ctypes.byref(huge), FAKE, FAKE, FAKE, None, sz(0), None) == -2


def test_range_evonorm_argument_errors(L):
    f = ctypes.c_float
    args = lambda C, groups, eps=1e-5: (FAKE, 2, 4, 4, C, groups, FAKE, FAKE, FAKE, f(eps), FAKE, FAKE, FAKE, FAKE, None,
                                        FAKE, sz(1 << 20), None)
    assert L.lpdt_range_evonorm_fwd(*args(16, 3)) == -2          # groups must divide C
    assert L.lpdt_range_evonorm_fwd(*args(16, 16)) == -2         # one channel per group: C(1) undefined
    assert "2 channels per group" in _err(L)
    assert L.lpdt_range_evonorm_fwd(*args(16, 0)) == -2
    assert L.lpdt_range_evonorm_fwd(*args(16, 8, eps=-1.0)) == -1
    a = list(args(16, 8)); a[15] = None; a[16] = sz(0)
    assert L.lpdt_range_evonorm_fwd(*a) == -3
    assert L.lpdt_range_evonorm_fwd_workspace_bytes(2, 4, 4, 16, 8) >= 2 * 8 * 16
    assert L.lpdt_range_evonorm_bwd_workspace_bytes(2, 4, 4, 16, 8) > 0


def test_gossip_argument_errors(L):
    import numpy as np
    import workloads as wl
    f, dbl = ctypes.c_float, ctypes.c_double

    def call(Wm, n, xhat=None, keep=1.0, seg=None, nseg=0, ws=None, wsb=0, d=1000):
        Wc = (ctypes.c_float * (n * n))(*np.asarray(Wm, np.float32).ravel().tolist())
        segc = None if seg is None else (ctypes.c_int64 * len(seg))(*seg)
        return L.lpdt_gossip_mix(FAKE, xhat, n, sz(d), Wc, f(1.0), dbl(keep), segc, nseg, ws, sz(wsb), None)

    Wm = wl.ring_matrix(8)
    bad = Wm.copy(); bad[0, 0] += 0.1
    assert call(bad, 8) == -1 and "sums to" in _err(L)
    bad = Wm.copy(); bad[0, 1] += 0.1; bad[0, 7] -= 0.1            # rows fine, columns not
    assert call(bad, 8) == -1 and "column" in _err(L)
    dense = np.full((16, 16), 1 / 16, np.float32)
    assert call(dense, 16) == -2                                     # more than 8 non-zeros per row
    assert call(np.eye(65, dtype=np.float32), 65) == -2
    assert call(Wm, 8, xhat=FAKE, keep=0.0) == -1
    assert call(Wm, 8, xhat=FAKE, keep=0.1, seg=[0, 500, 900], nseg=2) == -1      # must end at d
    assert call(Wm, 8, xhat=FAKE, keep=0.1, seg=[0, 600, 500, 1000], nseg=3) == -1
    assert call(Wm, 8, xhat=FAKE, keep=0.1) == -3                    # CHOCO needs a workspace
    assert L.lpdt_gossip_mix_workspace_bytes(8, sz(1000), 1, 1) >= 8 * 1000 * 8
    assert L.lpdt_gossip_mix_workspace_bytes(8, sz(1000), 1, 0) == 0


def test_gossip_ex_argument_errors(L):
    import numpy as np
    import workloads as wl
    f, dbl = ctypes.c_float, ctypes.c_double

    def call(Wm, n, state=None, mode=0, u=None, z=None, ws=None, wsb=0, d=1000):
        Wc = (ctypes.c_float * (n * n))(*np.asarray(Wm, np.float32).ravel().tolist())
        return L.lpdt_gossip_mix_ex(FAKE, state, n, sz(d), Wc, f(1.0), dbl(0.1), None, 0, mode, u, z, ws, sz(wsb), None)

    ring, dirg = wl.ring_matrix(8), wl.directed_matrix(8)
    assert call(ring, 8, mode=7) == -1 and "mode" in _err(L)
    assert call(ring, 8, state=None, mode=2) == -1 and "state" in _err(L)          # Deep-Squeeze without its error memory
    assert call(ring, 8, state=FAKE, mode=0) == -1                                 # plain mix takes no state
    assert call(ring, 8, z=FAKE) == -1 and "push-sum" in _err(L)                   # z without u
    assert call(dirg, 8) == -1 and "row" in _err(L)                                # directed graph needs push-sum weights
    assert call(dirg, 8, u=FAKE) == -3                                             # accepted with u; then the workspace is missing
    bad = dirg.copy(); bad[0, 0] += 0.2
    assert call(bad, 8, u=FAKE) == -1 and "column" in _err(L)
    need = L.lpdt_gossip_mix_ex_workspace_bytes(8, sz(1000), 1, 2, 1)
    assert need > L.lpdt_gossip_mix_ex_workspace_bytes(8, sz(1000), 1, 2, 0) > 0
    assert L.lpdt_gossip_mix_ex_workspace_bytes(8, sz(1000), 1, 0, 0) == 0
    assert call(ring, 8, state=FAKE, mode=2, ws=FAKE, wsb=16) == -3


def test_glue_argument_errors(L):
    assert L.lpdt_add(None, FAKE, sz(4), FAKE, None) == -1
    assert L.lpdt_sgd(FAKE, FAKE, sz(0), ctypes.c_float(0.1), None) == -2
    assert L.lpdt_maxpool_fwd(FAKE, 1, 4, 4, 8, 2, 0, 0, FAKE, FAKE, None) == -1
    assert L.lpdt_softmax_xent(FAKE, FAKE, 4, 5000, FAKE, FAKE, None) == -2
    assert L.lpdt_dequantize(FAKE, sz(0), FAKE, FAKE, FAKE, 0, None) == -2


def test_product_package_does_not_import_the_oracle():
    import subprocess, sys
    code = ("import sys; import paper_2111_09389_amd; "
            "bad=[m for m in sys.modules if m=='oracle' or m.startswith('oracle.')]; sys.exit(1 if bad else 0)")
    assert subprocess.run([sys.executable, "-c", code], cwd=ROOT).returncode == 0
    for fn in os.listdir(os.path.join(ROOT, "paper_2111_09389_amd")):
        if fn.endswith(".py"):
            assert "oracle" not in open(os.path.join(ROOT, "paper_2111_09389_amd", fn)).read().lower().replace("no cpu fallback", "")


def test_gossip_sample_stride_setter(L):
    assert L.lpdt_gossip_set_sample_stride(-2) == -1 and "stride" in _err(L)
    assert L.lpdt_gossip_set_sample_stride(3) == 0 and L.lpdt_gossip_set_sample_stride(-1) == 0


def test_qconv_kernel_id_argument_errors(L):
    d = lpdt.ConvDesc.make(2, 64, 8, 8, 64, 3, 3, 1, 1)
    assert L.lpdt_qconv_kernel_id(ctypes.byref(d), 5) == -1
    assert L.lpdt_qconv_kernel_id(None, 0) == -1
    assert L.lpdt_qconv_kernel_id(ctypes.byref(d), 0) >= 10


def test_planner_gives_the_benchmark_layers_their_kernels():
    """lpdt_qconv_kernel_id does no GPU work: the table of test_gpu_fullsize (which kernel family and tile each benchmark
    layer's three products take) is checked here too, so a planner change shows up without a GPU."""
    import test_gpu_fullsize as full
    for name, shp in full.LAYERS.items():
        ld = lpdt.ConvDesc.make(*shp)
        assert tuple(lpdt.qconv_kernel_id(ld, i) for i in range(3)) == full.KERNELS[name], name
