"""lpdt_quantize_static (the quantizer that takes no workspace: its abs-max partials live in a fixed device array inside
the library) against lpdt_quantize, the entry point it is a variant of: codes and scale bit for bit, on two calls in a
row that share the array, the second with a smaller input.  Collected last on purpose."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2111_09389_amd as lpdt
import workloads as wl
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


def _static(L, x, rounding, seed, offset):
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    s = torch.empty(1, dtype=torch.float32, device=x.device)
    rc = L.lpdt_quantize_static(ctypes.c_void_p(x.data_ptr()), ctypes.c_size_t(x.numel()), rounding, ctypes.c_uint64(seed),
                                ctypes.c_uint64(offset), ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(s.data_ptr()),
                                ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, L.lpdt_last_error().decode()
    return q, s


@pytest.mark.parametrize("rounding", [0, 1])
def test_static_quantizer_matches_workspace_quantizer(orc, rounding):
    L = lpdt.lib()
    seed, offset = wl.PHILOX_SEED, (3 << 32) + 77
    # the first call fills all 1024 partials of the shared array with a large abs-max; the second, smaller and with a
    # much smaller abs-max, must not see any of them
    big = wl.rng(41).standard_normal(6_000_011).astype(np.float32) * np.float32(5.0)
    small = wl.rng(42).standard_normal(70_001).astype(np.float32) * np.float32(1e-3)
    for x in (big, small):
        xd = dev(x)
        q0, s0 = lpdt.quantize(xd, rounding, seed, offset)
        q1, s1 = _static(L, xd, rounding, seed, offset)
        assert host(s1)[0] == host(s0)[0]
        assert np.array_equal(host(q1), host(q0))
        q_ref, s_ref = orc.quantize(x, rounding, seed, offset)
        assert host(s1)[0] == s_ref and np.array_equal(host(q1), q_ref)


def test_static_quantizer_rejects_oversize():
    L = lpdt.lib()
    L.lpdt_quantize_static_max_len.restype = ctypes.c_size_t
    fake = ctypes.c_void_p(0x10000)
    n = L.lpdt_quantize_static_max_len() + 1
    assert L.lpdt_quantize_static(fake, ctypes.c_size_t(n), 0, ctypes.c_uint64(0), ctypes.c_uint64(0), fake, fake, None) == -2
    assert "maximum" in L.lpdt_last_error().decode()
