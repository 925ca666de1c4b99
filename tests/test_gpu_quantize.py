"""GPU parity of the quantizer against the oracle: codes and scale bit-exact under the same
Philox counters; dequantized values within 1e-5 relative."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import assert_close, dev, host

pytestmark = pytest.mark.gpu
import paper_2111_09389_amd as lpdt  # noqa: E402  (a broken import must fail the run, not skip it)

SIZES = [1, 3, 4, 5, 255, 1024, 4099, 131072, 1 << 20, (1 << 20) + 7, 5_000_003]


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("rounding", [0, 1])
def test_quantize_bit_exact(orc, n, rounding):
    x = wl.rng(100 + n % 97).standard_normal(n).astype(np.float32) * np.float32(0.37)
    seed, offset = wl.PHILOX_SEED, (7 << 32) + 12345
    q_ref, s_ref = orc.quantize(x, rounding, seed, offset)
    q, s = lpdt.quantize(dev(x), rounding, seed, offset)
    assert host(s)[0] == s_ref
    assert np.array_equal(host(q), q_ref)


def test_quantize_offset_carry_and_geometry_independence(orc):
    # the Philox block counter crosses 2^32 inside the tensor; a sub-range quantized on its own with the
    # matching offset gives the same codes (the stream depends on the logical index only)
    n = 1 << 16
    x = wl.upstream_grad(5, (n,))
    x[0] = 1.0                                           # pins the abs-max for both calls
    seed, offset = 0xDEADBEEFCAFEF00D, (1 << 32) - 100
    q_ref, _ = orc.quantize(x, 1, seed, offset)
    q, _ = lpdt.quantize(dev(x), 1, seed, offset)
    assert np.array_equal(host(q), q_ref)
    sub = np.concatenate([x[:1], x[4096:8192]])          # keep the abs-max element, shift the rest
    amax = dev(np.array([1.0], np.float32))
    q_sub, _ = lpdt.quantize_with_absmax(dev(x[4096:8192].copy()), amax, 1, seed, offset + 1024)
    assert np.array_equal(host(q_sub), q_ref[4096:8192])
    assert sub.size == 4097


@pytest.mark.parametrize("rounding", [0, 1])
def test_quantize_with_absmax_matches(orc, rounding):
    x = wl.images(9, 8, 32, 32, 16)
    q_ref, s_ref = orc.quantize(x, rounding, 3, 4)
    amax = dev(np.array([np.abs(x).max()], np.float32))
    q, s = lpdt.quantize_with_absmax(dev(x), amax, rounding, 3, 4)
    assert host(s)[0] == s_ref and np.array_equal(host(q), q_ref)


def test_quantize_edge_values(orc):
    for x in (np.zeros(1000, np.float32),
              np.array([-1, 0.5, 0.25, 1], np.float32),
              np.array([127, 62.5, 61.5, -62.5, -0.5, 0.5, 1.5], np.float32),
              (wl.int8_codes(3, (4096,), "uniform").astype(np.float32) * np.float32(0.0173)),
              np.array([1e-30, -3e-30, 2e-30], np.float32), np.array([3e38, -1e38, 5e37], np.float32),
              np.array([1e-45, -5e-46, 0.0], np.float32), np.array([3.6e-37, -1e-37, 0.0, 2e-38], np.float32),   # 127/absmax overflows: zero
              np.array([4e-37, -2e-37, 0.0, 1e-37], np.float32)):
        for rounding in (0, 1):
            q_ref, s_ref = orc.quantize(x, rounding, 11, 0)
            q, s = lpdt.quantize(dev(x), rounding, 11, 0)
            assert host(s)[0] == s_ref and np.array_equal(host(q), q_ref)


def test_dequantize(orc):
    acc = wl.rng(4).integers(-2 ** 31, 2 ** 31, size=100_003, dtype=np.int64).astype(np.int32)
    acc[:4] = [0, 1, -1, 2 ** 31 - 1]
    sA, sB = np.float32(0.0123), np.float32(3.3e-4)
    ref = orc.dequantize(acc, sA, sB)
    y = lpdt.dequantize(dev(acc), dev(np.array([sA])), dev(np.array([sB])))
    assert_close(host(y), ref, 1e-5, 0.0, "dequantize")
    base = wl.rng(5).standard_normal(acc.size).astype(np.float32)
    yb = dev(base)
    lpdt.dequantize(dev(acc), dev(np.array([sA])), dev(np.array([sB])), y=yb, accumulate=True)
    assert_close(host(yb), ref + base, 1e-5, float(np.abs(ref).max()) * 1e-2, "dequantize accumulate")


def test_determinism():
    x = dev(wl.upstream_grad(6, (1 << 20,)))
    a, _ = lpdt.quantize(x, 1, 5, 6)
    b, _ = lpdt.quantize(x, 1, 5, 6)
    assert torch.equal(a, b)


@pytest.mark.parametrize("rounding", [0, 1])
def test_quantize_segments_equals_per_slice_quantize(orc, rounding):
    """Slices of one buffer, own scale each: the oracle's quantizer on every slice, with slice s at counter offset + s*2^24."""
    g = wl.rng(77)
    x = (g.standard_normal(40_000) * 0.1).astype(np.float32)
    x[300:420] = 0.0                                         # an all-zero slice: scale 0, codes 0
    begins = [0, 300, 420, 4096 + 4, 9001, 30_000]           # 9001: a slice that does not start on a 16-byte boundary
    ends = [300, 420, 4100, 9001, 29_999, 40_000]            # 29_999..30_000: a gap that must stay untouched
    seed, offset = wl.PHILOX_SEED, 12345
    q0 = torch.full((40_000,), 77, dtype=torch.int8, device="cuda")
    q, scales = lpdt.quantize_segments(dev(x), begins, ends, rounding, seed, offset, q=q0)
    q, scales = host(q), host(scales)
    for s, (b, e) in enumerate(zip(begins, ends)):
        qr, sr = orc.quantize(x[b:e], rounding, seed, offset + (s << 24))
        assert np.array_equal(q[b:e], qr), f"slice {s}"
        assert scales[s] == np.float32(sr)
    assert q[29_999] == 77
