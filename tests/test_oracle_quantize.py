"""Pins of the oracle's Philox generator and 8-bit quantizer (Section 3, "Low Precision
Training"; grid: symmetric per-tensor, scale = absmax/127, codes in [-127,127])."""
import os

import numpy as np

import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers(orc):
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = orc.philox4x32_10(v[0:4], v[4:6])
        assert [int(o) for o in out] == v[6:10]


def test_sr_uniform_counter_mapping(orc):
    # element i uses word i%4 of block offset + i//4, top 24 bits
    seed, off = 0x0123456789ABCDEF, (1 << 32) - 2     # block counter crosses the 32-bit carry
    u = orc.sr_uniform(seed, off, 0, 16)
    for i in range(16):
        blk = off + i // 4
        w = orc.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert u[i] == np.float32(int(w[i % 4]) >> 8) * np.float32(2.0 ** -24)
    assert np.array_equal(orc.sr_uniform(seed, off, 5, 7), u[5:12])   # depends on the logical index only
    assert (u >= 0).all() and (u < 1).all()


def test_sr_uniform_chi_square(orc):
    u = orc.sr_uniform(wl.PHILOX_SEED, 0, 0, 1 << 20)
    hist = np.bincount((u * 256).astype(np.int64), minlength=256)
    exp = (1 << 20) / 256
    chi2 = ((hist - exp) ** 2 / exp).sum()
    assert chi2 < 255 + 5 * np.sqrt(2 * 255)     # 5 sigma
    assert abs(u.mean() - 0.5) < 5 / np.sqrt(12 * (1 << 20))


def test_hand_example_rtn(orc):
    # t = x*127 = [-127, 63.5, 31.75, 127]; 63.5 -> 64 (even), 31.75 -> 32
    q, s = orc.quantize(np.array([-1, 0.5, 0.25, 1], np.float32))
    assert q.tolist() == [-127, 64, 32, 127]
    assert s == np.float32(1.0) / np.float32(127.0)
    # ties go to the even code in both directions
    q, _ = orc.quantize(np.array([127, 62.5, 61.5, -62.5, -0.5, 0.5, 1.5], np.float32))
    assert q.tolist() == [127, 62, 62, -62, 0, 0, 2]


def test_grid_invariants_rtn(orc):
    x = wl.images(1, 4, 32, 32, 16) * np.float32(3.7)
    q, s = orc.quantize(x)
    a = np.abs(x).max()
    assert s == np.float32(a) / np.float32(127)
    assert q.min() >= -127 and q.max() <= 127
    assert (np.abs(q[np.abs(x) == a]) == 127).all()
    err = np.abs(x.astype(np.float64) - q.astype(np.float64) * float(s))
    assert err.max() <= float(s) / 2 * (1 + 2.0 ** -20)
    q2, s2 = orc.quantize(-x)
    assert s2 == s and np.array_equal(q2, -q)          # sign symmetry
    # monotone: sorting x sorts the codes
    o = np.argsort(x.ravel(), kind="stable")
    assert (np.diff(q.ravel()[o].astype(np.int32)) >= 0).all()


def test_on_grid_inputs_are_fixed_points(orc):
    j = wl.int8_codes(2, (4096,), "uniform")
    j[0] = 127
    for s0 in (np.float32(0.03125), np.float32(0.0173), np.float32(1e-3)):
        x = j.astype(np.float32) * s0
        q, s = orc.quantize(x)
        assert np.array_equal(q, j)
        qs, _ = orc.quantize(x, rounding=1, seed=7, offset=3)
        # on-grid values may be off by fp32 rounding of x*inv, but SR must stay within floor/ceil of t
        assert np.abs(qs.astype(np.int32) - j).max() <= 1


def test_zero_and_tiny(orc):
    q, s = orc.quantize(np.zeros(17, np.float32))
    assert s == 0 and not q.any()
    q, s = orc.quantize(np.zeros(17, np.float32), rounding=1, seed=1)
    assert s == 0 and not q.any()
    q, s = orc.quantize(np.array([3.0], np.float32))
    assert q.tolist() == [127]


def test_abs_max_too_small_for_a_grid_counts_as_zero(orc):
    # 127/absmax overflows fp32 below about 3.7e-37 (subnormals included): codes 0, scale 0, for both roundings;
    # just above the limit the grid still holds
    for a in (1e-45, 1.2e-38, 3.6e-37):
        x = np.array([a, -a / 2, 0.0, a / 4], np.float32)
        for rounding in (0, 1):
            q, s = orc.quantize(x, rounding, 5, 0)
            assert s == 0.0 and not q.any()
    x = np.array([4e-37, -2e-37, 0.0, 1e-37], np.float32)
    q, s = orc.quantize(x, 0, 5, 0)
    assert s > 0 and list(q) == [127, -64, 0, 32] and np.all(np.abs(x - q.astype(np.float32) * s) <= s / 2 * (1 + 2 ** -20))


def test_sr_floor_ceil_and_determinism(orc):
    x = wl.upstream_grad(3, (8, 32, 32, 16))
    q, s = orc.quantize(x, rounding=1, seed=wl.PHILOX_SEED, offset=11)
    inv = np.float32(127) / np.abs(x).max()
    t = x * inv                                            # fp32 multiply
    f = np.floor(t)
    assert ((q == f) | (q == f + 1) | (np.abs(t) > 127)).all()
    assert np.abs(x.astype(np.float64) - q * float(s)).max() < float(s) * (1 + 1e-6)
    q_same, _ = orc.quantize(x, rounding=1, seed=wl.PHILOX_SEED, offset=11)
    q_other, _ = orc.quantize(x, rounding=1, seed=wl.PHILOX_SEED, offset=12 + x.size)
    assert np.array_equal(q, q_same) and not np.array_equal(q, q_other)
    # the decision is exactly u < frac with the documented uniform
    u = orc.sr_uniform(wl.PHILOX_SEED, 11, 0, x.size).reshape(x.shape)
    expect = np.clip(f + (u < (t - f)), -127, 127).astype(np.int8)
    assert np.array_equal(q, expect)


def test_sr_unbiased(orc):
    # one value repeated under 2^20 distinct counters: mean of dequantised codes -> x
    val = np.float32(0.3337)
    x = np.full(1 << 20, val, np.float32)
    x[0] = 1.0                                              # fixes absmax = 1 -> t = 42.38
    q, s = orc.quantize(x, rounding=1, seed=99, offset=0)
    t = float(val) * 127
    frac = t - np.floor(t)
    mean_code = q[1:].astype(np.float64).mean()
    sigma = np.sqrt(frac * (1 - frac) / (x.size - 1))
    assert abs(mean_code - t) < 4 * sigma + 1e-5
    assert set(np.unique(q[1:]).tolist()) == {42, 43}


def test_dequantize(orc):
    acc = np.array([0, 1, -5, 2 ** 31 - 1, -2 ** 31], np.int32)
    y = orc.dequantize(acc, np.float32(0.5), np.float32(0.25))
    assert np.array_equal(y, acc.astype(np.float64) * 0.125)
