"""ctypes front end of the CPU oracle (``lpdt_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke`` and
the ``cpu_baseline`` leg of ``bench.py``; never by the product package.  All
arrays are numpy, NHWC / KRSC / [n][d]; floating-point results are float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liblpdt_oracle.so")
_SRC = os.path.join(_HERE, "lpdt_oracle.c")


def build(force=False):
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(_SRC):
        return _SO
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
    subprocess.check_call(cmd)
    return _SO


_lib = None


class ConvDesc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]

    @property
    def P(self):
        return (self.H + 2 * self.pad_h - self.R) // self.stride_h + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad_w - self.S) // self.stride_w + 1


def conv_desc(N, C, H, W, K, R, S, stride=1, pad=0):
    return ConvDesc(N, C, H, W, K, R, S, stride, stride, pad, pad)


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        _lib.orc_softmax_xent.restype = ctypes.c_double
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


class OracleError(RuntimeError):
    pass


def _chk(rc, what):
    if rc != 0:
        raise OracleError(f"{what}: oracle returned {rc} ({'int32 overflow' if rc == -1 else 'invalid argument'})")


def philox4x32_10(ctr, key):
    c = _c(ctr, np.uint32)
    k = _c(key, np.uint32)
    out = np.empty(4, np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sr_uniform(seed, offset, first, count):
    u = np.empty(count, np.float32)
    lib().orc_sr_uniform(ctypes.c_uint64(seed), ctypes.c_uint64(offset), ctypes.c_uint64(first),
                         ctypes.c_uint64(count), _p(u))
    return u


def quantize(x, rounding=0, seed=0, offset=0):
    """-> (int8 codes of x's shape, float32 scale)."""
    xf = _c(x, np.float32)
    q = np.empty(xf.shape, np.int8)
    s = ctypes.c_float(0)
    rc = lib().orc_quantize(_p(xf), ctypes.c_size_t(xf.size), int(rounding), ctypes.c_uint64(seed),
                            ctypes.c_uint64(offset), _p(q), ctypes.byref(s))
    _chk(rc, "quantize")
    return q, np.float32(s.value)


def dequantize(acc, sA, sB):
    a = _c(acc, np.int32)
    y = np.empty(a.shape, np.float64)
    lib().orc_dequantize(_p(a), ctypes.c_size_t(a.size), ctypes.c_float(sA), ctypes.c_float(sB), _p(y))
    return y


def qconv_fwd(d, xq, wq):
    xq = _c(xq, np.int8)
    wq = _c(wq, np.int8)
    assert xq.shape == (d.N, d.H, d.W, d.C) and wq.shape == (d.K, d.R, d.S, d.C)
    acc = np.empty((d.N, d.P, d.Q, d.K), np.int32)
    _chk(lib().orc_qconv_fwd(ctypes.byref(d), _p(xq), _p(wq), _p(acc)), "qconv_fwd")
    return acc


def qconv_bwd_data(d, gq, wq):
    gq = _c(gq, np.int8)
    wq = _c(wq, np.int8)
    assert gq.shape == (d.N, d.P, d.Q, d.K) and wq.shape == (d.K, d.R, d.S, d.C)
    dx = np.empty((d.N, d.H, d.W, d.C), np.int32)
    _chk(lib().orc_qconv_bwd_data(ctypes.byref(d), _p(gq), _p(wq), _p(dx)), "qconv_bwd_data")
    return dx


def qconv_bwd_weight(d, gq, xq):
    gq = _c(gq, np.int8)
    xq = _c(xq, np.int8)
    assert gq.shape == (d.N, d.P, d.Q, d.K) and xq.shape == (d.N, d.H, d.W, d.C)
    dw = np.empty((d.K, d.R, d.S, d.C), np.int32)
    _chk(lib().orc_qconv_bwd_weight(ctypes.byref(d), _p(gq), _p(xq), _p(dw)), "qconv_bwd_weight")
    return dw


def to_bf16(x):
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    x = _c(x, np.float32)
    y = np.empty(x.shape, np.uint16)
    lib().orc_to_bf16(_p(x), ctypes.c_size_t(x.size), _p(y))
    return y


def qconv_bwd_weight_bf16(d, g16, xq, sx):
    """g16 uint16 bf16 patterns [N,P,Q,K], xq int8 [N,H,W,C], sx float -> (dw f64 [K,R,S,C], sum of |terms| f64)."""
    g16 = _c(g16, np.uint16)
    xq = _c(xq, np.int8)
    assert g16.shape == (d.N, d.P, d.Q, d.K) and xq.shape == (d.N, d.H, d.W, d.C)
    dw = np.empty((d.K, d.R, d.S, d.C), np.float64)
    da = np.empty((d.K, d.R, d.S, d.C), np.float64)
    _chk(lib().orc_qconv_bwd_weight_bf16(ctypes.byref(d), _p(g16), _p(xq), ctypes.c_float(sx), _p(dw), _p(da)),
         "qconv_bwd_weight_bf16")
    return dw, da


def range_evonorm_fwd(x, groups, v, gamma, beta, eps=1e-5):
    """x float32 [N,H,W,C] -> (y f64, range f64 [N,groups], argmax i32, argmin i32)."""
    x = _c(x, np.float32)
    N, H, W, C = x.shape
    v, gamma, beta = (_c(t, np.float32) for t in (v, gamma, beta))
    y = np.empty(x.shape, np.float64)
    rng = np.empty((N, groups), np.float64)
    amx = np.empty((N, groups), np.int32)
    amn = np.empty((N, groups), np.int32)
    rc = lib().orc_range_evonorm_fwd(_p(x), N, H, W, C, int(groups), _p(v), _p(gamma), _p(beta),
                                     ctypes.c_double(eps), _p(y), _p(rng), _p(amx), _p(amn))
    _chk(rc, "range_evonorm_fwd")
    return y, rng, amx, amn


def range_evonorm_bwd(dy, x, groups, v, gamma, eps=1e-5):
    """-> (dx [N,H,W,C], dv [C], dgamma [C], dbeta [C]), float64."""
    x = _c(x, np.float32)
    dy = _c(dy, np.float64)
    N, H, W, C = x.shape
    v, gamma = (_c(t, np.float32) for t in (v, gamma))
    dx = np.empty(x.shape, np.float64)
    dv, dg, db = (np.empty(C, np.float64) for _ in range(3))
    rc = lib().orc_range_evonorm_bwd(_p(dy), _p(x), N, H, W, C, int(groups), _p(v), _p(gamma),
                                     ctypes.c_double(eps), _p(dx), _p(dv), _p(dg), _p(db))
    _chk(rc, "range_evonorm_bwd")
    return dx, dv, dg, db


def evonorm_s0_fwd(x, groups, v, gamma, beta, eps=1e-5):
    """EvoNorm-S0 (Eq. "en").  x float32 [N,H,W,C] -> (y f64, mean f64 [N,groups], var f64 [N,groups])."""
    x = _c(x, np.float32)
    N, H, W, C = x.shape
    v, gamma, beta = (_c(t, np.float32) for t in (v, gamma, beta))
    y = np.empty(x.shape, np.float64)
    mean, var = np.empty((N, groups), np.float64), np.empty((N, groups), np.float64)
    rc = lib().orc_evonorm_s0_fwd(_p(x), N, H, W, C, int(groups), _p(v), _p(gamma), _p(beta), ctypes.c_double(eps),
                                  _p(y), _p(mean), _p(var))
    _chk(rc, "evonorm_s0_fwd")
    return y, mean, var


def evonorm_s0_bwd(dy, x, groups, v, gamma, eps=1e-5):
    """-> (dx [N,H,W,C], dv [C], dgamma [C], dbeta [C]), float64."""
    x = _c(x, np.float32)
    dy = _c(dy, np.float64)
    N, H, W, C = x.shape
    v, gamma = (_c(t, np.float32) for t in (v, gamma))
    dx = np.empty(x.shape, np.float64)
    dv, dg, db = (np.empty(C, np.float64) for _ in range(3))
    rc = lib().orc_evonorm_s0_bwd(_p(dy), _p(x), N, H, W, C, int(groups), _p(v), _p(gamma), ctypes.c_double(eps),
                                  _p(dx), _p(dv), _p(dg), _p(db))
    _chk(rc, "evonorm_s0_bwd")
    return dx, dv, dg, db


def range_bn_fwd(x, gamma, beta, eps=1e-5):
    """Range batch-norm (Eq. "rbn").  x float32 [N,H,W,C] -> (y f64, mean f64 [C], range f64 [C], argmax i64 [C], argmin i64 [C])."""
    x = _c(x, np.float32)
    N, H, W, C = x.shape
    gamma, beta = (_c(t, np.float32) for t in (gamma, beta))
    y = np.empty(x.shape, np.float64)
    mean, rng = np.empty(C, np.float64), np.empty(C, np.float64)
    amx, amn = np.empty(C, np.int64), np.empty(C, np.int64)
    rc = lib().orc_range_bn_fwd(_p(x), N, H, W, C, _p(gamma), _p(beta), ctypes.c_double(eps), _p(y), _p(mean), _p(rng),
                                _p(amx), _p(amn))
    _chk(rc, "range_bn_fwd")
    return y, mean, rng, amx, amn


def range_bn_bwd(dy, x, gamma, eps=1e-5):
    """-> (dx [N,H,W,C], dgamma [C], dbeta [C]), float64."""
    x = _c(x, np.float32)
    dy = _c(dy, np.float64)
    N, H, W, C = x.shape
    gamma = _c(gamma, np.float32)
    dx = np.empty(x.shape, np.float64)
    dg, db = np.empty(C, np.float64), np.empty(C, np.float64)
    rc = lib().orc_range_bn_bwd(_p(dy), _p(x), N, H, W, C, _p(gamma), ctypes.c_double(eps), _p(dx), _p(dg), _p(db))
    _chk(rc, "range_bn_bwd")
    return dx, dg, db


def gossip_mix(x, xhat, Wm, eta=1.0, keep_ratio=1.0, seg_offsets=None):
    """x float32 [n,d]; xhat float32 [n,d] or None (plain mix).
    -> (x_new float64 [n,d], xhat_new float32 [n,d] or None)."""
    x = _c(x, np.float32)
    n, d = x.shape
    Wm = _c(Wm, np.float32)
    assert Wm.shape == (n, n)
    if seg_offsets is None:
        seg_offsets = [0, d]
    seg = _c(seg_offsets, np.int64)
    out = np.empty((n, d), np.float64)
    xh = None if xhat is None else np.array(xhat, dtype=np.float32, order="C", copy=True)
    rc = lib().orc_gossip_mix(_p(x), None if xh is None else _p(xh), n, ctypes.c_size_t(d), _p(Wm),
                              ctypes.c_float(eta), ctypes.c_double(keep_ratio), _p(seg), len(seg) - 1, _p(out))
    _chk(rc, "gossip_mix")
    return out, xh


MIX_PLAIN, MIX_CHOCO, MIX_DEEPSQUEEZE = 0, 1, 2


def gossip_mix_ex(x, state, Wm, eta=1.0, keep_ratio=1.0, seg_offsets=None, mode=MIX_PLAIN, u=None):
    """One gossip step of the supplement's variants.  state: xhat (CHOCO) / delta (Deep-Squeeze) float32 [n,d] or None;
    u: push-sum bias weights float32 [n] or None.
    -> (x_new float64 [n,d], state_new float32 or None, u_new float64 [n] or None, z float64 [n,d] or None)."""
    x = _c(x, np.float32)
    n, d = x.shape
    Wm = _c(Wm, np.float32)
    assert Wm.shape == (n, n)
    if seg_offsets is None:
        seg_offsets = [0, d]
    seg = _c(seg_offsets, np.int64)
    out = np.empty((n, d), np.float64)
    st = None if state is None else np.array(state, dtype=np.float32, order="C", copy=True)
    uu = None if u is None else _c(u, np.float32)
    u_out = None if u is None else np.empty(n, np.float64)
    z_out = None if u is None else np.empty((n, d), np.float64)
    rc = lib().orc_gossip_mix_ex(_p(x), None if st is None else _p(st), n, ctypes.c_size_t(d), _p(Wm), ctypes.c_float(eta),
                                 ctypes.c_double(keep_ratio), _p(seg), len(seg) - 1, int(mode),
                                 None if uu is None else _p(uu), _p(out), None if u_out is None else _p(u_out),
                                 None if z_out is None else _p(z_out))
    _chk(rc, "gossip_mix_ex")
    return out, st, u_out, z_out


def add(a, b):
    a = _c(a, np.float64)
    b = _c(b, np.float64)
    y = np.empty(a.shape, np.float64)
    lib().orc_add(_p(a), _p(b), ctypes.c_size_t(a.size), _p(y))
    return y


def maxpool_fwd(x, k, stride, pad):
    x = _c(x, np.float32)
    N, H, W, C = x.shape
    P = (H + 2 * pad - k) // stride + 1
    Q = (W + 2 * pad - k) // stride + 1
    y = np.empty((N, P, Q, C), np.float32)
    idx = np.empty((N, P, Q, C), np.int32)
    lib().orc_maxpool_fwd(_p(x), N, H, W, C, k, stride, pad, _p(y), _p(idx))
    return y, idx


def maxpool_bwd(dy, idx, in_shape):
    dy = _c(dy, np.float64)
    idx = _c(idx, np.int32)
    N, H, W, C = in_shape
    _, P, Q, _ = dy.shape
    dx = np.empty(in_shape, np.float64)
    lib().orc_maxpool_bwd(_p(dy), _p(idx), N, H, W, C, P, Q, _p(dx))
    return dx


def avgpool_fwd(x):
    x = _c(x, np.float32)
    N, H, W, C = x.shape
    y = np.empty((N, C), np.float64)
    lib().orc_avgpool_fwd(_p(x), N, H * W, C, _p(y))
    return y


def avgpool_bwd(dy, in_shape):
    dy = _c(dy, np.float64)
    N, H, W, C = in_shape
    dx = np.empty(in_shape, np.float64)
    lib().orc_avgpool_bwd(_p(dy), N, H * W, C, _p(dx))
    return dx


def softmax_xent(logits, labels):
    lg = _c(logits, np.float32)
    lb = _c(labels, np.int32)
    N, classes = lg.shape
    dl = np.empty((N, classes), np.float64)
    loss = lib().orc_softmax_xent(_p(lg), _p(lb), N, classes, _p(dl))
    return float(loss), dl


def sgd(x, g, lr):
    x = _c(x, np.float32)
    g = _c(g, np.float32)
    y = np.empty(x.shape, np.float64)
    lib().orc_sgd(_p(x), _p(g), ctypes.c_size_t(x.size), ctypes.c_float(lr), _p(y))
    return y
