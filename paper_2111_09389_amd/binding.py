"""ctypes binding of liblpdt.so with the same names as the C entry points."""
import ctypes
import os

import torch

__all__ = [
    "LpdtError", "ConvDesc", "lib", "library_path", "ROUND_NEAREST", "ROUND_STOCHASTIC",
    "quantize", "quantize_static", "quantize_with_absmax", "quantize_segments", "dequantize",
    "qconv_fwd", "qconv_bwd_data", "qconv_bwd_weight", "qconv_kernel_id", "qconv_fwd_f32", "qconv_fwd_f32_add", "qconv_ren_fwd_q", "qconv_bwd_data_f32", "qconv_bwd_weight_f32",
    "to_bf16", "qconv_bwd_weight_bf16",
    "range_evonorm_fwd", "range_evonorm_fwd_q", "range_evonorm_bwd", "range_evonorm_maxpool_fwd", "range_evonorm_maxpool_bwd", "qconv_bwd_data_pack_filter", "qconv_bwd_data_pack_filters", "qconv_bwd_data_f32_packed", "qconv_fwd_f32_absmax", "qconv_bwd_data_f32_absmax", "evonorm_s0_fwd", "evonorm_s0_bwd", "range_bn_fwd", "range_bn_bwd", "gossip_mix", "gossip_mix_ex", "gossip_set_sample_stride", "qconv_set_wgrad_beside", "MIX_PLAIN", "MIX_CHOCO", "MIX_DEEPSQUEEZE",
    "add", "maxpool_fwd", "maxpool_bwd", "avgpool_fwd", "avgpool_bwd", "softmax_xent", "sgd",
    "Workspace", "EXPORTS",
]

ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1
MIX_PLAIN, MIX_CHOCO, MIX_DEEPSQUEEZE = 0, 1, 2
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblpdt.so")

# every symbol include/lpdt.h declares
EXPORTS = [
    "lpdt_last_error", "lpdt_version",
    "lpdt_quantize_workspace_bytes", "lpdt_quantize", "lpdt_quantize_with_absmax",
    "lpdt_quantize_static_max_len", "lpdt_quantize_static",
    "lpdt_quantize_segments_workspace_bytes", "lpdt_quantize_segments", "lpdt_dequantize",
    "lpdt_qconv_fwd_workspace_bytes", "lpdt_qconv_bwd_data_workspace_bytes", "lpdt_qconv_bwd_weight_workspace_bytes",
    "lpdt_qconv_fwd", "lpdt_qconv_bwd_data", "lpdt_qconv_bwd_weight", "lpdt_qconv_kernel_id",
    "lpdt_qconv_fwd_f32_workspace_bytes", "lpdt_qconv_bwd_data_f32_workspace_bytes", "lpdt_qconv_bwd_weight_f32_workspace_bytes",
    "lpdt_qconv_fwd_f32", "lpdt_qconv_bwd_data_f32", "lpdt_qconv_bwd_weight_f32",
    "lpdt_qconv_fwd_f32_add_workspace_bytes", "lpdt_qconv_fwd_f32_add",
    "lpdt_qconv_ren_fwd_q_workspace_bytes", "lpdt_qconv_ren_fwd_q",
    "lpdt_to_bf16", "lpdt_qconv_bwd_weight_bf16_workspace_bytes", "lpdt_qconv_bwd_weight_bf16",
    "lpdt_range_evonorm_fwd_workspace_bytes", "lpdt_range_evonorm_bwd_workspace_bytes",
    "lpdt_range_evonorm_fwd", "lpdt_range_evonorm_bwd",
    "lpdt_range_evonorm_fwd_q_workspace_bytes", "lpdt_range_evonorm_fwd_q",
    "lpdt_range_evonorm_maxpool_fwd_workspace_bytes", "lpdt_range_evonorm_maxpool_bwd_workspace_bytes",
    "lpdt_range_evonorm_maxpool_fwd", "lpdt_range_evonorm_maxpool_bwd",
    "lpdt_qconv_bwd_data_packed_filter_bytes", "lpdt_qconv_bwd_data_pack_filter", "lpdt_qconv_bwd_data_pack_filters",
    "lpdt_qconv_bwd_data_f32_packed",
    "lpdt_qconv_fwd_f32_absmax_workspace_bytes", "lpdt_qconv_bwd_data_f32_absmax_workspace_bytes",
    "lpdt_qconv_fwd_f32_absmax", "lpdt_qconv_bwd_data_f32_absmax",
    "lpdt_evonorm_s0_fwd_workspace_bytes", "lpdt_evonorm_s0_bwd_workspace_bytes", "lpdt_evonorm_s0_fwd", "lpdt_evonorm_s0_bwd",
    "lpdt_range_bn_fwd_workspace_bytes", "lpdt_range_bn_bwd_workspace_bytes", "lpdt_range_bn_fwd", "lpdt_range_bn_bwd",
    "lpdt_gossip_mix_workspace_bytes", "lpdt_gossip_mix", "lpdt_gossip_set_sample_stride", "lpdt_gossip_mix_ex_workspace_bytes", "lpdt_gossip_mix_ex",
    "lpdt_add", "lpdt_maxpool_fwd", "lpdt_maxpool_bwd", "lpdt_avgpool_fwd", "lpdt_avgpool_bwd",
    "lpdt_softmax_xent", "lpdt_sgd", "lpdt_qconv_set_wgrad_beside",
]


class LpdtError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"lpdt error {code}: {message}")
        self.code = code


class ConvDesc(ctypes.Structure):
    """Mirror of lpdt_conv_desc."""
    _fields_ = [(k, ctypes.c_int) for k in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]

    @classmethod
    def make(cls, N, C, H, W, K, R, S, stride=1, pad=0):
        return cls(N, C, H, W, K, R, S, stride, stride, pad, pad)

    @property
    def P(self):
        return (self.H + 2 * self.pad_h - self.R) // self.stride_h + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad_w - self.S) // self.stride_w + 1


_lib = None
_sz = ctypes.c_size_t
_vp = ctypes.c_void_p


def library_path():
    return _LIB_PATH


def lib():
    """Loads liblpdt.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise LpdtError(-100, f"{_LIB_PATH} is missing: run `python -m paper_2111_09389_amd.build` "
                                  "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(_LIB_PATH)
        L.lpdt_last_error.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name.endswith("_workspace_bytes"):
                getattr(L, name).restype = _sz
        L.lpdt_quantize_workspace_bytes.argtypes = [_sz]
        L.lpdt_quantize_static_max_len.restype = _sz
        L.lpdt_quantize_segments_workspace_bytes.argtypes = [ctypes.c_int]
        for name in ("lpdt_qconv_fwd_workspace_bytes", "lpdt_qconv_bwd_data_workspace_bytes",
                     "lpdt_qconv_bwd_weight_workspace_bytes", "lpdt_qconv_fwd_f32_workspace_bytes",
                     "lpdt_qconv_bwd_data_f32_workspace_bytes", "lpdt_qconv_bwd_weight_f32_workspace_bytes",
                     "lpdt_qconv_bwd_weight_bf16_workspace_bytes", "lpdt_qconv_fwd_f32_add_workspace_bytes",
                     "lpdt_qconv_fwd_f32_absmax_workspace_bytes", "lpdt_qconv_bwd_data_f32_absmax_workspace_bytes"):
            getattr(L, name).argtypes = [ctypes.POINTER(ConvDesc)]
        for name in ("lpdt_range_evonorm_fwd_workspace_bytes", "lpdt_range_evonorm_bwd_workspace_bytes",
                     "lpdt_range_evonorm_fwd_q_workspace_bytes", "lpdt_range_evonorm_maxpool_fwd_workspace_bytes",
                     "lpdt_range_evonorm_maxpool_bwd_workspace_bytes", "lpdt_evonorm_s0_fwd_workspace_bytes", "lpdt_evonorm_s0_bwd_workspace_bytes"):
            getattr(L, name).argtypes = [ctypes.c_int] * 5
        L.lpdt_qconv_ren_fwd_q_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc), ctypes.c_int]
        L.lpdt_qconv_bwd_data_packed_filter_bytes.restype = _sz
        L.lpdt_qconv_bwd_data_packed_filter_bytes.argtypes = [ctypes.POINTER(ConvDesc)]
        for name in ("lpdt_range_bn_fwd_workspace_bytes", "lpdt_range_bn_bwd_workspace_bytes"):
            getattr(L, name).argtypes = [ctypes.c_int] * 4
        L.lpdt_gossip_mix_workspace_bytes.argtypes = [ctypes.c_int, _sz, ctypes.c_int, ctypes.c_int]
        L.lpdt_gossip_mix_ex_workspace_bytes.argtypes = [ctypes.c_int, _sz, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise LpdtError(rc, lib().lpdt_last_error().decode())


def _ptr(t):
    return _vp(0) if t is None else _vp(t.data_ptr())


def _stream():
    return _vp(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise LpdtError(-1, f"{what}: expected a contiguous CUDA tensor of dtype {dtype}")
    return t


class Workspace:
    """A caller-owned scratch buffer that grows on demand (allocation happens here, in Python,
    never inside the library)."""

    def __init__(self, device="cuda"):
        self.device = device
        self.buf = None

    def get(self, nbytes):
        if nbytes == 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=self.device)
        off = (-self.buf.data_ptr()) % 256
        return self.buf[off:], self.buf.numel() - off


_default_ws = None


def _ws(ws, nbytes):
    global _default_ws
    if ws is None:
        if _default_ws is None:
            _default_ws = Workspace()
        ws = _default_ws
    return ws.get(nbytes)


# ---------------------------------------------------------------- quantizer
def quantize(x, rounding=ROUND_NEAREST, seed=0, offset=0, q=None, scale=None, ws=None):
    """x fp32 -> (int8 codes of x's shape, fp32 device scalar scale)."""
    _dev(x, torch.float32, "quantize x")
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device) if q is None else q
    scale = torch.empty(1, dtype=torch.float32, device=x.device) if scale is None else scale
    n = x.numel()
    buf, nb = _ws(ws, lib().lpdt_quantize_workspace_bytes(n))
    _check(lib().lpdt_quantize(_ptr(x), _sz(n), int(rounding), ctypes.c_uint64(seed), ctypes.c_uint64(offset),
                               _ptr(q), _ptr(scale), _ptr(buf), _sz(nb), _stream()))
    return q, scale


def quantize_static(x, rounding=ROUND_NEAREST, seed=0, offset=0, q=None, scale=None):
    """lpdt_quantize_static: the quantizer that takes no workspace (q and scale must be given by callers that may not allocate)."""
    _dev(x, torch.float32, "quantize x")
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device) if q is None else q
    scale = torch.empty(1, dtype=torch.float32, device=x.device) if scale is None else scale
    _check(lib().lpdt_quantize_static(_ptr(x), _sz(x.numel()), int(rounding), ctypes.c_uint64(seed), ctypes.c_uint64(offset),
                                      _ptr(q), _ptr(scale), _stream()))
    return q, scale


def quantize_with_absmax(x, absmax, rounding=ROUND_NEAREST, seed=0, offset=0, q=None, scale=None):
    _dev(x, torch.float32, "quantize x")
    _dev(absmax, torch.float32, "quantize absmax")
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device) if q is None else q
    scale = torch.empty(1, dtype=torch.float32, device=x.device) if scale is None else scale
    _check(lib().lpdt_quantize_with_absmax(_ptr(x), _sz(x.numel()), _ptr(absmax), int(rounding), ctypes.c_uint64(seed),
                                           ctypes.c_uint64(offset), _ptr(q), _ptr(scale), _stream()))
    return q, scale


def quantize_segments(x, seg_begin, seg_end, rounding=ROUND_NEAREST, seed=0, offset=0, q=None, scales=None, ws=None):
    """Slices x.flat[seg_begin[s]:seg_end[s]] of one fp32 buffer, each with its own scale -> (int8 codes laid out like x,
    fp32 scales[nseg])."""
    _dev(x, torch.float32, "quantize_segments x")
    nseg = len(seg_begin)
    if len(seg_end) != nseg:
        raise ValueError("seg_begin and seg_end differ in length")
    q = torch.zeros(x.shape, dtype=torch.int8, device=x.device) if q is None else q
    scales = torch.empty(max(nseg, 1), dtype=torch.float32, device=x.device) if scales is None else scales
    b = (ctypes.c_int64 * max(nseg, 1))(*[int(v) for v in seg_begin])
    e = (ctypes.c_int64 * max(nseg, 1))(*[int(v) for v in seg_end])
    buf, nb = _ws(ws, lib().lpdt_quantize_segments_workspace_bytes(nseg))
    _check(lib().lpdt_quantize_segments(_ptr(x), b, e, nseg, int(rounding), ctypes.c_uint64(seed), ctypes.c_uint64(offset),
                                        _ptr(q), _ptr(scales), _ptr(buf), _sz(nb), _stream()))
    return q, scales


def dequantize(acc, sA, sB, y=None, accumulate=False):
    _dev(acc, torch.int32, "dequantize acc")
    y = torch.empty(acc.shape, dtype=torch.float32, device=acc.device) if y is None else y
    _check(lib().lpdt_dequantize(_ptr(acc), _sz(acc.numel()), _ptr(sA), _ptr(sB), _ptr(y), int(bool(accumulate)), _stream()))
    return y


# ---------------------------------------------------------------- convolutions
def qconv_kernel_id(d, product):
    """lpdt_qconv_kernel_id: which kernel / tile the product (0 forward, 1 backward-data, 2 backward-weight) takes."""
    rc = lib().lpdt_qconv_kernel_id(ctypes.byref(d), int(product))
    if rc < 0:
        _check(rc)
    return rc


def qconv_fwd(d, xq, wq, acc=None, ws=None):
    _dev(xq, torch.int8, "qconv_fwd xq"); _dev(wq, torch.int8, "qconv_fwd wq")
    assert tuple(xq.shape) == (d.N, d.H, d.W, d.C) and tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    acc = torch.empty((d.N, d.P, d.Q, d.K), dtype=torch.int32, device=xq.device) if acc is None else acc
    buf, nb = _ws(ws, lib().lpdt_qconv_fwd_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_fwd(ctypes.byref(d), _ptr(xq), _ptr(wq), _ptr(acc), _ptr(buf), _sz(nb), _stream()))
    return acc


def qconv_bwd_data(d, gq, wq, dx=None, ws=None):
    _dev(gq, torch.int8, "qconv_bwd_data gq"); _dev(wq, torch.int8, "qconv_bwd_data wq")
    assert tuple(gq.shape) == (d.N, d.P, d.Q, d.K) and tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    dx = torch.empty((d.N, d.H, d.W, d.C), dtype=torch.int32, device=gq.device) if dx is None else dx
    buf, nb = _ws(ws, lib().lpdt_qconv_bwd_data_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_bwd_data(ctypes.byref(d), _ptr(gq), _ptr(wq), _ptr(dx), _ptr(buf), _sz(nb), _stream()))
    return dx


def qconv_bwd_weight(d, gq, xq, dw=None, ws=None):
    _dev(gq, torch.int8, "qconv_bwd_weight gq"); _dev(xq, torch.int8, "qconv_bwd_weight xq")
    assert tuple(gq.shape) == (d.N, d.P, d.Q, d.K) and tuple(xq.shape) == (d.N, d.H, d.W, d.C)
    dw = torch.empty((d.K, d.R, d.S, d.C), dtype=torch.int32, device=gq.device) if dw is None else dw
    buf, nb = _ws(ws, lib().lpdt_qconv_bwd_weight_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_bwd_weight(ctypes.byref(d), _ptr(gq), _ptr(xq), _ptr(dw), _ptr(buf), _sz(nb), _stream()))
    return dw


def qconv_fwd_f32(d, xq, wq, sx, sw, y=None, ws=None):
    _dev(xq, torch.int8, "qconv_fwd_f32 xq"); _dev(wq, torch.int8, "qconv_fwd_f32 wq")
    assert tuple(xq.shape) == (d.N, d.H, d.W, d.C) and tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    y = torch.empty((d.N, d.P, d.Q, d.K), dtype=torch.float32, device=xq.device) if y is None else y
    buf, nb = _ws(ws, lib().lpdt_qconv_fwd_f32_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_fwd_f32(ctypes.byref(d), _ptr(xq), _ptr(wq), _ptr(sx), _ptr(sw), _ptr(y), _ptr(buf), _sz(nb), _stream()))
    return y


def qconv_fwd_f32_add(d, xq, wq, sx, sw, y, ws=None):
    """y += sx*sw*conv(xq, wq), in place (the skip connection's addition in the convolution's epilogue)."""
    _dev(xq, torch.int8, "qconv_fwd_f32_add xq"); _dev(wq, torch.int8, "qconv_fwd_f32_add wq"); _dev(y, torch.float32, "qconv_fwd_f32_add y")
    assert tuple(xq.shape) == (d.N, d.H, d.W, d.C) and tuple(wq.shape) == (d.K, d.R, d.S, d.C) and tuple(y.shape) == (d.N, d.P, d.Q, d.K)
    buf, nb = _ws(ws, lib().lpdt_qconv_fwd_f32_add_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_fwd_f32_add(ctypes.byref(d), _ptr(xq), _ptr(wq), _ptr(sx), _ptr(sw), _ptr(y), _ptr(buf), _sz(nb), _stream()))
    return y


def qconv_ren_fwd_q(d, xq, wq, sx, sw, groups, v, gamma, beta, eps=1e-5, y=None, accumulate=False, z=None, ws=None):
    """lpdt_qconv_ren_fwd_q: conv -> Range-EvoNorm -> quantizer in one call -> (y, q, scale, range, argmax, argmin);
    accumulate: y (given) += product before the normalisation."""
    _dev(xq, torch.int8, "qconv_ren_fwd_q xq"); _dev(wq, torch.int8, "qconv_ren_fwd_q wq")
    assert tuple(xq.shape) == (d.N, d.H, d.W, d.C) and tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    dev = xq.device
    if y is None:
        assert not accumulate
        y = torch.empty((d.N, d.P, d.Q, d.K), dtype=torch.float32, device=dev)
    q = torch.empty((d.N, d.P, d.Q, d.K), dtype=torch.int8, device=dev)
    scale = torch.empty(1, dtype=torch.float32, device=dev)
    rng = torch.empty((d.N, groups), dtype=torch.float32, device=dev)
    amx = torch.empty((d.N, groups), dtype=torch.int32, device=dev)
    amn = torch.empty((d.N, groups), dtype=torch.int32, device=dev)
    buf, nb = _ws(ws, lib().lpdt_qconv_ren_fwd_q_workspace_bytes(ctypes.byref(d), int(groups)))
    _check(lib().lpdt_qconv_ren_fwd_q(ctypes.byref(d), _ptr(xq), _ptr(wq), _ptr(sx), _ptr(sw), int(bool(accumulate)), int(groups), _ptr(v),
                                      _ptr(gamma), _ptr(beta), ctypes.c_float(eps), _ptr(y), _ptr(z), _ptr(q), _ptr(scale), _ptr(rng), _ptr(amx),
                                      _ptr(amn), _ptr(buf), _sz(nb), _stream()))
    return y, q, scale, rng, amx, amn


def qconv_bwd_data_f32(d, gq, wq, sg, sw, dx=None, accumulate=False, ws=None):
    _dev(gq, torch.int8, "qconv_bwd_data_f32 gq"); _dev(wq, torch.int8, "qconv_bwd_data_f32 wq")
    assert tuple(gq.shape) == (d.N, d.P, d.Q, d.K) and tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    dx = torch.empty((d.N, d.H, d.W, d.C), dtype=torch.float32, device=gq.device) if dx is None else dx
    buf, nb = _ws(ws, lib().lpdt_qconv_bwd_data_f32_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_bwd_data_f32(ctypes.byref(d), _ptr(gq), _ptr(wq), _ptr(sg), _ptr(sw), _ptr(dx), int(bool(accumulate)),
                                         _ptr(buf), _sz(nb), _stream()))
    return dx


def qconv_fwd_f32_absmax(d, xq, wq, sx, sw, y=None, ws=None):
    """-> (y, absmax): lpdt_qconv_fwd_f32 plus max|y| as a device scalar."""
    _dev(xq, torch.int8, "qconv_fwd_f32_absmax xq"); _dev(wq, torch.int8, "qconv_fwd_f32_absmax wq")
    assert tuple(xq.shape) == (d.N, d.H, d.W, d.C) and tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    y = torch.empty((d.N, d.P, d.Q, d.K), dtype=torch.float32, device=xq.device) if y is None else y
    absmax = torch.empty(1, dtype=torch.float32, device=xq.device)
    buf, nb = _ws(ws, lib().lpdt_qconv_fwd_f32_absmax_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_fwd_f32_absmax(ctypes.byref(d), _ptr(xq), _ptr(wq), _ptr(sx), _ptr(sw), _ptr(y), _ptr(absmax), _ptr(buf),
                                           _sz(nb), _stream()))
    return y, absmax


def qconv_bwd_data_f32_absmax(d, gq, wq, sg, sw, packed=None, dx=None, accumulate=False, ws=None):
    """-> (dx, absmax): lpdt_qconv_bwd_data_f32 (filter as wq or packed) plus max|dx| as a device scalar."""
    _dev(gq, torch.int8, "qconv_bwd_data_f32_absmax gq")
    assert tuple(gq.shape) == (d.N, d.P, d.Q, d.K)
    dx = torch.empty((d.N, d.H, d.W, d.C), dtype=torch.float32, device=gq.device) if dx is None else dx
    absmax = torch.empty(1, dtype=torch.float32, device=gq.device)
    buf, nb = _ws(ws, lib().lpdt_qconv_bwd_data_f32_absmax_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_bwd_data_f32_absmax(ctypes.byref(d), _ptr(gq), _ptr(wq), _ptr(packed), _ptr(sg), _ptr(sw), _ptr(dx),
                                                int(bool(accumulate)), _ptr(absmax), _ptr(buf), _sz(nb), _stream()))
    return dx, absmax


def qconv_set_wgrad_beside(beside):
    """Size the backward-weight launches for running beside other kernels (True) or alone (False, the default)."""
    _check(lib().lpdt_qconv_set_wgrad_beside(int(bool(beside))))


def qconv_bwd_data_pack_filter(d, wq):
    """The filter as backward-data reads it (transposed panels), for qconv_bwd_data_f32_packed; None when the shape has no
    prepared form."""
    _dev(wq, torch.int8, "qconv_bwd_data_pack_filter wq")
    assert tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    nb = int(lib().lpdt_qconv_bwd_data_packed_filter_bytes(ctypes.byref(d)))
    if nb == 0:
        return None
    packed = torch.empty(nb, dtype=torch.uint8, device=wq.device)
    _check(lib().lpdt_qconv_bwd_data_pack_filter(ctypes.byref(d), _ptr(wq), _ptr(packed), _sz(nb), _stream()))
    return packed


def qconv_bwd_data_pack_filters(descs, wqs):
    """qconv_bwd_data_pack_filter for several filters in one launch; every shape must have a prepared form."""
    n = len(descs)
    assert n == len(wqs)
    for d, wq in zip(descs, wqs):
        _dev(wq, torch.int8, "qconv_bwd_data_pack_filters wq")
        assert tuple(wq.shape) == (d.K, d.R, d.S, d.C)
    darr = (ConvDesc * n)(*descs)
    sizes = [int(lib().lpdt_qconv_bwd_data_packed_filter_bytes(ctypes.byref(darr[i]))) for i in range(n)]
    packed = [torch.empty(max(nb, 16), dtype=torch.uint8, device=wq.device) for nb, wq in zip(sizes, wqs)]
    _check(lib().lpdt_qconv_bwd_data_pack_filters(darr, n, (ctypes.c_void_p * n)(*[w.data_ptr() for w in wqs]),
                                                  (ctypes.c_void_p * n)(*[t.data_ptr() for t in packed]),
                                                  (_sz * n)(*sizes), _stream()))
    return packed


def qconv_bwd_data_f32_packed(d, gq, packed, sg, sw, dx=None, accumulate=False, ws=None):
    _dev(gq, torch.int8, "qconv_bwd_data_f32_packed gq")
    assert tuple(gq.shape) == (d.N, d.P, d.Q, d.K)
    dx = torch.empty((d.N, d.H, d.W, d.C), dtype=torch.float32, device=gq.device) if dx is None else dx
    buf, nb = _ws(ws, lib().lpdt_qconv_bwd_data_f32_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_bwd_data_f32_packed(ctypes.byref(d), _ptr(gq), _ptr(packed), _ptr(sg), _ptr(sw), _ptr(dx),
                                                int(bool(accumulate)), _ptr(buf), _sz(nb), _stream()))
    return dx


def qconv_bwd_weight_f32(d, gq, xq, sg, sx, dw=None, ws=None):
    _dev(gq, torch.int8, "qconv_bwd_weight_f32 gq"); _dev(xq, torch.int8, "qconv_bwd_weight_f32 xq")
    assert tuple(gq.shape) == (d.N, d.P, d.Q, d.K) and tuple(xq.shape) == (d.N, d.H, d.W, d.C)
    dw = torch.empty((d.K, d.R, d.S, d.C), dtype=torch.float32, device=gq.device) if dw is None else dw
    buf, nb = _ws(ws, lib().lpdt_qconv_bwd_weight_f32_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_bwd_weight_f32(ctypes.byref(d), _ptr(gq), _ptr(xq), _ptr(sg), _ptr(sx), _ptr(dw), _ptr(buf), _sz(nb),
                                           _stream()))
    return dw


# ---------------------------------------------------------------- Range-EvoNorm
def range_evonorm_fwd(x, groups, v, gamma, beta, eps=1e-5, y=None, want_absmax=False, ws=None):
    """-> (y, range [N,groups], argmax, argmin[, absmax])."""
    _dev(x, torch.float32, "range_evonorm_fwd x")
    N, H, W, C = x.shape
    dev = x.device
    y = torch.empty_like(x) if y is None else y
    rng = torch.empty((N, groups), dtype=torch.float32, device=dev)
    amx = torch.empty((N, groups), dtype=torch.int32, device=dev)
    amn = torch.empty((N, groups), dtype=torch.int32, device=dev)
    absmax = torch.empty(1, dtype=torch.float32, device=dev) if want_absmax else None
    buf, nb = _ws(ws, lib().lpdt_range_evonorm_fwd_workspace_bytes(N, H, W, C, groups))
    _check(lib().lpdt_range_evonorm_fwd(_ptr(x), N, H, W, C, int(groups), _ptr(v), _ptr(gamma), _ptr(beta),
                                        ctypes.c_float(eps), _ptr(y), _ptr(rng), _ptr(amx), _ptr(amn), _ptr(absmax),
                                        _ptr(buf), _sz(nb), _stream()))
    return (y, rng, amx, amn, absmax) if want_absmax else (y, rng, amx, amn)


def range_evonorm_fwd_q(x, groups, v, gamma, beta, eps=1e-5, q=None, y=None, ws=None):
    """Range-EvoNorm forward with int8 output -> (q int8, scale [1], range [N,groups], argmax, argmin); y: optional fp32
    tensor that also receives the unquantized output."""
    _dev(x, torch.float32, "range_evonorm_fwd_q x")
    N, H, W, C = x.shape
    dev = x.device
    q = torch.empty(x.shape, dtype=torch.int8, device=dev) if q is None else q
    scale = torch.empty(1, dtype=torch.float32, device=dev)
    rng = torch.empty((N, groups), dtype=torch.float32, device=dev)
    amx = torch.empty((N, groups), dtype=torch.int32, device=dev)
    amn = torch.empty((N, groups), dtype=torch.int32, device=dev)
    buf, nb = _ws(ws, lib().lpdt_range_evonorm_fwd_q_workspace_bytes(N, H, W, C, int(groups)))
    _check(lib().lpdt_range_evonorm_fwd_q(_ptr(x), N, H, W, C, int(groups), _ptr(v), _ptr(gamma), _ptr(beta), ctypes.c_float(eps),
                                          _ptr(q), _ptr(scale), _ptr(y), _ptr(rng), _ptr(amx), _ptr(amn), _ptr(buf), _sz(nb), _stream()))
    return q, scale, rng, amx, amn


def range_evonorm_maxpool_fwd(x, groups, v, gamma, beta, k, stride, pad, eps=1e-5, want_absmax=False, ws=None):
    """maxpool(range_evonorm(x)) without storing the normalised tensor -> (z, idx, range, argmax, argmin[, absmax])."""
    _dev(x, torch.float32, "range_evonorm_maxpool_fwd x")
    N, H, W, C = x.shape
    dev = x.device
    P, Q = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    z = torch.empty((N, P, Q, C), dtype=torch.float32, device=dev)
    idx = torch.empty((N, P, Q, C), dtype=torch.int32, device=dev)
    rng = torch.empty((N, groups), dtype=torch.float32, device=dev)
    amx = torch.empty((N, groups), dtype=torch.int32, device=dev)
    amn = torch.empty((N, groups), dtype=torch.int32, device=dev)
    absmax = torch.empty(1, dtype=torch.float32, device=dev) if want_absmax else None
    buf, nb = _ws(ws, lib().lpdt_range_evonorm_maxpool_fwd_workspace_bytes(N, H, W, C, int(groups)))
    _check(lib().lpdt_range_evonorm_maxpool_fwd(_ptr(x), N, H, W, C, int(groups), _ptr(v), _ptr(gamma), _ptr(beta),
                                                ctypes.c_float(eps), int(k), int(stride), int(pad), _ptr(z), _ptr(idx), _ptr(rng),
                                                _ptr(amx), _ptr(amn), _ptr(absmax), _ptr(buf), _sz(nb), _stream()))
    return (z, idx, rng, amx, amn, absmax) if want_absmax else (z, idx, rng, amx, amn)


def range_evonorm_maxpool_bwd(dz, idx, x, groups, v, gamma, rng, amx, amn, k, stride, pad, eps=1e-5, want_absmax=False, ws=None):
    """Backward of range_evonorm_maxpool_fwd -> (dx, dv, dgamma, dbeta[, absmax])."""
    _dev(x, torch.float32, "range_evonorm_maxpool_bwd x"); _dev(dz, torch.float32, "range_evonorm_maxpool_bwd dz")
    _dev(idx, torch.int32, "range_evonorm_maxpool_bwd idx")
    N, H, W, C = x.shape
    dev = x.device
    dx = torch.empty_like(x)
    dv, dg, db = (torch.empty(C, dtype=torch.float32, device=dev) for _ in range(3))
    absmax = torch.empty(1, dtype=torch.float32, device=dev) if want_absmax else None
    buf, nb = _ws(ws, lib().lpdt_range_evonorm_maxpool_bwd_workspace_bytes(N, H, W, C, int(groups)))
    _check(lib().lpdt_range_evonorm_maxpool_bwd(_ptr(dz), _ptr(idx), _ptr(x), N, H, W, C, int(groups), _ptr(v), _ptr(gamma),
                                                ctypes.c_float(eps), int(k), int(stride), int(pad), _ptr(rng), _ptr(amx), _ptr(amn),
                                                _ptr(dx), _ptr(dv), _ptr(dg), _ptr(db), _ptr(absmax), _ptr(buf), _sz(nb), _stream()))
    return (dx, dv, dg, db, absmax) if want_absmax else (dx, dv, dg, db)


def range_evonorm_bwd(dy, x, groups, v, gamma, rng, amx, amn, eps=1e-5, dx=None, want_absmax=False, ws=None):
    """-> (dx, dv, dgamma, dbeta[, absmax])."""
    _dev(x, torch.float32, "range_evonorm_bwd x"); _dev(dy, torch.float32, "range_evonorm_bwd dy")
    N, H, W, C = x.shape
    dev = x.device
    dx = torch.empty_like(x) if dx is None else dx
    dv, dg, db = (torch.empty(C, dtype=torch.float32, device=dev) for _ in range(3))
    absmax = torch.empty(1, dtype=torch.float32, device=dev) if want_absmax else None
    buf, nb = _ws(ws, lib().lpdt_range_evonorm_bwd_workspace_bytes(N, H, W, C, groups))
    _check(lib().lpdt_range_evonorm_bwd(_ptr(dy), _ptr(x), N, H, W, C, int(groups), _ptr(v), _ptr(gamma),
                                        ctypes.c_float(eps), _ptr(rng), _ptr(amx), _ptr(amn), _ptr(dx), _ptr(dv), _ptr(dg),
                                        _ptr(db), _ptr(absmax), _ptr(buf), _sz(nb), _stream()))
    return (dx, dv, dg, db, absmax) if want_absmax else (dx, dv, dg, db)


# ---------------------------------------------------------------- full-precision comparison layers
def evonorm_s0_fwd(x, groups, v, gamma, beta, eps=1e-5, y=None, ws=None):
    """EvoNorm-S0 -> (y, mean [N,groups], var [N,groups])."""
    _dev(x, torch.float32, "evonorm_s0_fwd x")
    N, H, W, C = x.shape
    y = torch.empty_like(x) if y is None else y
    mean = torch.empty((N, groups), dtype=torch.float32, device=x.device)
    var = torch.empty((N, groups), dtype=torch.float32, device=x.device)
    buf, nb = _ws(ws, lib().lpdt_evonorm_s0_fwd_workspace_bytes(N, H, W, C, int(groups)))
    _check(lib().lpdt_evonorm_s0_fwd(_ptr(x), N, H, W, C, int(groups), _ptr(v), _ptr(gamma), _ptr(beta), ctypes.c_float(eps),
                                     _ptr(y), _ptr(mean), _ptr(var), _ptr(buf), _sz(nb), _stream()))
    return y, mean, var


def evonorm_s0_bwd(dy, x, groups, v, gamma, mean, var, eps=1e-5, dx=None, ws=None):
    """-> (dx, dv, dgamma, dbeta)."""
    _dev(x, torch.float32, "evonorm_s0_bwd x"); _dev(dy, torch.float32, "evonorm_s0_bwd dy")
    N, H, W, C = x.shape
    dx = torch.empty_like(x) if dx is None else dx
    dv, dg, db = (torch.empty(C, dtype=torch.float32, device=x.device) for _ in range(3))
    buf, nb = _ws(ws, lib().lpdt_evonorm_s0_bwd_workspace_bytes(N, H, W, C, int(groups)))
    _check(lib().lpdt_evonorm_s0_bwd(_ptr(dy), _ptr(x), N, H, W, C, int(groups), _ptr(v), _ptr(gamma), ctypes.c_float(eps),
                                     _ptr(mean), _ptr(var), _ptr(dx), _ptr(dv), _ptr(dg), _ptr(db), _ptr(buf), _sz(nb), _stream()))
    return dx, dv, dg, db


def range_bn_fwd(x, gamma, beta, eps=1e-5, y=None, ws=None):
    """Range batch-norm -> (y, mean [C], range [C], argmax int64 [C], argmin int64 [C])."""
    _dev(x, torch.float32, "range_bn_fwd x")
    N, H, W, C = x.shape
    y = torch.empty_like(x) if y is None else y
    mean = torch.empty(C, dtype=torch.float32, device=x.device)
    rng = torch.empty(C, dtype=torch.float32, device=x.device)
    amx = torch.empty(C, dtype=torch.int64, device=x.device)
    amn = torch.empty(C, dtype=torch.int64, device=x.device)
    buf, nb = _ws(ws, lib().lpdt_range_bn_fwd_workspace_bytes(N, H, W, C))
    _check(lib().lpdt_range_bn_fwd(_ptr(x), N, H, W, C, _ptr(gamma), _ptr(beta), ctypes.c_float(eps), _ptr(y), _ptr(mean),
                                   _ptr(rng), _ptr(amx), _ptr(amn), _ptr(buf), _sz(nb), _stream()))
    return y, mean, rng, amx, amn


def range_bn_bwd(dy, x, gamma, mean, rng, amx, amn, eps=1e-5, dx=None, ws=None):
    """-> (dx, dgamma, dbeta)."""
    _dev(x, torch.float32, "range_bn_bwd x"); _dev(dy, torch.float32, "range_bn_bwd dy")
    N, H, W, C = x.shape
    dx = torch.empty_like(x) if dx is None else dx
    dg, db = (torch.empty(C, dtype=torch.float32, device=x.device) for _ in range(2))
    buf, nb = _ws(ws, lib().lpdt_range_bn_bwd_workspace_bytes(N, H, W, C))
    _check(lib().lpdt_range_bn_bwd(_ptr(dy), _ptr(x), N, H, W, C, _ptr(gamma), ctypes.c_float(eps), _ptr(mean), _ptr(rng),
                                   _ptr(amx), _ptr(amn), _ptr(dx), _ptr(dg), _ptr(db), _ptr(buf), _sz(nb), _stream()))
    return dx, dg, db


# ---------------------------------------------------------------- gossip
def gossip_set_sample_stride(stride):
    """lpdt_gossip_set_sample_stride: -1 automatic, 0 two-pass selection, s > 0 one pass with every s-th tile sampled."""
    _check(lib().lpdt_gossip_set_sample_stride(int(stride)))


def gossip_mix(x, xhat, W, rate=1.0, keep_ratio=1.0, seg_offsets=None, ws=None):
    """In-place gossip step on x [n,d] (and xhat for CHOCO).  W: host matrix (numpy / nested list / CPU tensor)."""
    _dev(x, torch.float32, "gossip_mix x")
    n, d = x.shape
    if xhat is not None:
        _dev(xhat, torch.float32, "gossip_mix xhat")
        assert tuple(xhat.shape) == (n, d)
    Wh = torch.as_tensor(W, dtype=torch.float32, device="cpu").contiguous()
    assert tuple(Wh.shape) == (n, n)
    Wc = (ctypes.c_float * (n * n)).from_buffer_copy(Wh.numpy().tobytes())
    if seg_offsets is None:
        seg, nseg = None, 0
    else:
        so = [int(v) for v in seg_offsets]
        seg, nseg = (ctypes.c_int64 * len(so))(*so), len(so) - 1
    buf, nb = _ws(ws, lib().lpdt_gossip_mix_workspace_bytes(n, _sz(d), nseg, int(xhat is not None)))
    _check(lib().lpdt_gossip_mix(_ptr(x), _ptr(xhat), n, _sz(d), Wc, ctypes.c_float(rate), ctypes.c_double(keep_ratio),
                                 seg, nseg, _ptr(buf), _sz(nb), _stream()))
    return x, xhat


def gossip_mix_ex(x, state, W, rate=1.0, keep_ratio=1.0, seg_offsets=None, mode=MIX_PLAIN, u=None, z=None, ws=None):
    """In-place gossip step of the supplement's variants: state = xhat (MIX_CHOCO) / delta (MIX_DEEPSQUEEZE) / None;
    u: device fp32 [n] push-sum weights or None; z: device fp32 [n,d] receiving x/u, or None."""
    _dev(x, torch.float32, "gossip_mix_ex x")
    n, d = x.shape
    for t, what in ((state, "state"), (z, "z")):
        if t is not None:
            _dev(t, torch.float32, "gossip_mix_ex " + what)
            assert tuple(t.shape) == (n, d)
    if u is not None:
        _dev(u, torch.float32, "gossip_mix_ex u")
        assert u.numel() == n
    Wh = torch.as_tensor(W, dtype=torch.float32, device="cpu").contiguous()
    assert tuple(Wh.shape) == (n, n)
    Wc = (ctypes.c_float * (n * n)).from_buffer_copy(Wh.numpy().tobytes())
    if seg_offsets is None:
        seg, nseg = None, 0
    else:
        so = [int(v) for v in seg_offsets]
        seg, nseg = (ctypes.c_int64 * len(so))(*so), len(so) - 1
    buf, nb = _ws(ws, lib().lpdt_gossip_mix_ex_workspace_bytes(n, _sz(d), nseg, int(mode), int(u is not None)))
    _check(lib().lpdt_gossip_mix_ex(_ptr(x), _ptr(state), n, _sz(d), Wc, ctypes.c_float(rate), ctypes.c_double(keep_ratio),
                                    seg, nseg, int(mode), _ptr(u), _ptr(z), _ptr(buf), _sz(nb), _stream()))
    return x, state, u, z


def to_bf16(x, y=None):
    """fp32 tensor -> bfloat16 bit patterns (int16 tensor of the same shape), round to nearest even."""
    _dev(x, torch.float32, "to_bf16 x")
    y = torch.empty(x.shape, dtype=torch.int16, device=x.device) if y is None else y
    _check(lib().lpdt_to_bf16(_ptr(x), _sz(x.numel()), _ptr(y), _stream()))
    return y


def qconv_bwd_weight_bf16(d, g16, xq, sx, dw=None, ws=None):
    """Weight gradient from the bfloat16 copy of the layer gradient (int16 bit patterns [N,P,Q,K]) and int8 input codes."""
    _dev(g16, torch.int16, "qconv_bwd_weight_bf16 g16"); _dev(xq, torch.int8, "qconv_bwd_weight_bf16 xq")
    assert tuple(g16.shape) == (d.N, d.P, d.Q, d.K) and tuple(xq.shape) == (d.N, d.H, d.W, d.C)
    dw = torch.empty((d.K, d.R, d.S, d.C), dtype=torch.float32, device=xq.device) if dw is None else dw
    buf, nb = _ws(ws, lib().lpdt_qconv_bwd_weight_bf16_workspace_bytes(ctypes.byref(d)))
    _check(lib().lpdt_qconv_bwd_weight_bf16(ctypes.byref(d), _ptr(g16), _ptr(xq), _ptr(sx), _ptr(dw), _ptr(buf), _sz(nb), _stream()))
    return dw


# ---------------------------------------------------------------- glue
def add(a, b, y=None):
    _dev(a, torch.float32, "add a"); _dev(b, torch.float32, "add b")
    y = torch.empty_like(a) if y is None else y
    _check(lib().lpdt_add(_ptr(a), _ptr(b), _sz(a.numel()), _ptr(y), _stream()))
    return y


def maxpool_fwd(x, k, stride, pad):
    _dev(x, torch.float32, "maxpool_fwd x")
    N, H, W, C = x.shape
    P, Q = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = torch.empty((N, P, Q, C), dtype=torch.float32, device=x.device)
    idx = torch.empty((N, P, Q, C), dtype=torch.int32, device=x.device)
    _check(lib().lpdt_maxpool_fwd(_ptr(x), N, H, W, C, k, stride, pad, _ptr(y), _ptr(idx), _stream()))
    return y, idx


def maxpool_bwd(dy, idx, in_shape, k, stride, pad):
    _dev(dy, torch.float32, "maxpool_bwd dy"); _dev(idx, torch.int32, "maxpool_bwd idx")
    N, H, W, C = in_shape
    dx = torch.empty(in_shape, dtype=torch.float32, device=dy.device)
    _check(lib().lpdt_maxpool_bwd(_ptr(dy), _ptr(idx), N, H, W, C, k, stride, pad, _ptr(dx), _stream()))
    return dx


def avgpool_fwd(x):
    _dev(x, torch.float32, "avgpool_fwd x")
    N, H, W, C = x.shape
    y = torch.empty((N, C), dtype=torch.float32, device=x.device)
    _check(lib().lpdt_avgpool_fwd(_ptr(x), N, H * W, C, _ptr(y), _stream()))
    return y


def avgpool_bwd(dy, in_shape):
    _dev(dy, torch.float32, "avgpool_bwd dy")
    N, H, W, C = in_shape
    dx = torch.empty(in_shape, dtype=torch.float32, device=dy.device)
    _check(lib().lpdt_avgpool_bwd(_ptr(dy), N, H * W, C, _ptr(dx), _stream()))
    return dx


def softmax_xent(logits, labels):
    """-> (loss buffer [1+N]: mean loss then per-sample losses, dlogits)."""
    _dev(logits, torch.float32, "softmax_xent logits"); _dev(labels, torch.int32, "softmax_xent labels")
    N, classes = logits.shape
    loss = torch.empty(1 + N, dtype=torch.float32, device=logits.device)
    dl = torch.empty_like(logits)
    _check(lib().lpdt_softmax_xent(_ptr(logits), _ptr(labels), N, classes, _ptr(loss), _ptr(dl), _stream()))
    return loss, dl


def sgd(x, g, lr):
    _dev(x, torch.float32, "sgd x"); _dev(g, torch.float32, "sgd g")
    _check(lib().lpdt_sgd(_ptr(x), _ptr(g), _sz(x.numel()), ctypes.c_float(lr), _stream()))
    return x
