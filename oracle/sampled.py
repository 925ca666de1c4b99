"""Single outputs of the three convolution sums and the top-k selection rule, written out in numpy.

Test infrastructure only, like the rest of this package: at the benchmark's full sizes the C oracle's seven nested
loops take minutes, so the parity tests there compare sampled outputs, each computed here straight from the
definitions (Section 3, "Low Precision Training": the three int8 products with exact accumulation; supplement,
Algorithm "CHOCO-SGD" with the top-k rule of this build: larger |v| first by fp32 bit pattern, lower index on ties).
"""
import numpy as np


def qconv_fwd_at(x, w, stride, pad, coords):
    """x int8 [N,H,W,C], w int8 [K,R,S,C]; coords: iterable of (n, p, q, k) -> int64 sums acc[n,p,q,k]."""
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    out = []
    for n, p, q, k in coords:
        s = 0
        for r in range(R):
            h = p * stride + r - pad
            if h < 0 or h >= H:
                continue
            for t in range(S):
                ww = q * stride + t - pad
                if ww < 0 or ww >= W:
                    continue
                s += int(np.dot(x[n, h, ww].astype(np.int64), w[k, r, t].astype(np.int64)))
        out.append(s)
    return np.array(out, np.int64)


def qconv_bwd_data_at(g, w, H, W, stride, pad, coords):
    """g int8 [N,P,Q,K], w int8 [K,R,S,C]; coords: (n, h, w, c) -> int64 sums dx[n,h,w,c]."""
    N, P, Q, K = g.shape
    _, R, S, C = w.shape
    out = []
    for n, h, ww, c in coords:
        s = 0
        for r in range(R):
            ty = h + pad - r
            if ty < 0 or ty % stride or ty // stride >= P:
                continue
            for t in range(S):
                tx = ww + pad - t
                if tx < 0 or tx % stride or tx // stride >= Q:
                    continue
                s += int(np.dot(g[n, ty // stride, tx // stride].astype(np.int64), w[:, r, t, c].astype(np.int64)))
        out.append(s)
    return np.array(out, np.int64)


def qconv_bwd_weight_at(g, x, R, S, stride, pad, coords):
    """g int8 [N,P,Q,K], x int8 [N,H,W,C]; coords: (k, r, s, c) -> int64 sums dw[k,r,s,c] over all output pixels."""
    N, P, Q, K = g.shape
    _, H, W, C = x.shape
    out = []
    for k, r, t, c in coords:
        ps = np.arange(P)
        qs = np.arange(Q)
        hs, ws = ps * stride + r - pad, qs * stride + t - pad
        pv, qv = ps[(hs >= 0) & (hs < H)], qs[(ws >= 0) & (ws < W)]
        gg = g[:, pv][:, :, qv, k].astype(np.int64)
        xx = x[:, pv * stride + r - pad][:, :, qv * stride + t - pad, c].astype(np.int64)
        out.append(int((gg * xx).sum()))
    return np.array(out, np.int64)


def topk_mask(v, k):
    """Boolean mask of the k entries of the fp32 vector v that the top-k rule keeps: order by (|v| as fp32 bit
    pattern, descending; index, ascending).  One 64-bit key per element makes the order total, so the set is unique."""
    v = np.ascontiguousarray(v, np.float32)
    mag = (v.view(np.uint32) & np.uint32(0x7FFFFFFF)).astype(np.uint64)
    keys = (mag << np.uint64(32)) | (np.uint64(0xFFFFFFFF) - np.arange(v.size, dtype=np.uint64))
    if k >= v.size:
        return np.ones(v.size, bool)
    thr = np.partition(keys, v.size - k)[v.size - k]
    return keys >= thr
