"""Seeded synthetic inputs and network shape tables shared by the tests, the
benchmark and the smoke check.

This module holds NO arithmetic of the method: it only draws random tensors
(numpy PCG64, fixed seeds) with the shapes and distributions of the paper's
workloads (Section 4: 32x32x3 CIFAR-10-shaped and 224x224x3 Imagenette-shaped
normalised images, 10 / 100 classes) and lists layer shapes.  Both the GPU
path and the CPU oracle are fed from here; neither imports the other.
"""
import numpy as np

BASE_SEED = 20211109
PHILOX_SEED = 0x211109389


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def conv_out(size, pad, filt, stride):
    return (size + 2 * pad - filt) // stride + 1


def images(seed, N, H, W, C=3):
    """Normalised images ~N(0,1), fp32, NHWC."""
    return rng(seed).standard_normal((N, H, W, C), dtype=np.float32)


def kaiming_filter(seed, K, R, S, C):
    """Kaiming-normal filter, std = sqrt(2 / (C*R*S)), fp32, KRSC."""
    std = np.sqrt(2.0 / (C * R * S))
    return (rng(seed).standard_normal((K, R, S, C), dtype=np.float32) * np.float32(std)).astype(np.float32)


def upstream_grad(seed, shape, var=1e-2):
    """Upstream error signal ~N(0, var), fp32."""
    return (rng(seed).standard_normal(shape, dtype=np.float32) * np.float32(np.sqrt(var))).astype(np.float32)


def int8_codes(seed, shape, kind="gauss"):
    """int8 codes in [-127,127]: 'gauss' looks like a quantised N(0,1) tensor whose abs-max maps
    to 127 (most codes small), 'uniform' spreads over the whole grid, 'extreme' is all +-127."""
    g = rng(seed)
    if kind == "uniform":
        return g.integers(-127, 128, size=shape, dtype=np.int64).astype(np.int8)
    if kind == "extreme":
        return (g.integers(0, 2, size=shape, dtype=np.int64) * 254 - 127).astype(np.int8)
    x = g.standard_normal(shape)
    return np.clip(np.rint(x * (127.0 / 4.5)), -127, 127).astype(np.int8)


def labels_uniform(seed, N, classes):
    return rng(seed).integers(0, classes, size=N, dtype=np.int64).astype(np.int32)


def labels_dirichlet(seed, N, classes, alpha=0.1):
    """Per-agent label skew: class probabilities ~ Dirichlet(alpha), then N labels drawn from them."""
    g = rng(seed)
    p = g.dirichlet(np.full(classes, alpha))
    return g.choice(classes, size=N, p=p).astype(np.int32)


def ring_matrix(n, self_w=1.0 / 3.0):
    """Undirected ring: weight self_w on the node itself, the rest split over its two neighbours
    (symmetric, doubly stochastic).  W[i, j] = weight node i gives node j's model."""
    Wm = np.zeros((n, n), np.float32)
    side = (1.0 - self_w) / 2.0
    for i in range(n):
        Wm[i, i] += self_w
        Wm[i, (i + 1) % n] += side
        Wm[i, (i - 1) % n] += side
    return Wm


def torus_matrix(rows, cols):
    """Undirected 2-D torus, uniform weight 1/5 on self and the four neighbours."""
    n = rows * cols
    Wm = np.zeros((n, n), np.float32)
    for r in range(rows):
        for c in range(cols):
            i = r * cols + c
            for j in (i, ((r + 1) % rows) * cols + c, ((r - 1) % rows) * cols + c,
                      r * cols + (c + 1) % cols, r * cols + (c - 1) % cols):
                Wm[i, j] += 0.2
    return Wm


def directed_matrix(n):
    """A strongly connected directed graph for push-sum: node j sends to itself, to j+1 and, when j is even, to j+3
    (mod n), each with weight 1/out-degree(j).  Columns sum to 1, rows do not (in-degrees differ).
    W[i, j] = weight node i gives what it receives from node j."""
    Wm = np.zeros((n, n), np.float32)
    for j in range(n):
        outs = {j, (j + 1) % n} | ({(j + 3) % n} if j % 2 == 0 else set())
        for i in outs:
            Wm[i, j] = np.float32(1.0 / len(outs))
    return Wm


def agent_params(seed, n, d, spread=1e-2):
    """n agents' parameter vectors: a common model ~N(0, 0.05^2) plus a per-agent drift, fp32 [n,d]."""
    g = rng(seed)
    base = g.standard_normal(d, dtype=np.float32) * np.float32(0.05)
    return (base[None, :] + g.standard_normal((n, d), dtype=np.float32) * np.float32(spread)).astype(np.float32)
