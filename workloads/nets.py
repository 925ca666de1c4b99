"""Layer tables of the benchmark networks (shapes only; no arithmetic).

A network is a list of ops over named NHWC tensors, executed in order for the
forward pass and in reverse for the backward pass:

  ("conv",    out, inp, {"w": param, "K", "R", "stride", "pad"})   8-bit quantized convolution / linear layer
  ("ren",     out, inp, {"p": param prefix, "groups"})             Range-EvoNorm, parameters p.v, p.gamma, p.beta
  ("add",     out, a, b)                                            skip connection
  ("maxpool", out, inp, {"k", "stride", "pad"})
  ("avgpool", out, inp)                                             global average pool -> [N,1,1,C]
  ("loss",    inp)                                                  softmax cross-entropy on [N,1,1,classes]

Wiring follows the paper's recipe of replacing every BatchNorm+ReLU pair with the
normalisation-activation layer (Section 4): conv -> REN -> conv -> (+ shortcut) -> REN;
a stride-2 stage entry uses a 1x1 stride-2 quantized convolution as projection shortcut.
"""


class Net:
    def __init__(self, name, in_shape, classes):
        self.name, self.in_shape, self.classes = name, in_shape, classes   # in_shape = (H, W, C)
        self.ops = []
        self.params = []          # (name, shape) in creation order; conv filters are KRSC
        self.shapes = {"x": in_shape}

    def _param(self, name, shape):
        self.params.append((name, tuple(shape)))
        return name

    def conv(self, out, inp, K, R, stride=1, pad=0):
        H, W, C = self.shapes[inp]
        w = self._param(f"{out}.w", (K, R, R, C))
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
        self.shapes[out] = (P, Q, K)
        self.ops.append(("conv", out, inp, {"w": w, "K": K, "R": R, "stride": stride, "pad": pad}))
        return out

    def ren(self, out, inp, groups):
        H, W, C = self.shapes[inp]
        for s in ("v", "gamma", "beta"):
            self._param(f"{out}.{s}", (C,))
        self.shapes[out] = (H, W, C)
        self.ops.append(("ren", out, inp, {"p": out, "groups": groups}))
        return out

    def add(self, out, a, b):
        assert self.shapes[a] == self.shapes[b]
        self.shapes[out] = self.shapes[a]
        self.ops.append(("add", out, a, b))
        return out

    def maxpool(self, out, inp, k, stride, pad):
        H, W, C = self.shapes[inp]
        self.shapes[out] = ((H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1, C)
        self.ops.append(("maxpool", out, inp, {"k": k, "stride": stride, "pad": pad}))
        return out

    def avgpool(self, out, inp):
        self.shapes[out] = (1, 1, self.shapes[inp][2])
        self.ops.append(("avgpool", out, inp))
        return out

    def loss(self, inp):
        assert self.shapes[inp] == (1, 1, self.classes)
        self.ops.append(("loss", inp))

    # ---- bookkeeping used by the benchmark
    def num_params(self):
        n = 0
        for _, shp in self.params:
            k = 1
            for s in shp:
                k *= s
            n += k
        return n

    def param_offsets(self):
        """Flat-vector offsets of the parameter tensors (the segments of layer-wise top-k)."""
        offs, at = [0], 0
        for _, shp in self.params:
            k = 1
            for s in shp:
                k *= s
            at += k
            offs.append(at)
        return offs

    def conv_macs(self, batch):
        """(forward MACs, forward+backward MACs) per step by the paper's count b*Cout*Cin*K^2*P^2 per product;
        the first layer has no backward-data product (nothing upstream of the image)."""
        fwd = tot = 0
        first = True
        for op in self.ops:
            if op[0] != "conv":
                continue
            _, out, inp, a = op
            P, Q, K = self.shapes[out]
            C = self.shapes[inp][2]
            m = batch * P * Q * K * C * a["R"] * a["R"]
            fwd += m
            tot += m * (2 if first else 3)
            first = False
        return fwd, tot


def single_layer():
    """Config 1: one 3x3 16->16 convolution on 32x32 followed by Range-EvoNorm (groups 8)."""
    n = Net("single-layer", (32, 32, 16), 0)
    n.conv("c", "x", 16, 3, 1, 1)
    n.ren("z", "c", 8)
    return n


def transformer_ffn():
    """Quantized linear layers at the shapes of a DistilBERT feed-forward block (hidden 768, inner 3072) plus a
    768 -> 768 projection, as 1x1 convolutions over tokens (the batch axis holds the tokens; H = W = 1).  Only the
    int8 products and their quantizers: no normalisation between the layers."""
    n = Net("transformer-ffn", (1, 1, 768), 0)
    n.conv("fc1", "x", 3072, 1, 1, 0)
    n.conv("fc2", "fc1", 768, 1, 1, 0)
    n.conv("proj", "fc2", 768, 1, 1, 0)
    return n


def _basic_block(n, name, inp, K, stride, groups):
    a = n.conv(f"{name}.c1", inp, K, 3, stride, 1)
    a = n.ren(f"{name}.n1", a, groups)
    a = n.conv(f"{name}.c2", a, K, 3, 1, 1)
    sc = inp
    if stride != 1 or n.shapes[inp][2] != K:
        sc = n.conv(f"{name}.sc", inp, K, 1, stride, 0)
    a = n.add(f"{name}.sum", a, sc)
    return n.ren(f"{name}.n2", a, groups)


def resnet20(classes=10, groups=8):
    """Configs 2 and 3: 3 stages x 3 basic blocks, widths 16/32/64, 32x32x3 input (0.27 M parameters)."""
    n = Net("resnet20", (32, 32, 3), classes)
    a = n.ren("stem.n", n.conv("stem.c", "x", 16, 3, 1, 1), groups)
    for si, K in enumerate((16, 32, 64)):
        for b in range(3):
            a = _basic_block(n, f"s{si}b{b}", a, K, 2 if (si > 0 and b == 0) else 1, groups)
    a = n.avgpool("pool", a)
    a = n.conv("fc", a, classes, 1, 1, 0)
    n.loss(a)
    return n


def vgg11(classes=10, groups=32):
    """Config 4: channels 64,128,256,256,512,512,512,512 with max-pools after stages, classifier
    Linear(512,512) -> REN -> Linear(512,classes) (9.49 M parameters)."""
    n = Net("vgg11", (32, 32, 3), classes)
    a = "x"
    plan = [(64, True), (128, True), (256, False), (256, True), (512, False), (512, True), (512, False), (512, True)]
    for i, (K, pool) in enumerate(plan):
        a = n.ren(f"n{i}", n.conv(f"c{i}", a, K, 3, 1, 1), groups)
        if pool:
            a = n.maxpool(f"p{i}", a, 2, 2, 0)
    a = n.ren("fc1.n", n.conv("fc1", a, 512, 1, 1, 0), groups)
    a = n.conv("fc2", a, classes, 1, 1, 0)
    n.loss(a)
    return n


def resnet18(classes=100, groups=32):
    """Config 5: 7x7 stride-2 stem, 3x3 stride-2 max-pool, 4 stages x 2 basic blocks, widths
    64/128/256/512, 224x224x3 input (11.2 M parameters)."""
    n = Net("resnet18", (224, 224, 3), classes)
    a = n.ren("stem.n", n.conv("stem.c", "x", 64, 7, 2, 3), groups)
    a = n.maxpool("stem.p", a, 3, 2, 1)
    for si, K in enumerate((64, 128, 256, 512)):
        for b in range(2):
            a = _basic_block(n, f"s{si}b{b}", a, K, 2 if (si > 0 and b == 0) else 1, groups)
    a = n.avgpool("pool", a)
    a = n.conv("fc", a, classes, 1, 1, 0)
    n.loss(a)
    return n


def init_params(net, seed):
    """Kaiming-normal filters, Range-EvoNorm v = gamma = 1, beta = 0; returns {name: fp32 array}."""
    import numpy as np
    from . import kaiming_filter
    out = {}
    for i, (name, shp) in enumerate(net.params):
        if name.endswith(".w"):
            out[name] = kaiming_filter(seed + i, *shp)
        elif name.endswith(".beta"):
            out[name] = np.zeros(shp, np.float32)
        else:
            out[name] = np.ones(shp, np.float32)
    return out
