"""One agent's 8-bit training step as a fixed sequence of liblpdt calls.

This is sequencing only: it plans buffers once (torch supplies device memory), then
`run()` issues the library calls of the forward pass, the loss, the backward pass and the
local SGD step on the current stream.  No arithmetic happens in Python, nothing is
allocated inside `run()`, so the step can be captured in a HIP graph.

Per quantized convolution (Section 3, "Low Precision Training"):
  forward : Wq = Q_nearest(W), Xq = Q_nearest(X) (shared by all consumers of X),
            Y = sX*sW * conv(Xq, Wq)
  backward: Gq = Q_stochastic(dY), quantized once and used by both products,
            dX (+)= sG*sW * conv_bwd_data(Gq, Wq)      (skipped for the network input)
            (the scale products are applied in the convolution kernels' epilogues)
            dW   = sG*sX * conv_bwd_weight(Gq, Xq)      (fp32, never re-quantized)
Range-EvoNorm hands the abs-max of its outputs to the quantizer that follows it, so that
quantizer makes a single pass.

The weight-gradient products have no consumer before the SGD update, so `run()` issues them
on a second stream (default priority) behind an event recorded after the gradient quantizer,
and the main stream waits for that stream once, before the update: they fill the gaps the
chain of backward-data / normalisation kernels leaves on the chip.
"""
import ctypes

import torch

from .binding import ConvDesc, LpdtError, lib, ROUND_NEAREST, ROUND_STOCHASTIC

_sz, _vp, _u64, _f32 = ctypes.c_size_t, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_float


def _p(t):
    return _vp(0) if t is None else _vp(t.data_ptr())


_second_streams = {}


def _second_stream(dev):
    """One second stream (default priority) per device and process, shared by every TrainStep.  HIP spreads the streams a
    process creates over a few hardware queues (4 here); a stream made per object sooner or later lands on the queue of
    the main stream, and the two then run one after the other (measured: a VGG-11 step 1.09 ms as the first step object of
    a process, 1.23 ms as the twentieth).  Step objects of one device run one at a time, so they can share it."""
    key = (dev.type, dev.index if dev.index is not None else torch.cuda.current_device())
    if key not in _second_streams:
        _second_streams[key] = torch.cuda.Stream(device=dev)
    return _second_streams[key]


class TrainStep:
    """net: a workloads.nets.Net-like object (ops, params, shapes, in_shape, classes).
    params / grads: flat fp32 device vectors of net.num_params() elements (e.g. a row of the
    agents' matrix); x: [batch,H,W,C] fp32 device tensor; labels: int32 device tensor or None
    (then `upstream` must be the gradient of the last tensor)."""

    def __init__(self, net, batch, params, grads, x, labels=None, upstream=None, lr=0.1, seed=0, eps=1e-5,
                 wgrad_16bit=False, overlap_wgrad=True, fuse_ren_quant=True, prepack_filters=True, conv_absmax=True,
                 fuse_conv_ren=False):
        self.L = lib()
        self.overlap_wgrad = overlap_wgrad
        self.fork_batch = 2              # second-stream calls issued behind one fork event (measured: 1 and 3 are slower, and so is
                                         # 2 with the pairs shifted by one call: +30 us)
        self.fuse_ren_quant = fuse_ren_quant   # Range-EvoNorm layers that feed only convolutions emit int8 codes directly
        # backward-data's transposed filters are made once per step, on the second stream beside the forward pass
        self.prepack_filters = prepack_filters and overlap_wgrad
        self.conv_absmax = conv_absmax   # products followed directly by a quantizer hand max|result| over
        # convolution -> Range-EvoNorm -> quantizer as one call where the shape allows; off by default: measured on the
        # ResNet-18 step it costs 0.04 ms (the statistics in the epilogue cost more than the pass over the tensor they replace)
        self.fuse_conv_ren = fuse_conv_ren
        self.net, self.N, self.lr, self.seed, self.eps = net, batch, lr, seed, eps
        # gradient bifurcation as the paper states it: weight gradients from a bfloat16 copy of the layer gradient
        # (the 8-bit codes still feed backward-data), for every layer but the one that reads the image; default: both
        # products from the 8-bit codes
        self.wgrad_16bit = wgrad_16bit
        self.dev = params.device
        # the library reads these tensors through raw addresses: a wrong type, size or device would be misread, not refused
        H0, W0, C0 = net.in_shape
        if params.dtype != torch.float32 or grads.dtype != torch.float32 or params.numel() != net.num_params() or grads.numel() != params.numel():
            raise LpdtError(-1, f"params and grads must be float32 vectors of {net.num_params()} elements")
        if x.dtype != torch.float32 or tuple(x.shape) != (batch, H0, W0, C0):
            raise LpdtError(-1, f"x must be a float32 tensor of shape {(batch, H0, W0, C0)}, got {x.dtype} {tuple(x.shape)}")
        if labels is not None and (labels.dtype != torch.int32 or labels.numel() != batch):
            raise LpdtError(-1, f"labels must be {batch} int32 values, got {labels.dtype} x {labels.numel()}")
        for name, t in (("grads", grads), ("x", x), ("labels", labels), ("upstream", upstream)):
            if t is not None and (t.device != self.dev or not t.is_contiguous()):
                raise LpdtError(-1, f"{name} must be contiguous and on {self.dev}")
        if not params.is_contiguous():
            raise LpdtError(-1, "params must be contiguous")
        self.params, self.grads = params, grads
        # the call list holds raw addresses: every tensor behind one must live as long as this object (labels handed over
        # as a temporary would otherwise be freed, and their memory reused, while the loss call still reads it)
        self.labels, self.upstream = labels, upstream
        f32 = lambda *s: torch.empty(s, dtype=torch.float32, device=self.dev)
        i8 = lambda *s: torch.empty(s, dtype=torch.int8, device=self.dev)
        i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=self.dev)
        self.pview, self.gview, self._poff = {}, {}, {}
        at = 0
        for name, shp in net.params:
            k = 1
            for s in shp:
                k *= s
            if at % 4:
                raise LpdtError(-1, "parameter tensors must start at multiples of 4 elements (16-byte alignment)")
            self.pview[name] = params[at:at + k].view(shp)
            self.gview[name] = grads[at:at + k].view(shp)
            self._poff[name] = (at, at + k)
            at += k
        self.act = {"x": x}
        self.absmax = {}                 # tensor name -> device scalar max|t| (when its producer supplies it)
        self.calls = []                  # (function, [args...], sr_layer or None)
        self.ws = torch.empty(1, dtype=torch.uint8, device=self.dev)
        self._ws_need = 256
        self._ws_side_need = 256
        self.loss = None
        consumers = {}
        for op in net.ops:
            for src in (op[2:4] if op[0] == "add" else ([op[1]] if op[0] == "loss" else [op[2]])):
                consumers[src] = consumers.get(src, 0) + 1
        self.consumers = consumers
        self._f32, self._i8, self._i32 = f32, i8, i32
        self._plan_forward(labels, upstream)
        self._plan_backward()
        self.ws = torch.empty(self._ws_need + 256, dtype=torch.uint8, device=self.dev)
        off = (-self.ws.data_ptr()) % 256
        self._ws_ptr, self._ws_bytes = _vp(self.ws.data_ptr() + off), _sz(self._ws_need)
        # the calls of the second stream have a workspace of their own
        self.ws_side = torch.empty(self._ws_side_need + 256, dtype=torch.uint8, device=self.dev)
        off = (-self.ws_side.data_ptr()) % 256
        side_ptr, side_bytes = _vp(self.ws_side.data_ptr() + off), _sz(self._ws_side_need)
        for c in self.calls:             # workspace arguments were planned as placeholders
            for i, a in enumerate(c[1]):
                if a == "WS":
                    c[1][i] = side_ptr if c[3] else self._ws_ptr
                elif a == "WSB":
                    c[1][i] = side_bytes if c[3] else self._ws_bytes
        self._side_stream = _second_stream(self.dev) if self.dev.type == "cuda" else None
        self._fork_events = [torch.cuda.Event() for c in self.calls if c[3]] if self._side_stream else []
        self._join_event = torch.cuda.Event() if self._side_stream else None

    # ------------------------------------------------------------------ planning helpers
    def _need_ws(self, nbytes, side=False):
        if side:
            self._ws_side_need = max(self._ws_side_need, int(nbytes))
        else:
            self._ws_need = max(self._ws_need, int(nbytes))

    def _emit(self, fn, args, sr_layer=None, side=False):
        """side: the call may run on the second stream (its inputs are final when it is issued and nothing
        before the SGD update reads its output)."""
        self.calls.append((fn, list(args), sr_layer, bool(side and self.overlap_wgrad)))

    def _quantize(self, src, q, scale, rounding, absmax=None, sr_layer=None):
        n = src.numel()
        if sr_layer is not None:
            # the counter ranges of run(): 2^24 Philox blocks (2^26 elements) per layer, 2^8 layers per step; beyond them
            # two tensors would share random numbers, against the independent stochastic rounding of Section 3
            if n > (1 << 26):
                raise LpdtError(-2, f"a stochastically rounded tensor of {n} elements exceeds the 2^26 elements a layer's "
                                    "Philox counter range holds")
            if sr_layer >= 256:
                raise LpdtError(-2, f"layer index {sr_layer} exceeds the 256 stochastic-rounding ranges of a step")
        if absmax is not None:
            self._emit(self.L.lpdt_quantize_with_absmax,
                       [_p(src), _sz(n), _p(absmax), rounding, _u64(self.seed), _u64(0), _p(q), _p(scale)], sr_layer)
        else:
            self._need_ws(self.L.lpdt_quantize_workspace_bytes(n))
            self._emit(self.L.lpdt_quantize,
                       [_p(src), _sz(n), rounding, _u64(self.seed), _u64(0), _p(q), _p(scale), "WS", "WSB"], sr_layer)

    def _desc(self, inp, a):
        H, W, C = self.net.shapes[inp]
        return ConvDesc.make(self.N, C, H, W, a["K"], a["R"], a["R"], a["stride"], a["pad"])

    # ------------------------------------------------------------------ forward
    def _plan_forward(self, labels, upstream):
        net, N, L = self.net, self.N, self.L
        self.xq, self.sx, self.wq, self.sw, self.desc, self.ren_saved, self.pool_idx = {}, {}, {}, {}, {}, {}, {}
        self.wpacked = {}                # conv output -> its filter as backward-data reads it
        # All filters are quantized by one call on the flat parameter vector (own scale each); their codes keep the
        # vector's layout, so a filter's codes are a 16-byte aligned slice when its offset is a multiple of 16.
        convs = [op for op in net.ops if op[0] == "conv"]
        # tensors all of whose consumers are quantized convolutions (only their int8 codes are ever read)
        readers = {}
        for op in net.ops:
            for src in (op[2:4] if op[0] == "add" else ([op[1]] if op[0] == "loss" else [op[2]])):
                readers.setdefault(src, set()).add(op[0])
        conv_only = {t for t, kinds in readers.items() if kinds == {"conv"}}
        # normalised tensors read by exactly one op, a max-pool: tensor -> that op
        pooled_by = {}
        for op in net.ops:
            if op[0] == "maxpool" and self.consumers.get(op[2], 0) == 1:
                pooled_by[op[2]] = op
        self.fused_pool = {}             # pooled tensor -> the normalised tensor that is never stored
        # Skip connections done in a convolution's epilogue: of an add's two operands, the one produced later, when it
        # is a convolution output nobody else reads, is accumulated straight into the other operand's buffer, provided
        # that buffer may be overwritten: its other readers are convolutions (they read its int8 copy) and the first of
        # them, which makes that copy, comes earlier.  conv output -> (sum tensor, buffer's tensor)
        pos = {"x": -1}
        for i, op in enumerate(net.ops):
            if op[0] != "loss":
                pos[op[1]] = i
        producer = {op[1]: op for op in net.ops if op[0] != "loss"}
        self.acc_conv, self.fused_add = {}, set()
        if self.fuse_ren_quant:
            for i, op in enumerate(net.ops):
                if op[0] != "add":
                    continue
                _, out, a_, b_ = op
                later, other = (a_, b_) if pos[a_] > pos[b_] else (b_, a_)
                if later not in producer or producer[later][0] != "conv" or self.consumers.get(later, 0) != 1 or other == "x":
                    continue
                others = [o for o in net.ops if o is not op and o[0] != "loss" and other in (o[2:4] if o[0] == "add" else [o[2]])]
                if any(o[0] != "conv" for o in others):
                    continue
                if others and min(pos[o[1]] for o in others) > pos[later]:
                    continue
                if other in conv_only or other in pooled_by:
                    continue                     # never stored as fp32
                self.acc_conv[later] = (out, other)
                self.fused_add.add(out)
        # conv -> Range-EvoNorm -> quantizer as one call (lpdt_qconv_ren_fwd_q): a convolution whose result (or, with the skip
        # connection in its epilogue, the sum) is read by a normalisation layer only, which in turn emits int8 codes, on
        # shapes where the convolution can take the layer's statistics on the way out.  conv output -> the ren op
        self.chain, self.chained_ren = {}, set()
        if self.fuse_ren_quant and self.fuse_conv_ren:
            ren_of = {op[2]: op for op in net.ops if op[0] == "ren"}
            for op in convs:
                res = self.acc_conv[op[1]][0] if op[1] in self.acc_conv else op[1]
                rop = ren_of.get(res)
                if rop is None or self.consumers.get(res, 0) != 1 or rop[1] in pooled_by or "conv" not in readers.get(rop[1], ()):
                    continue
                d = self._desc(op[2], op[3])
                H, W, C = net.shapes[rop[2]]
                if (self.conv_absmax and op[1] in conv_only) or L.lpdt_range_evonorm_fwd_q_workspace_bytes(N, H, W, C, rop[3]["groups"]) == 0:
                    continue
                if L.lpdt_qconv_kernel_id(ctypes.byref(d), 3) < 40:
                    continue                     # the library would run the two calls anyway
                self.chain[op[1]] = rop
                self.chained_ren.add(rop[1])
        spans = [self._poff[op[3]["w"]] for op in convs]
        batched = len(convs) > 1 and all(b % 16 == 0 for b, _ in spans)
        if batched:
            wq_flat, sw_all = self._i8(self.params.numel()), self._f32(len(convs))
            self._seg_arrays = ((ctypes.c_int64 * len(spans))(*[b for b, _ in spans]),
                                (ctypes.c_int64 * len(spans))(*[e for _, e in spans]))
            self._need_ws(L.lpdt_quantize_segments_workspace_bytes(len(spans)))
            self._emit(L.lpdt_quantize_segments,
                       [_p(self.params), self._seg_arrays[0], self._seg_arrays[1], len(spans), ROUND_NEAREST, _u64(self.seed),
                        _u64(0), _p(wq_flat), _p(sw_all), "WS", "WSB"])
            for i, (op, (b, e)) in enumerate(zip(convs, spans)):
                self.wq[op[1]] = wq_flat[b:e].view(self.pview[op[3]["w"]].shape)
                self.sw[op[1]] = sw_all[i:i + 1]
            if self.prepack_filters:     # the codes of every filter are final here: one launch prepares them all
                todo = []
                for op in convs:
                    if op[2] == "x":
                        continue         # no backward-data for the image layer
                    d = self._desc(op[2], op[3])
                    nb = int(L.lpdt_qconv_bwd_data_packed_filter_bytes(ctypes.byref(d)))
                    if nb == 0 or self.wq[op[1]].data_ptr() % 16:
                        continue
                    self.wpacked[op[1]] = torch.empty(nb, dtype=torch.uint8, device=self.dev)
                    todo.append((d, self.wq[op[1]], self.wpacked[op[1]], nb))
                if todo:
                    n = len(todo)
                    self._pack_arrays = ((ConvDesc * n)(*[t[0] for t in todo]), (ctypes.c_void_p * n)(*[t[1].data_ptr() for t in todo]),
                                         (ctypes.c_void_p * n)(*[t[2].data_ptr() for t in todo]), (ctypes.c_size_t * n)(*[t[3] for t in todo]))
                    self._emit(L.lpdt_qconv_bwd_data_pack_filters, [self._pack_arrays[0], n, *self._pack_arrays[1:]], side=True)
        for op in net.ops:
            kind = op[0]
            if kind == "conv":
                _, out, inp, a = op
                d = self._desc(inp, a)
                self.desc[out] = d
                w = self.pview[a["w"]]
                if not batched:
                    self.wq[out], self.sw[out] = self._i8(*w.shape), self._f32(1)
                    self._quantize(w, self.wq[out], self.sw[out], ROUND_NEAREST)
                if inp not in self.xq:       # one quantization per tensor, shared by its consumers
                    src = self.act[inp]
                    self.xq[inp], self.sx[inp] = self._i8(*src.shape), self._f32(1)
                    self._quantize(src, self.xq[inp], self.sx[inp], ROUND_NEAREST, self.absmax.get(inp))
                if out in self.chain:        # the normalisation layer and its quantizer ride along
                    rop = self.chain[out]
                    _, rout, rinp, ra = rop
                    g = ra["groups"]
                    H, W, C = net.shapes[rinp]
                    if out in self.acc_conv:
                        sum_name, other = self.acc_conv[out]
                        self.act[sum_name] = self.act[other]
                        y, accumulate = self.act[other], 1
                    else:
                        y, accumulate = self._f32(N, *net.shapes[out]), 0
                        self.act[out] = y
                    rng, amx, amn = self._f32(N, g), self._i32(N, g), self._i32(N, g)
                    self.ren_saved[rout] = (rng, amx, amn)
                    self.xq[rout], self.sx[rout] = self._i8(N, H, W, C), self._f32(1)
                    z = None
                    if rout not in conv_only:
                        z = self._f32(N, H, W, C)
                        self.act[rout] = z
                    pv = self.pview
                    self._need_ws(L.lpdt_qconv_ren_fwd_q_workspace_bytes(ctypes.byref(d), g))
                    self._emit(L.lpdt_qconv_ren_fwd_q,
                               [ctypes.byref(d), _p(self.xq[inp]), _p(self.wq[out]), _p(self.sx[inp]), _p(self.sw[out]), accumulate, g,
                                _p(pv[ra["p"] + ".v"]), _p(pv[ra["p"] + ".gamma"]), _p(pv[ra["p"] + ".beta"]), _f32(self.eps), _p(y), _p(z),
                                _p(self.xq[rout]), _p(self.sx[rout]), _p(rng), _p(amx), _p(amn), "WS", "WSB"])
                    continue
                if out in self.acc_conv:     # y += conv: the sum of the skip connection, in the other operand's buffer
                    sum_name, other = self.acc_conv[out]
                    self.act[sum_name] = self.act[other]
                    self._need_ws(L.lpdt_qconv_fwd_f32_add_workspace_bytes(ctypes.byref(d)))
                    self._emit(L.lpdt_qconv_fwd_f32_add, [ctypes.byref(d), _p(self.xq[inp]), _p(self.wq[out]), _p(self.sx[inp]),
                                                          _p(self.sw[out]), _p(self.act[other]), "WS", "WSB"])
                    continue
                y = self._f32(N, *net.shapes[out])
                self.act[out] = y
                if self.conv_absmax and out in conv_only:         # quantized next, with no normalisation layer between: the product hands max|y| over
                    self.absmax[out] = self._f32(1)
                    self._need_ws(L.lpdt_qconv_fwd_f32_absmax_workspace_bytes(ctypes.byref(d)))
                    self._emit(L.lpdt_qconv_fwd_f32_absmax, [ctypes.byref(d), _p(self.xq[inp]), _p(self.wq[out]), _p(self.sx[inp]),
                                                             _p(self.sw[out]), _p(y), _p(self.absmax[out]), "WS", "WSB"])
                    continue
                self._need_ws(L.lpdt_qconv_fwd_f32_workspace_bytes(ctypes.byref(d)))
                self._emit(L.lpdt_qconv_fwd_f32, [ctypes.byref(d), _p(self.xq[inp]), _p(self.wq[out]), _p(self.sx[inp]),
                                                  _p(self.sw[out]), _p(y), "WS", "WSB"])
            elif kind == "ren":
                _, out, inp, a = op
                if out in self.chained_ren:      # done by the call of the convolution before it
                    continue
                H, W, C = net.shapes[inp]
                g = a["groups"]
                rng, amx, amn = self._f32(N, g), self._i32(N, g), self._i32(N, g)
                self.ren_saved[out] = (rng, amx, amn)
                pv = self.pview
                pool = pooled_by.get(out)
                if (self.fuse_ren_quant and pool is not None and pool[3]["k"] <= 2 * pool[3]["stride"]
                        and L.lpdt_range_evonorm_maxpool_fwd_workspace_bytes(N, H, W, C, g) > 0):
                    # the only reader is a max-pool: one call gives the pooled tensor, y is never stored
                    pa, pout = pool[3], pool[1]
                    z, idx = self._f32(N, *net.shapes[pout]), self._i32(N, *net.shapes[pout])
                    self.act[pout], self.pool_idx[pout] = z, idx
                    self.fused_pool[pout] = out
                    self.absmax[pout] = self._f32(1)
                    self._need_ws(L.lpdt_range_evonorm_maxpool_fwd_workspace_bytes(N, H, W, C, g))
                    self._emit(L.lpdt_range_evonorm_maxpool_fwd,
                               [_p(self.act[inp]), N, H, W, C, g, _p(pv[a["p"] + ".v"]), _p(pv[a["p"] + ".gamma"]),
                                _p(pv[a["p"] + ".beta"]), _f32(self.eps), pa["k"], pa["stride"], pa["pad"], _p(z), _p(idx), _p(rng),
                                _p(amx), _p(amn), _p(self.absmax[pout]), "WS", "WSB"])
                    continue
                if (self.fuse_ren_quant and "conv" in readers.get(out, ())
                        and L.lpdt_range_evonorm_fwd_q_workspace_bytes(N, H, W, C, g) > 0):
                    # a quantized convolution reads the output: the layer emits the int8 codes itself; y is stored as well only
                    # when something else (a skip connection) reads it at full precision
                    self.xq[out], self.sx[out] = self._i8(N, H, W, C), self._f32(1)
                    y = None
                    if out not in conv_only:
                        y = self._f32(N, H, W, C)
                        self.act[out] = y
                    self._need_ws(L.lpdt_range_evonorm_fwd_q_workspace_bytes(N, H, W, C, g))
                    self._emit(L.lpdt_range_evonorm_fwd_q,
                               [_p(self.act[inp]), N, H, W, C, g, _p(pv[a["p"] + ".v"]), _p(pv[a["p"] + ".gamma"]),
                                _p(pv[a["p"] + ".beta"]), _f32(self.eps), _p(self.xq[out]), _p(self.sx[out]), _p(y), _p(rng), _p(amx),
                                _p(amn), "WS", "WSB"])
                    continue
                y = self._f32(N, H, W, C)
                self.act[out] = y
                self.absmax[out] = self._f32(1)
                self._need_ws(L.lpdt_range_evonorm_fwd_workspace_bytes(N, H, W, C, g))
                self._emit(L.lpdt_range_evonorm_fwd,
                           [_p(self.act[inp]), N, H, W, C, g, _p(pv[a["p"] + ".v"]), _p(pv[a["p"] + ".gamma"]),
                            _p(pv[a["p"] + ".beta"]), _f32(self.eps), _p(y), _p(rng), _p(amx), _p(amn),
                            _p(self.absmax[out]), "WS", "WSB"])
            elif kind == "add":
                _, out, a_, b_ = op
                if out in self.fused_add:        # done in the epilogue of the convolution that produced one operand
                    continue
                y = self._f32(N, *net.shapes[out])
                self.act[out] = y
                self._emit(L.lpdt_add, [_p(self.act[a_]), _p(self.act[b_]), _sz(y.numel()), _p(y)])
            elif kind == "maxpool":
                _, out, inp, a = op
                if out in self.fused_pool:       # produced together with the normalisation layer before it
                    continue
                H, W, C = net.shapes[inp]
                y = self._f32(N, *net.shapes[out])
                idx = self._i32(N, *net.shapes[out])
                self.act[out], self.pool_idx[out] = y, idx
                self._emit(L.lpdt_maxpool_fwd, [_p(self.act[inp]), N, H, W, C, a["k"], a["stride"], a["pad"], _p(y), _p(idx)])
            elif kind == "avgpool":
                _, out, inp = op
                H, W, C = net.shapes[inp]
                y = self._f32(N, 1, 1, C)
                self.act[out] = y
                self._emit(L.lpdt_avgpool_fwd, [_p(self.act[inp]), N, H * W, C, _p(y)])
            elif kind == "loss":
                inp = op[1]
                self.loss = self._f32(1 + N)
                self.grad = {inp: self._f32(N, 1, 1, net.classes)}
                self._emit(L.lpdt_softmax_xent, [_p(self.act[inp]), _p(labels), N, net.classes, _p(self.loss), _p(self.grad[inp])])
        if net.ops[-1][0] != "loss":
            self.grad = {net.ops[-1][1]: upstream}

    # ------------------------------------------------------------------ backward
    def _grad_target(self, name, pending):
        """Buffer that receives a gradient contribution for tensor `name` and whether to accumulate.
        A buffer still owed to another tensor whose producer has not run yet is never updated in place."""
        if name not in self.grad:
            self.grad[name] = self._f32(self.N, *self.net.shapes[name])
            return self.grad[name], 0
        buf = self.grad[name]
        for other, t in self.grad.items():
            if other != name and other in pending and t.data_ptr() == buf.data_ptr():
                raise LpdtError(-2, f"gradient buffer of {name} is shared with pending tensor {other}")
        return buf, 1

    def _plan_backward(self):
        net, N, L = self.net, self.N, self.L
        self.gabsmax, self.gq, self.sg, self._keep = {}, {}, {}, []
        self.pooled_grad = {}            # normalised tensor -> (pooled gradient, winners, pool attributes) when fused
        pending = {op[1] for op in net.ops if op[0] != "loss"}      # tensors whose producer's backward has not run
        conv_index = 0
        deferred = {}                    # tensor -> backward-data calls waiting for another writer of its gradient
        producer_kind = {op[1]: op[0] for op in net.ops if op[0] != "loss"}
        if self.wpacked:
            self.calls.append((None, [], None, False))   # the main stream waits here for the second stream's filter copies
        for op in reversed(net.ops):
            kind = op[0]
            if kind == "loss":
                continue
            out = op[1]
            pending.discard(out)
            for f in deferred.pop(out, []):      # (never left over in the benchmark networks)
                f()
            dy = self.grad.get(out)
            if dy is None and out not in self.pooled_grad:
                raise LpdtError(-2, f"tensor {out} has no gradient (dead branch)")
            if kind == "conv":
                _, _, inp, a = op
                d = self.desc[out]
                conv_index += 1
                gq, sg = self._i8(*dy.shape), self._f32(1)
                self.gq[out], self.sg[out] = gq, sg
                self._quantize(dy, gq, sg, ROUND_STOCHASTIC, self.gabsmax.get(out), sr_layer=conv_index)
                if inp != "x":
                    def bwd_data(out=out, d=d, gq=gq, sg=sg, inp=inp):
                        buf, accumulate = self._grad_target(inp, pending)
                        self.gabsmax.pop(inp, None)
                        if self.conv_absmax and producer_kind.get(inp) == "conv" and self.consumers.get(inp, 0) == 1:
                            # the whole gradient of a convolution's output, quantized next: the product hands max|dx| over
                            self.gabsmax[inp] = self._f32(1)
                            self._need_ws(L.lpdt_qconv_bwd_data_f32_absmax_workspace_bytes(ctypes.byref(d)))
                            self._emit(L.lpdt_qconv_bwd_data_f32_absmax,
                                       [ctypes.byref(d), _p(gq), _p(self.wq[out]), _p(self.wpacked.get(out)), _p(sg), _p(self.sw[out]),
                                        _p(buf), accumulate, _p(self.gabsmax[inp]), "WS", "WSB"])
                            return
                        self._need_ws(L.lpdt_qconv_bwd_data_f32_workspace_bytes(ctypes.byref(d)))
                        if out in self.wpacked:
                            self._emit(L.lpdt_qconv_bwd_data_f32_packed, [ctypes.byref(d), _p(gq), _p(self.wpacked[out]), _p(sg),
                                                                          _p(self.sw[out]), _p(buf), accumulate, "WS", "WSB"])
                        else:
                            self._emit(L.lpdt_qconv_bwd_data_f32, [ctypes.byref(d), _p(gq), _p(self.wq[out]), _p(sg),
                                                                   _p(self.sw[out]), _p(buf), accumulate, "WS", "WSB"])
                    # A strided 1x1 projection reaches only every stride-th pixel of its input.  As the first writer of that
                    # gradient it would have to fill the rest with zeros, and the block's other convolution would then read
                    # everything back to add to it; after that convolution it adds into a quarter of the pixels instead.
                    later = [o for o in net.ops if o[0] == "conv" and o[2] == inp and o[1] in pending]
                    if a["R"] == 1 and a["stride"] > 1 and inp not in self.grad and later:
                        deferred.setdefault(inp, []).append(bwd_data)
                    else:
                        bwd_data()
                        for f in deferred.pop(inp, []):
                            f()
                gw = self.gview[a["w"]]
                if self.wgrad_16bit and inp != "x":   # the image layer (3 channels) has no tiled 16-bit kernel: 8-bit path
                    g16 = torch.empty(dy.shape, dtype=torch.int16, device=self.dev)
                    self._keep.append(g16)
                    self._emit(L.lpdt_to_bf16, [_p(dy), _sz(dy.numel()), _p(g16)])
                    self._need_ws(L.lpdt_qconv_bwd_weight_bf16_workspace_bytes(ctypes.byref(d)), side=self.overlap_wgrad)
                    self._emit(L.lpdt_qconv_bwd_weight_bf16, [ctypes.byref(d), _p(g16), _p(self.xq[inp]), _p(self.sx[inp]), _p(gw),
                                                              "WS", "WSB"], side=True)
                else:
                    # the image layer's product is the last of the backward pass and nothing is left to run beside it: on
                    # the main stream it saves the fork and join around it
                    beside = inp != "x"
                    self._need_ws(L.lpdt_qconv_bwd_weight_f32_workspace_bytes(ctypes.byref(d)), side=self.overlap_wgrad and beside)
                    self._emit(L.lpdt_qconv_bwd_weight_f32, [ctypes.byref(d), _p(gq), _p(self.xq[inp]), _p(sg), _p(self.sx[inp]),
                                                             _p(gw), "WS", "WSB"], side=beside)
            elif kind == "ren":
                _, _, inp, a = op
                H, W, C = net.shapes[inp]
                g = a["groups"]
                if inp in self.grad:
                    raise LpdtError(-2, f"Range-EvoNorm input {inp} has another consumer")
                dx = self._f32(N, H, W, C)
                self.grad[inp] = dx
                self.gabsmax[inp] = self._f32(1)
                rng, amx, amn = self.ren_saved[out]
                pv, gv = self.pview, self.gview
                if out in self.pooled_grad:      # the layer's output went through a max-pool only: gather its gradient on the fly
                    dz, idx, pa = self.pooled_grad[out]
                    self._need_ws(L.lpdt_range_evonorm_maxpool_bwd_workspace_bytes(N, H, W, C, g))
                    self._emit(L.lpdt_range_evonorm_maxpool_bwd,
                               [_p(dz), _p(idx), _p(self.act[inp]), N, H, W, C, g, _p(pv[a["p"] + ".v"]), _p(pv[a["p"] + ".gamma"]),
                                _f32(self.eps), pa["k"], pa["stride"], pa["pad"], _p(rng), _p(amx), _p(amn), _p(dx),
                                _p(gv[a["p"] + ".v"]), _p(gv[a["p"] + ".gamma"]), _p(gv[a["p"] + ".beta"]), _p(self.gabsmax[inp]),
                                "WS", "WSB"])
                    continue
                self._need_ws(L.lpdt_range_evonorm_bwd_workspace_bytes(N, H, W, C, g))
                self._emit(L.lpdt_range_evonorm_bwd,
                           [_p(dy), _p(self.act[inp]), N, H, W, C, g, _p(pv[a["p"] + ".v"]), _p(pv[a["p"] + ".gamma"]),
                            _f32(self.eps), _p(rng), _p(amx), _p(amn), _p(dx), _p(gv[a["p"] + ".v"]),
                            _p(gv[a["p"] + ".gamma"]), _p(gv[a["p"] + ".beta"]), _p(self.gabsmax[inp]), "WS", "WSB"])
            elif kind == "add":
                _, _, a_, b_ = op
                for src in (a_, b_):
                    if src not in self.grad:
                        self.grad[src] = dy                      # fan-out of the same gradient: no copy
                        if out in self.gabsmax:
                            self.gabsmax[src] = self.gabsmax[out]
                    else:
                        buf, _ = self._grad_target(src, pending)
                        self.gabsmax.pop(src, None)
                        self._emit(L.lpdt_add, [_p(buf), _p(dy), _sz(buf.numel()), _p(buf)])
            elif kind == "maxpool":
                _, _, inp, a = op
                if out in self.fused_pool:       # its backward is part of the normalisation layer's
                    self.pooled_grad[inp] = (dy, self.pool_idx[out], a)
                    continue
                H, W, C = net.shapes[inp]
                if inp in self.grad:
                    raise LpdtError(-2, f"max-pool input {inp} has another consumer")
                dx = self._f32(N, H, W, C)
                self.grad[inp] = dx
                self._emit(L.lpdt_maxpool_bwd, [_p(dy), _p(self.pool_idx[out]), N, H, W, C, a["k"], a["stride"], a["pad"], _p(dx)])
            elif kind == "avgpool":
                _, _, inp = op
                H, W, C = net.shapes[inp]
                if inp in self.grad:
                    raise LpdtError(-2, f"average-pool input {inp} has another consumer")
                dx = self._f32(N, H, W, C)
                self.grad[inp] = dx
                self._emit(L.lpdt_avgpool_bwd, [_p(dy), N, H * W, C, _p(dx)])
        # Algorithm 1 step 3: x~ = x - lr * g
        self._emit(L.lpdt_sgd, [_p(self.params), _p(self.grads), _sz(self.params.numel()), _f32(self.lr)])

    # ------------------------------------------------------------------ execution
    def run(self, step=0, upto=None):
        """Enqueue the whole step on the current stream (the weight-gradient calls on the second stream, joined
        before the SGD update).  Stochastic-rounding counters are offset = step * 2^32 + conv_index * 2^24 (in
        Philox blocks of 4 elements)."""
        main = torch.cuda.current_stream()
        stream = _vp(main.cuda_stream)
        side = self._side_stream
        side_ptr = _vp(side.cuda_stream) if side is not None else stream
        last = self.L.lpdt_last_error
        forks, joined = 0, True
        calls = self.calls if upto is None else self.calls[:upto]
        n = len(calls)
        pending = []                         # calls of the second stream not yet issued: they go out in batches behind one fork

        def flush():
            nonlocal forks, joined
            if not pending:
                return
            ev = self._fork_events[forks]
            forks += 1
            ev.record(main)                  # everything issued so far (the quantizers of these layers' gradients included)
            side.wait_event(ev)
            for f, a in pending:
                rc_ = f(*a, side_ptr)
                if rc_ != 0:
                    raise LpdtError(rc_, last().decode())
            pending.clear()
            joined = False

        def join():
            nonlocal joined
            flush()
            if not joined:
                self._join_event.record(side)
                main.wait_event(self._join_event)
                joined = True

        # the weight-gradient products are sized at launch: tell the library that they run beside the main chain
        self.L.lpdt_qconv_set_wgrad_beside(1 if side is not None else 0)
        try:
            self._issue(calls, n, step, stream, pending, flush, join)
        finally:
            self.L.lpdt_qconv_set_wgrad_beside(0)

    def _issue(self, calls, n, step, stream, pending, flush, join):
        last = self.L.lpdt_last_error
        for i, (fn, args, sr, on_side) in enumerate(calls):
            if sr is not None:
                pos = 5 if fn is self.L.lpdt_quantize_with_absmax else 4
                args[pos] = _u64((int(step) << 32) + (sr << 24))
            if on_side:
                pending.append((fn, args))
                if i + 1 < n and calls[i + 1][3]:
                    continue                 # a run of consecutive second-stream calls is never split
                # a call goes out at once when no partner follows before the next join (the filter preparation at the
                # start of the step would otherwise wait for the first weight gradient and be joined right after it)
                partner = False
                for j in range(i + 1, n):
                    if calls[j][0] is None or calls[j][0] is self.L.lpdt_sgd:
                        break
                    if calls[j][3]:
                        partner = True
                        break
                if len(pending) >= self.fork_batch or not partner:
                    flush()
                continue
            if fn is None:
                join()
                continue
            if fn is self.L.lpdt_sgd or i == n - 1:
                join()
            rc = fn(*args, stream)
            if rc != 0:
                raise LpdtError(rc, last().decode())
        join()

    def run_timed(self, step=0, with_desc=False):
        """Like run(), but everything on the current stream, every library call bracketed with events on it; returns
        [(entry point name, milliseconds)] in call order (one synchronisation at the end); with_desc adds the
        convolution descriptor of the call as a third item (None for other calls)."""
        stream = _vp(torch.cuda.current_stream().cuda_stream)
        marks = []
        for fn, args, sr, _ in self.calls:
            if fn is None:
                continue
            if sr is not None:
                pos = 5 if fn is self.L.lpdt_quantize_with_absmax else 4
                args[pos] = _u64((int(step) << 32) + (sr << 24))
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rc = fn(*args, stream)
            b.record()
            if rc != 0:
                raise LpdtError(rc, self.L.lpdt_last_error().decode())
            desc = getattr(args[0], "_obj", None) if fn.__name__.startswith("lpdt_qconv_") else None
            marks.append((fn.__name__, a, b, desc))
        torch.cuda.synchronize()
        if with_desc:
            return [(name, a.elapsed_time(b), desc) for name, a, b, desc in marks]
        return [(name, a.elapsed_time(b)) for name, a, b, _ in marks]

    def conv_work(self):
        """[(entry point name, multiply-adds)] for every convolution call of one step, in call order."""
        out = []
        for fn, args, _, _ in self.calls:
            if fn is None:
                continue
            if fn.__name__ in ("lpdt_qconv_fwd_f32", "lpdt_qconv_fwd_f32_add", "lpdt_qconv_fwd_f32_absmax", "lpdt_qconv_bwd_data_f32",
                               "lpdt_qconv_bwd_data_f32_packed", "lpdt_qconv_bwd_data_f32_absmax", "lpdt_qconv_bwd_weight_f32",
                               "lpdt_qconv_bwd_weight_bf16"):
                d = args[0]._obj
                out.append((fn.__name__, d.N * d.P * d.Q * d.K * d.C * d.R * d.S))
        return out
