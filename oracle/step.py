"""One agent's 8-bit training step composed from the oracle's functions (test infrastructure).

Walks the same layer table as the GPU step driver, calling only `oracle.*`.  Arithmetic inside each
operation is the oracle's (fp64 / exact integers); tensors handed from one operation to the next are
stored as fp32, the precision the method's tensors have.  Every intermediate is kept so that tests can
feed any single stage of the GPU path with the oracle's inputs for that stage.
"""
import numpy as np

import oracle as orc


def f32(a):
    return np.asarray(a, dtype=np.float32)


def run_step(net, batch, params, x, labels=None, upstream=None, lr=0.1, seed=0, step=0, eps=1e-5):
    """params: {name: fp32 array}.  Returns a dict with activations `act`, gradients `grad`, parameter
    gradients `pgrad`, updated parameters `new_params`, codes/scales `q`, Range-EvoNorm stats `ren`, `loss`."""
    act = {"x": f32(x)}
    q = {}            # "x:<tensor>" / "w:<conv>" / "g:<conv>" -> (codes, scale)
    ren, pool_idx, desc = {}, {}, {}
    loss = None
    for op in net.ops:
        kind = op[0]
        if kind == "conv":
            _, out, inp, a = op
            H, W, C = net.shapes[inp]
            d = orc.conv_desc(batch, C, H, W, a["K"], a["R"], a["R"], a["stride"], a["pad"])
            desc[out] = d
            q["w:" + out] = orc.quantize(params[a["w"]], 0)
            if "x:" + inp not in q:
                q["x:" + inp] = orc.quantize(act[inp], 0)
            xq, sx = q["x:" + inp]
            wq, sw = q["w:" + out]
            acc = orc.qconv_fwd(d, xq, wq)
            act[out] = f32(orc.dequantize(acc, sx, sw))
        elif kind == "ren":
            _, out, inp, a = op
            y, rng, amx, amn = orc.range_evonorm_fwd(act[inp], a["groups"], params[a["p"] + ".v"],
                                                     params[a["p"] + ".gamma"], params[a["p"] + ".beta"], eps)
            act[out] = f32(y)
            ren[out] = (rng, amx, amn)
        elif kind == "add":
            _, out, a_, b_ = op
            act[out] = f32(orc.add(act[a_], act[b_]))
        elif kind == "maxpool":
            _, out, inp, a = op
            act[out], pool_idx[out] = orc.maxpool_fwd(act[inp], a["k"], a["stride"], a["pad"])
        elif kind == "avgpool":
            _, out, inp = op
            N, H, W, C = act[inp].shape
            act[out] = f32(orc.avgpool_fwd(act[inp])).reshape(N, 1, 1, C)
        elif kind == "loss":
            inp = op[1]
            loss, dl = orc.softmax_xent(act[inp].reshape(batch, net.classes), labels)
            grad = {inp: f32(dl).reshape(batch, 1, 1, net.classes)}
    if net.ops[-1][0] != "loss":
        grad = {net.ops[-1][1]: f32(upstream)}

    def contribute(name, g):
        grad[name] = f32(g) if name not in grad else f32(orc.add(grad[name], g))

    pgrad = {}
    conv_index = 0
    for op in reversed(net.ops):
        kind = op[0]
        if kind == "loss":
            continue
        out = op[1]
        dy = grad[out]
        if kind == "conv":
            _, _, inp, a = op
            conv_index += 1
            d = desc[out]
            gq, sg = orc.quantize(dy, 1, seed, (int(step) << 32) + (conv_index << 24))
            q["g:" + out] = (gq, sg)
            xq, sx = q["x:" + inp]
            wq, sw = q["w:" + out]
            if inp != "x":
                contribute(inp, orc.dequantize(orc.qconv_bwd_data(d, gq, wq), sg, sw))
            pgrad[a["w"]] = f32(orc.dequantize(orc.qconv_bwd_weight(d, gq, xq), sg, sx))
        elif kind == "ren":
            _, _, inp, a = op
            dx, dv, dg, db = orc.range_evonorm_bwd(dy.astype(np.float64), act[inp], a["groups"], params[a["p"] + ".v"],
                                                   params[a["p"] + ".gamma"], eps)
            contribute(inp, dx)
            pgrad[a["p"] + ".v"], pgrad[a["p"] + ".gamma"], pgrad[a["p"] + ".beta"] = f32(dv), f32(dg), f32(db)
        elif kind == "add":
            _, _, a_, b_ = op
            contribute(a_, dy)
            contribute(b_, dy)
        elif kind == "maxpool":
            _, _, inp, a = op
            contribute(inp, orc.maxpool_bwd(dy.astype(np.float64), pool_idx[out], act[inp].shape))
        elif kind == "avgpool":
            _, _, inp = op
            N, H, W, C = act[inp].shape
            contribute(inp, orc.avgpool_bwd(dy.reshape(N, C).astype(np.float64), act[inp].shape))
    new_params = {k: f32(orc.sgd(params[k], pgrad[k], lr)) for k in params}
    return {"act": act, "grad": grad, "pgrad": pgrad, "new_params": new_params, "q": q, "ren": ren, "loss": loss}
