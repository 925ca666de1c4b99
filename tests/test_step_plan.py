"""Host-side checks of the step planner (no GPU: a TrainStep on CPU tensors only plans its call list, nothing is launched)."""
import gc
import weakref

import numpy as np
import pytest
import torch

import workloads as wl
from workloads import nets

step_mod = pytest.importorskip("paper_2111_09389_amd.step")


def _build(net, N, **kw):
    """Builds a step object from temporaries only: nothing but the object itself can keep its operands alive."""
    H, W, C = net.in_shape
    params = nets.init_params(net, 1)
    flat = torch.from_numpy(np.concatenate([params[n].ravel() for n, _ in net.params]).astype(np.float32))
    return step_mod.TrainStep(net, N, flat, torch.zeros_like(flat), torch.from_numpy(wl.images(1, N, H, W, C)),
                              torch.from_numpy(wl.labels_uniform(2, N, net.classes)), **kw)


@pytest.mark.parametrize("name,N", [("resnet20", 4), ("resnet18", 2), ("vgg11", 2)])
@pytest.mark.parametrize("kw", [{}, {"wgrad_16bit": True}, {"fuse_ren_quant": False}, {"overlap_wgrad": False}, {"fuse_conv_ren": True}],
                         ids=["default", "wgrad16", "plain_norm", "one_stream", "conv_norm_chain"])
def test_every_address_in_the_call_list_belongs_to_a_tensor_the_step_keeps_alive(monkeypatch, name, N, kw):
    """The call list stores raw addresses.  A tensor behind one of them that only the caller held (labels passed as a
    temporary, a planner local) would be freed and its memory handed to the next allocation while the calls still use it."""
    record = []
    plain = step_mod._p

    def recording(t):
        if t is not None:
            record.append((weakref.ref(t), t.data_ptr(), t.numel() * t.element_size()))
        return plain(t)

    monkeypatch.setattr(step_mod, "_p", recording)
    ts = _build(getattr(nets, name)(), N, **kw)
    gc.collect()
    live = []
    for ref, _, _ in record:
        t = ref()
        if t is not None:
            st = t.untyped_storage()
            live.append((st.data_ptr(), st.data_ptr() + st.nbytes()))
    assert record and ts.calls
    for ref, ptr, nbytes in record:
        # the tensor object itself, or (for a view made on the fly) the storage it pointed into, must still exist
        assert ref() is not None or any(a <= ptr and ptr + nbytes <= b for a, b in live)


def test_operands_of_the_wrong_type_or_size_are_refused():
    """The library reads a step's tensors through raw addresses: int64 labels, a float64 image, a short parameter vector
    would be misread, so the step object refuses them when it is built."""
    from paper_2111_09389_amd.binding import LpdtError
    net, N = nets.resnet20(), 4
    H, W, C = net.in_shape
    params = nets.init_params(net, 1)
    flat = torch.from_numpy(np.concatenate([params[n].ravel() for n, _ in net.params]).astype(np.float32))
    x = torch.from_numpy(wl.images(1, N, H, W, C))
    lb = torch.from_numpy(wl.labels_uniform(2, N, net.classes))
    step_mod.TrainStep(net, N, flat, torch.zeros_like(flat), x, lb)                       # the well-formed call
    for bad in (dict(labels=lb.to(torch.int64)), dict(labels=lb[:-1]), dict(x=x.double()), dict(x=x[:, :, :-1]),
                dict(params=flat[:-4]), dict(grads=torch.zeros(flat.numel(), dtype=torch.float64)), dict(x=x.permute(0, 2, 1, 3))):
        kw = dict(params=flat, grads=torch.zeros_like(flat), x=x, labels=lb)
        kw.update(bad)
        with pytest.raises(LpdtError):
            step_mod.TrainStep(net, N, kw["params"], kw["grads"], kw["x"], kw["labels"])


@pytest.mark.parametrize("name,N", [("resnet20", 4), ("resnet18", 2), ("vgg11", 2), ("transformer_ffn", 8)])
def test_call_list_invariants(name, N):
    """Stochastic-rounding counter ranges are one per tensor (Section 3: independent rounding noise), every workspace
    placeholder was replaced by an address and a size, second-stream calls exist only with overlap, the update is last."""
    net = getattr(nets, name)()
    H, W, C = net.in_shape
    params = nets.init_params(net, 1)
    flat = torch.from_numpy(np.concatenate([params[n].ravel() for n, _ in net.params]).astype(np.float32))
    x = torch.from_numpy(wl.images(1, N, H, W, C))
    if net.classes:
        labels, upstream = torch.from_numpy(wl.labels_uniform(2, N, net.classes)), None
    else:
        labels, upstream = None, torch.from_numpy(wl.upstream_grad(3, (N,) + tuple(net.shapes[net.ops[-1][1]])))
    for overlap in (True, False):
        ts = step_mod.TrainStep(net, N, flat, torch.zeros_like(flat), x, labels, upstream, overlap_wgrad=overlap)
        sr = [c[2] for c in ts.calls if c[2] is not None]
        assert sr and len(sr) == len(set(sr)) and max(sr) < 256 and min(sr) >= 0
        for fn, args, _, side in ts.calls:
            assert "WS" not in [a for a in args if isinstance(a, str)] and "WSB" not in [a for a in args if isinstance(a, str)]
            assert overlap or not side
        real = [c for c in ts.calls if c[0] is not None]
        assert real[-1][0].__name__ == "lpdt_sgd"
        n_wgrad = sum(c[0].__name__.startswith("lpdt_qconv_bwd_weight") for c in real)
        n_conv = sum(op[0] == "conv" for op in net.ops)
        assert n_wgrad == n_conv
