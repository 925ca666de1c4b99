"""Helpers of the GPU parity tests: move seeded numpy inputs to the device, compare with the oracle."""
import numpy as np
import torch


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def assert_close(got, ref, tol, floor, what=""):
    """|got - ref| <= tol * max(|got|, |ref|, floor), elementwise."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    bound = tol * np.maximum(np.maximum(np.abs(got), np.abs(ref)), floor)
    err = np.abs(got - ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err / bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance {tol}; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r}")
