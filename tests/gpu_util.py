"""Helpers for the GPU parity tests: the tolerance metric and host<->device plumbing."""
import numpy as np
import torch

TAU = 0.05
TOL_F32 = 1e-4     # max relative error of the fp32 path (spec tolerance)
TOL_BF16 = 2e-2


def rel_err(got, ref):
    """E = max_i |got_i - ref_i| / max(|ref_i|, TAU * max|ref|): element-wise relative error with a floor
    for entries that are (near) zero by cancellation."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    scale = np.abs(ref).max()
    if scale == 0:
        return float(np.abs(got).max())
    return float((np.abs(got - ref) / np.maximum(np.abs(ref), TAU * scale)).max())


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to("cuda:0")


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()
