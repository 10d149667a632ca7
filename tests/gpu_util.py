"""Helpers for the GPU parity tests: torch is used for device memory only."""
import ctypes as C

import numpy as np
import torch

import paper_2008_11421_amd as K


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def ptr(t):
    return C.c_void_p(t.data_ptr())


def stream_ptr():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def call(fn, *args):
    st = fn(*args)
    assert st == 0, "status %d" % st
    torch.cuda.synchronize()


def elem_ratio(got, ref, ulps, row_share, axis=-1):
    """Element-wise bound beside the relative L2 norm (which one bad row among thousands passes):
    the largest |got - ref| / (ulps * 2^-8 * |ref| + row_share * rms of ref along `axis`).
    `ulps` counts bf16 roundings of the element itself, `row_share` bounds what cancellation inside a
    sum leaves (errors of the terms do not shrink with the result).  A value <= 1 passes."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    row = np.sqrt(np.mean(ref * ref, axis=axis, keepdims=True))
    whole = np.sqrt(np.mean(ref * ref))
    bound = ulps * 2.0 ** -8 * np.abs(ref) + row_share * row + 1e-6 * whole + 1e-30     # (rows that are exactly zero)
    return float(np.max(np.abs(got - ref) / bound))
