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
