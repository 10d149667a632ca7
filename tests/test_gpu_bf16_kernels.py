"""bf16 kernels against the oracle, element by element, at sizes that span several
tiles and ragged tails.  Inputs are rounded to bf16 first (that is what the device
holds); the oracle then works in fp64.  Tolerances: a bf16 result carries one
round-to-nearest-even (relative error <= 2^-9 per element, so relative L2 <= 2^-8 with
margin for fp32 accumulation); an fp32 result only carries accumulation error (1e-4)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import nn
import synth_inputs as si

TOL_BF16 = 2.0 ** -8
TOL_F32 = 1e-4


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def bf(a):
    """Round to bf16, return (float64 view of rounded values, torch bf16 device tensor)."""
    import torch
    r = nn.bf16_round(np.asarray(a, dtype=np.float32))
    return r.astype(np.float64), torch.from_numpy(r).to(torch.bfloat16).cuda()


def back(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("m,n,k", [(256, 256, 128), (200, 136, 72), (4, 8, 8), (384, 520, 1032), (1024, 1024, 1024)])
@pytest.mark.parametrize("flags", [0, K.GEMM_A_STRIDED, K.GEMM_B_STRIDED, K.GEMM_A_STRIDED | K.GEMM_B_STRIDED])
def test_gemm_layouts(g, m, n, k, flags):
    import torch
    a, ad = bf(si.normal(1, (m, k)))
    b, bd = bf(si.normal(2, (n, k)))
    ref = a @ b.T
    if flags & K.GEMM_A_STRIDED:
        ad = ad.t().contiguous()
    if flags & K.GEMM_B_STRIDED:
        bd = bd.t().contiguous()
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c), None, None, m, n, k, flags, g.stream_ptr())
    assert g.rel_l2(back(c), ref) <= TOL_BF16
    c32 = torch.empty(m, n, dtype=torch.float32, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c32), None, None, m, n, k, flags | K.GEMM_OUT_F32,
           g.stream_ptr())
    assert g.rel_l2(back(c32), ref) <= TOL_F32
    # element-wise bound as well: no single entry may be off by more than a few ulps of bf16
    scale = np.abs(a) @ np.abs(b.T)
    assert np.all(np.abs(back(c32) - ref) <= 1e-5 * scale + 1e-30)


def test_gemm_epilogues(g):
    import torch
    m, n, k = 200, 136, 72
    a, ad = bf(si.normal(3, (m, k)))
    b, bd = bf(si.normal(4, (n, k)))
    bias, biasd = bf(si.normal(5, (n,)))
    res, resd = bf(si.normal(6, (m, n)))
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c), g.ptr(biasd), g.ptr(resd), m, n, k, 0, g.stream_ptr())
    assert g.rel_l2(back(c), a @ b.T + bias + res) <= TOL_BF16
    acc0 = si.normal(7, (m, n)).astype(np.float32)
    c32 = torch.from_numpy(acc0).cuda()
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c32), None, None, m, n, k,
           K.GEMM_OUT_F32 | K.GEMM_ACCUMULATE, g.stream_ptr())
    assert g.rel_l2(back(c32), acc0.astype(np.float64) + a @ b.T) <= TOL_F32


def test_gemm_rejects_bad_shapes(g):
    import torch
    t = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    lib = K.lib()
    assert lib.karma_k_gemm_bf16(g.ptr(t), g.ptr(t), g.ptr(t), None, None, 8, 8, 12, 0, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_bf16(g.ptr(t), g.ptr(t), g.ptr(t), None, None, 6, 8, 8, K.GEMM_A_STRIDED, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_bf16(g.ptr(t), g.ptr(t), g.ptr(t), None, None, 8, 8, 8, K.GEMM_ACCUMULATE, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_bf16(None, g.ptr(t), g.ptr(t), None, None, 8, 8, 8, 0, g.stream_ptr()) == K.E_INVAL
