"""The GEMM entry point that allocates nothing (its split-reduction workspace is a fixed device
array inside the library) against the entry point that takes the caller's workspace: same bits, on
two calls in a row, the second with a smaller product, so that what the first call left in the
shared array is seen not to matter."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
import synth_inputs as si
from test_gpu_bf16_kernels import TOL_BF16, back, bf

STATIC_WS_BYTES = 64 << 20


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def test_static_workspace_gemm_matches_the_workspace_entry_point(g):
    import torch
    lib = K.lib()
    ws = torch.empty(STATIC_WS_BYTES // 4, dtype=torch.float32, device="cuda")
    # weight-gradient shapes (both operands strided, long reduction: the split path), then a smaller
    # ragged one, then one that takes no split at all
    for (m, n, k, flags) in ((1024, 1024, 32768, 3), (200, 136, 4096 + 72, 0), (512, 256, 8192, 3), (256, 256, 128, 0)):
        a, ad = bf(si.normal(71, (m, k)))
        b, bd = bf(si.normal(72, (n, k)))
        ref = a @ b.T
        if flags & K.GEMM_A_STRIDED:
            ad = ad.t().contiguous()
        if flags & K.GEMM_B_STRIDED:
            bd = bd.t().contiguous()
        want = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
        ws.fill_(float("nan"))
        g.call(lib.karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(want), None, None, m, n, k, flags, g.ptr(ws),
               C.c_uint64(STATIC_WS_BYTES), g.stream_ptr())
        got = torch.full((m, n), 7.0, dtype=torch.bfloat16, device="cuda")
        g.call(lib.karma_k_gemm_bf16_static_ws, g.ptr(ad), g.ptr(bd), g.ptr(got), None, None, m, n, k, flags, g.stream_ptr())
        assert torch.equal(got, want), (m, n, k)
        assert g.rel_l2(back(got), ref) <= TOL_BF16, (m, n, k)
    # a result too large for two partial results in the array is refused, nothing is launched
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    assert lib.karma_k_gemm_bf16_static_ws(g.ptr(t), g.ptr(t), g.ptr(t), None, None, 4096, 4096, 8, 0, g.stream_ptr()) == K.E_OOM
    assert lib.karma_k_gemm_bf16_static_ws(None, g.ptr(t), g.ptr(t), None, None, 8, 8, 8, 0, g.stream_ptr()) == K.E_INVAL
