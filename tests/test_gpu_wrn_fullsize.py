"""Convolutions of the WRN-28-10 workload at the size `bench.py --config 5` runs them (batch 1024,
32x32 images), in the launch configurations the step uses: whole images of the forward result and
of the input gradient against the fp64 oracle (they depend on their image only), and whole weight
gradients, whose reduction runs over all 1024 images (up to a million pixels, split over the chip)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import cnn
from test_gpu_bf16_kernels import back
from test_gpu_cnn_fullsize import close, dev_normal, splitk_ws

B = 1024
# (name, H, Cin, Cout, R, stride, pad)
LAYERS = [("group1_3x3", 32, 160, 160, 3, 1, 1), ("first_block_3x3", 32, 16, 160, 3, 1, 1), ("group2_strided_3x3", 32, 160, 320, 3, 2, 1),
          ("group2_shortcut_1x1", 32, 160, 320, 1, 2, 0), ("group3_3x3", 8, 640, 640, 3, 1, 1)]


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


@pytest.mark.parametrize("name,h,ci,co,r,stride,pad", LAYERS, ids=[l[0] for l in LAYERS])
def test_wrn_convolution_at_workload_size(g, name, h, ci, co, r, stride, pad):
    import torch
    lib = K.lib()
    ho = cnn.conv_out(h, r, stride, pad)
    sh = K.ConvShape(B, h, h, ci, co, r, r, stride, pad)
    x = dev_normal(41, (B, h, h, ci))
    w = dev_normal(42, (co, r, r, ci), (2.0 / (r * r * co)) ** 0.5)
    res = dev_normal(43, (B, ho, ho, co))
    y = torch.empty(B, ho, ho, co, dtype=torch.bfloat16, device="cuda")
    ws = splitk_ws(co, r * r * max(ci, co))
    # forward with the residual the block's second convolution adds
    g.call(lib.karma_k_conv2d_fwd_add_bf16, g.ptr(x), g.ptr(w), g.ptr(res), g.ptr(y), C.byref(sh), g.stream_ptr())
    wh = back(w)
    images = (0, 517, B - 1)
    for n in images:
        close(back(y[n]), cnn.conv2d_fwd(back(x[n:n + 1]), wh, stride, pad)[0] + back(res[n]))
    del res, y

    dy = dev_normal(44, (B, ho, ho, co))
    wt_ws = torch.empty(r * r * ci * co + 8, dtype=torch.bfloat16, device="cuda")
    dx = torch.empty(B, h, h, ci, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_dgrad_bf16, g.ptr(dy), g.ptr(w), g.ptr(wt_ws), None, g.ptr(dx), C.byref(sh), g.stream_ptr())
    for n in images:
        dxo, _ = cnn.conv2d_bwd(back(x[n:n + 1]), wh, back(dy[n:n + 1]), stride, pad)
        close(back(dx[n]), dxo[0])
    del dx

    dw = torch.empty(co, r, r, ci, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_wgrad_bf16, g.ptr(dy), g.ptr(x), g.ptr(dw), g.ptr(ws), C.c_uint64(ws.numel() * 4),
           C.byref(sh), g.stream_ptr())
    dwo = np.zeros((co, r, r, ci))
    for n0 in range(0, B, 64):       # the oracle in slabs of 64 images (memory), summed in fp64
        dwo += cnn.conv2d_bwd(back(x[n0:n0 + 64]), wh, back(dy[n0:n0 + 64]), stride, pad)[1]
    close(back(dw), dwo)
