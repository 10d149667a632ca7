"""Kernels of the convolutional workload against the oracle, element by element: implicit
GEMM convolution (forward, input gradient, weight gradient), batch normalisation, ReLU
mask, pooling.  Inputs are rounded to bf16 first (that is what the device holds); the
oracle works in fp64.  A bf16 result carries one round-to-nearest-even: relative L2
<= 2^-8; fp32 per-channel sums: 1e-4 (1e-3 where they are differences of large sums)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import cnn
import synth_inputs as si
from test_gpu_bf16_kernels import back, bf

TOL = 2.0 ** -8


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def shape(n, h, w, ci, co, r, stride, pad):
    return K.ConvShape(n, h, w, ci, co, r, r, stride, pad)


CONV_CASES = [
    (2, 14, 14, 64, 64, 3, 1, 1),      # the 3x3 of a bottleneck
    (3, 9, 7, 24, 40, 3, 1, 1),        # ragged: taps straddle k-tiles, rows and columns leave tails
    (2, 16, 16, 128, 72, 3, 2, 1),     # strided 3x3
    (2, 15, 13, 16, 32, 3, 2, 1),      # strided, odd sizes
    (4, 12, 12, 64, 256, 1, 1, 0),     # 1x1: a plain GEMM
    (2, 14, 14, 256, 136, 1, 2, 0),    # strided 1x1 (projection shortcut)
    (2, 32, 32, 8, 64, 7, 2, 3),       # the stem: 3 channels stored as 8
    (1, 5, 5, 8, 8, 3, 1, 1),          # one tile, mostly padding
    # large enough for the direct-to-LDS kernel with a gathered operand (>= 1024 pixels, >= 128 output channels)
    (4, 20, 20, 160, 136, 3, 1, 1),    # forward and input gradient, every dimension leaves a tail
    (4, 18, 18, 128, 136, 3, 2, 1),    # input gradient of a strided 3x3 (three taps in four fall between pixels)
    (16, 16, 16, 256, 136, 1, 2, 0),   # strided 1x1, both directions
    (2, 33, 31, 128, 128, 3, 1, 1),    # odd image sizes
    (3, 24, 24, 136, 264, 5, 1, 2),    # 5x5 taps, two tile columns
    (8, 24, 24, 128, 136, 3, 1, 1),    # weight gradient over 4608 pixels: the gathered second operand
    (32, 32, 32, 128, 160, 3, 2, 1),   # the same, strided, 8192 pixels
]


@pytest.mark.parametrize("n,h,w,ci,co,r,stride,pad", CONV_CASES)
def test_conv_forward_and_gradients(g, n, h, w, ci, co, r, stride, pad):
    import torch
    x, xd = bf(si.normal(1, (n, h, w, ci)))
    if ci == 8 and r == 7:
        x[..., 3:] = 0
        xd = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).cuda()
    wt, wd = bf(si.normal(2, (co, r, r, ci), 0.2))
    sh = shape(n, h, w, ci, co, r, stride, pad)
    ho, wo = cnn.conv_out(h, r, stride, pad), cnn.conv_out(w, r, stride, pad)
    lib = K.lib()
    y = torch.empty(n, ho, wo, co, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_fwd_bf16, g.ptr(xd), g.ptr(wd), g.ptr(y), C.byref(sh), g.stream_ptr())
    ref = cnn.conv2d_fwd(x, wt, stride, pad)
    assert g.rel_l2(back(y), ref) <= TOL
    assert np.all(np.abs(back(y) - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-4 * np.abs(ref).max())

    dy, dyd = bf(si.normal(3, (n, ho, wo, co)))
    add, addd = bf(si.normal(4, (n, h, w, ci)))
    dxo, dwo = cnn.conv2d_bwd(x, wt, dy, stride, pad)
    wt_ws = torch.empty(r * r * ci * co + 8, dtype=torch.bfloat16, device="cuda")
    for with_add in (False, True):
        dx = torch.full((n, h, w, ci), 7.0, dtype=torch.bfloat16, device="cuda")
        g.call(lib.karma_k_conv2d_dgrad_bf16, g.ptr(dyd), g.ptr(wd), g.ptr(wt_ws), g.ptr(addd) if with_add else None,
               g.ptr(dx), C.byref(sh), g.stream_ptr())
        assert g.rel_l2(back(dx), dxo + (add if with_add else 0)) <= TOL, with_add
    ws = torch.empty(16 * co * r * r * ci, dtype=torch.float32, device="cuda")
    res = []
    for use_ws in (False, True):
        dw = torch.full((co, r, r, ci), 7.0, dtype=torch.bfloat16, device="cuda")
        g.call(lib.karma_k_conv2d_wgrad_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(dw), g.ptr(ws) if use_ws else None,
               C.c_uint64(ws.numel() * 4 if use_ws else 0), C.byref(sh), g.stream_ptr())
        assert g.rel_l2(back(dw), dwo) <= TOL, use_ws
        res.append(back(dw))
    # twice the same call: bit-identical (no atomics anywhere)
    dw2 = torch.empty(co, r, r, ci, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_wgrad_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(dw2), g.ptr(ws), C.c_uint64(ws.numel() * 4),
           C.byref(sh), g.stream_ptr())
    assert np.array_equal(back(dw2), res[1])


def test_conv_rejects_bad_shapes(g):
    import torch
    t = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    lib = K.lib()
    for sh in (shape(1, 4, 4, 3, 8, 3, 1, 1), shape(1, 4, 4, 8, 12, 3, 1, 1), shape(1, 2, 2, 8, 8, 7, 1, 0), shape(1, 4, 4, 8, 8, 3, 0, 1)):
        assert lib.karma_k_conv2d_fwd_bf16(g.ptr(t), g.ptr(t), g.ptr(t), C.byref(sh), g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_conv2d_fwd_bf16(None, g.ptr(t), g.ptr(t), C.byref(shape(1, 4, 4, 8, 8, 3, 1, 1)), g.stream_ptr()) == K.E_INVAL


@pytest.mark.parametrize("rows,c", [(1000, 64), (257, 24), (64, 2048), (5000, 128), (3, 8), (70000, 64), (300, 2304)])
@pytest.mark.parametrize("relu,with_add", [(0, False), (1, False), (1, True)])
def test_batchnorm(g, rows, c, relu, with_add):
    import torch
    x, xd = bf(si.normal(5, (rows, c)) * (1.0 + 0.1 * np.arange(c)[None, :] % 3) + 0.5 * (np.arange(c)[None, :] % 5 - 2))
    gam, gd = bf(1.0 + si.normal(6, (c,), 0.2))
    bet, bd = bf(si.normal(7, (c,), 0.2))
    add, addd = bf(si.normal(8, (rows, c)))
    lib = K.lib()
    lib.karma_k_batchnorm_ws_bytes.restype = C.c_uint64
    ws = torch.empty(lib.karma_k_batchnorm_ws_bytes(rows, c) // 4, dtype=torch.float32, device="cuda")
    stats = torch.empty(2, c, dtype=torch.float32, device="cuda")
    y = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_batchnorm_fwd_bf16, g.ptr(xd), g.ptr(gd), g.ptr(bd), g.ptr(addd) if with_add else None, g.ptr(y),
           g.ptr(stats), g.ptr(ws), rows, c, relu, g.stream_ptr())
    x4 = x.reshape(1, 1, rows, c)
    yo, cache = cnn.batchnorm_fwd(x4, gam, bet)
    yo = yo.reshape(rows, c) + (add if with_add else 0)
    if relu:
        yo = np.maximum(yo, 0)
    st = stats.cpu().numpy().astype(np.float64)
    assert g.rel_l2(st[0], x.mean(axis=0)) <= 1e-4 and g.rel_l2(st[1], cache[1]) <= 1e-4
    assert g.rel_l2(back(y), yo) <= TOL
    ratio = g.elem_ratio(back(y), yo, 1, 1e-3, axis=0)
    assert ratio <= 1, ratio

    dy, dyd = bf(si.normal(9, (rows, c)))
    # the ReLU decision is the kernel's own (its forward output, add excluded): both sides use it
    if relu and not with_add:
        dym = dy * (back(y) > 0)
    elif relu:
        y_plain = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
        g.call(lib.karma_k_batchnorm_fwd_bf16, g.ptr(xd), g.ptr(gd), g.ptr(bd), None, g.ptr(y_plain), g.ptr(stats), g.ptr(ws),
               rows, c, 1, g.stream_ptr())
        dym = dy * (back(y_plain) > 0)
    else:
        dym = dy
    dxo, dgo, dbo = cnn.batchnorm_bwd(dym.reshape(1, 1, rows, c), gam, cache)
    dx = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
    dg = torch.empty(c, dtype=torch.float32, device="cuda"); db = torch.empty(c, dtype=torch.float32, device="cuda")
    g.call(lib.karma_k_batchnorm_bwd_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), g.ptr(bd), relu, g.ptr(dx),
           g.ptr(dg), g.ptr(db), g.ptr(ws), rows, c, g.stream_ptr())
    scale = np.sqrt(rows)
    assert np.all(np.abs(dg.cpu().numpy() - dgo) <= 1e-3 * scale + 1e-4 * np.abs(dgo))
    assert np.all(np.abs(db.cpu().numpy() - dbo) <= 1e-3 * scale + 1e-4 * np.abs(dbo))
    assert g.rel_l2(back(dx), dxo.reshape(rows, c)) <= (TOL if rows > 3 else 0.1)
    if rows > 3:    # per element, scaled by the channel's size (dx is dy minus two per-channel sums)
        ratio = g.elem_ratio(back(dx), dxo.reshape(rows, c), 1, 1e-3, axis=0)
        assert ratio <= 1, ratio


def test_relu_mask(g):
    import torch
    y, yd = bf(np.maximum(si.normal(10, (4096 + 8,)), 0))
    dy, dyd = bf(si.normal(11, (4096 + 8,)))
    dz = torch.empty_like(dyd)
    g.call(K.lib().karma_k_relu_mask_bwd_bf16, g.ptr(dyd), g.ptr(yd), g.ptr(dz), C.c_uint64(4096 + 8), g.stream_ptr())
    assert np.array_equal(back(dz), dy * (y > 0))


@pytest.mark.parametrize("n,h,w,c", [(2, 16, 16, 64), (3, 7, 6, 8), (1, 1, 1, 8), (2, 9, 12, 24)])
def test_maxpool(g, n, h, w, c):
    import torch
    # few distinct values: plenty of ties inside windows
    x, xd = bf(np.round(si.normal(12, (n, h, w, c)) * 2) / 2)
    yo, arg = cnn.maxpool_fwd(x)
    y = torch.empty(*yo.shape, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_maxpool_fwd_bf16, g.ptr(xd), g.ptr(y), n, h, w, c, g.stream_ptr())
    assert np.array_equal(back(y), yo)
    dy, dyd = bf(si.normal(13, yo.shape))
    dx = torch.empty(n, h, w, c, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_maxpool_bwd_bf16, g.ptr(xd), g.ptr(dyd), g.ptr(dx), n, h, w, c, g.stream_ptr())
    ref = cnn.maxpool_bwd(dy, arg, x.shape)
    assert np.all(np.abs(back(dx) - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-30)
    assert np.array_equal(back(dx) != 0, ref != 0)


@pytest.mark.parametrize("n,hw,c", [(64, 49, 2048), (3, 5, 8), (2, 1, 16)])
def test_avgpool(g, n, hw, c):
    import torch
    x, xd = bf(si.normal(14, (n, hw, c)))
    y = torch.empty(n, c, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_avgpool_fwd_bf16, g.ptr(xd), g.ptr(y), n, hw, c, g.stream_ptr())
    assert g.rel_l2(back(y), x.mean(axis=1)) <= TOL
    dy, dyd = bf(si.normal(15, (n, c)))
    dx = torch.empty(n, hw, c, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_avgpool_bwd_bf16, g.ptr(dyd), g.ptr(dx), n, hw, c, g.stream_ptr())
    assert g.rel_l2(back(dx), np.broadcast_to(dy[:, None, :] / hw, (n, hw, c))) <= TOL
