"""Convolution, batch normalisation and pooling kernels at the sizes of the ResNet-200-shaped
workload (batch 64, 224x224 images), in the launch configurations the step uses (split
reductions with the step's workspace sizes).  The fp64 oracle computes whole images (a
convolution's output and input gradient for one image depend on that image only), whole
weight gradients where the reduction is short enough, and whole batch normalisations."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import cnn
import synth_inputs as si
from test_gpu_bf16_kernels import back

TOL = 2.0 ** -8
B = 64


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def dev_normal(seed, shape, std=1.0, zero_from_channel=None):
    import torch
    # tensors of hundreds of millions of elements repeat a block of 2^25 draws (drawing them all takes longer
    # than everything else in these tests; the period is far longer than any reduction's reach in one image)
    n = int(np.prod(shape))
    a = si.normal(seed, (min(n, 1 << 25),), std).astype(np.float32)
    a = (np.resize(a, n) if n > a.size else a).reshape(shape)
    if zero_from_channel is not None:
        a[..., zero_from_channel:] = 0
    return torch.from_numpy(a).to(torch.bfloat16).cuda()


def splitk_ws(m, n):
    """fp32 workspace the step hands to a product with an m x n result (up to 256 partial results)."""
    import torch
    tiles = ((m + 127) // 128) * ((n + 127) // 128)
    splits = min(256, (512 + tiles - 1) // tiles)
    return torch.empty(splits * m * n, dtype=torch.float32, device="cuda")


def close(got, ref, rows_scale=None):
    """Relative L2 of one bf16 rounding, and every element within two bf16 ulps of its value plus a
    small share of the tensor's largest entry (sums of many terms cancel)."""
    assert np.linalg.norm(got - ref) <= TOL * np.linalg.norm(ref), np.linalg.norm(got - ref) / np.linalg.norm(ref)
    worst = np.abs(got - ref) - 2.0 ** -7 * np.abs(ref) - 2e-3 * np.abs(ref).max()
    assert worst.max() <= 0, worst.max()


# (name, H, Cin, Cout, R, stride, pad): the stem, the first stage's 3x3 and 1x1s, the strided
# projection into the second stage, a strided 3x3, the last stage's 3x3 and 1x1s
LAYERS = [("stem", 224, 8, 64, 7, 2, 3), ("s1_3x3", 56, 64, 64, 3, 1, 1), ("s1_expand", 56, 64, 256, 1, 1, 0),
          ("s1_reduce", 56, 256, 64, 1, 1, 0), ("s2_projection", 56, 256, 512, 1, 2, 0), ("s2_3x3_strided", 56, 128, 128, 3, 2, 1),
          ("s4_3x3", 7, 512, 512, 3, 1, 1), ("s4_expand", 7, 512, 2048, 1, 1, 0), ("s4_reduce", 7, 2048, 512, 1, 1, 0)]


@pytest.mark.parametrize("name,h,ci,co,r,stride,pad", LAYERS, ids=[l[0] for l in LAYERS])
def test_convolution_at_workload_size_whole_images(g, name, h, ci, co, r, stride, pad):
    import torch
    lib = K.lib()
    ho = cnn.conv_out(h, r, stride, pad)
    sh = K.ConvShape(B, h, h, ci, co, r, r, stride, pad)
    x = dev_normal(21, (B, h, h, ci), zero_from_channel=3 if name == "stem" else None)
    w = dev_normal(22, (co, r, r, ci), (2.0 / (r * r * co)) ** 0.5)
    y = torch.empty(B, ho, ho, co, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_fwd_bf16, g.ptr(x), g.ptr(w), g.ptr(y), C.byref(sh), g.stream_ptr())
    wh = back(w)
    images = (0, 37, B - 1)
    for n in images:
        close(back(y[n]), cnn.conv2d_fwd(back(x[n:n + 1]), wh, stride, pad)[0])

    dy = dev_normal(23, (B, ho, ho, co))
    add = dev_normal(24, (B, h, h, ci))
    wt_ws = torch.empty(r * r * ci * co + 8, dtype=torch.bfloat16, device="cuda")
    dx = torch.empty(B, h, h, ci, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_dgrad_bf16, g.ptr(dy), g.ptr(w), g.ptr(wt_ws), g.ptr(add), g.ptr(dx), C.byref(sh), g.stream_ptr())
    for n in images:
        dxo, _ = cnn.conv2d_bwd(back(x[n:n + 1]), wh, back(dy[n:n + 1]), stride, pad)
        close(back(dx[n]), dxo[0] + back(add[n]))

    # the weight gradient reduces over all 64 images: the whole result against the oracle
    ws = splitk_ws(co, r * r * ci)
    dw = torch.empty(co, r, r, ci, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_wgrad_bf16, g.ptr(dy), g.ptr(x), g.ptr(dw), g.ptr(ws), C.c_uint64(ws.numel() * 4),
           C.byref(sh), g.stream_ptr())
    dwo = np.zeros((co, r, r, ci))
    for n0 in range(0, B, 8):        # the oracle in slabs of 8 images (memory), summed in fp64
        dwo += cnn.conv2d_bwd(back(x[n0:n0 + 8]), wh, back(dy[n0:n0 + 8]), stride, pad)[1]
    close(back(dw), dwo)
    if name == "stem":
        assert np.all(back(dw)[..., 3:] == 0)


@pytest.mark.parametrize("rows,c", [(B * 112 * 112, 64), (B * 56 * 56, 256), (B * 14 * 14, 1024), (B * 7 * 7, 2048)])
def test_batchnorm_at_workload_size(g, rows, c):
    import torch
    lib = K.lib()
    lib.karma_k_batchnorm_ws_bytes.restype = C.c_uint64
    xd = dev_normal(31, (rows, c))
    xd = (xd.float() * (1.0 + 0.25 * (torch.arange(c, device="cuda") % 4)) + 0.5 * (torch.arange(c, device="cuda") % 5 - 2)).to(torch.bfloat16)
    gd = (1.0 + 0.2 * dev_normal(32, (c,)).float()).to(torch.bfloat16)
    bd = (0.2 * dev_normal(33, (c,)).float()).to(torch.bfloat16)
    addd = dev_normal(34, (rows, c))
    ws = torch.empty(lib.karma_k_batchnorm_ws_bytes(rows, c) // 4, dtype=torch.float32, device="cuda")
    stats = torch.empty(2, c, dtype=torch.float32, device="cuda")
    y = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
    y_plain = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_batchnorm_fwd_bf16, g.ptr(xd), g.ptr(gd), g.ptr(bd), None, g.ptr(y_plain), g.ptr(stats), g.ptr(ws),
           rows, c, 1, g.stream_ptr())
    g.call(lib.karma_k_batchnorm_fwd_bf16, g.ptr(xd), g.ptr(gd), g.ptr(bd), g.ptr(addd), g.ptr(y), g.ptr(stats), g.ptr(ws),
           rows, c, 1, g.stream_ptr())
    x, gam, bet = back(xd), back(gd), back(bd)
    n, cache = cnn.batchnorm_fwd(x.reshape(1, 1, rows, c), gam, bet)
    n = n.reshape(rows, c)
    st = stats.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(st[0] - x.mean(axis=0)) <= 1e-4 * (np.abs(x.mean(axis=0)) + x.std(axis=0)))
    assert np.all(np.abs(st[1] - cache[1]) <= 1e-4 * cache[1])
    close(back(y), np.maximum(n + back(addd), 0))
    got = back(y_plain)
    close(got, np.maximum(n, 0))
    del y, addd
    dyd = dev_normal(35, (rows, c))
    dym = back(dyd) * (got > 0)          # the ReLU decision is the kernel's own forward output
    dxo, dgo, dbo = cnn.batchnorm_bwd(dym.reshape(1, 1, rows, c), gam, cache)
    dx = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
    dg = torch.empty(c, dtype=torch.float32, device="cuda")
    db = torch.empty(c, dtype=torch.float32, device="cuda")
    g.call(lib.karma_k_batchnorm_bwd_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), g.ptr(bd), 1, g.ptr(dx),
           g.ptr(dg), g.ptr(db), g.ptr(ws), rows, c, g.stream_ptr())
    scale = np.sqrt(rows)
    assert np.all(np.abs(dg.cpu().numpy() - dgo) <= 1e-3 * scale + 1e-4 * np.abs(dgo))
    assert np.all(np.abs(db.cpu().numpy() - dbo) <= 1e-3 * scale + 1e-4 * np.abs(dbo))
    close(back(dx), dxo.reshape(rows, c))


def test_maxpool_at_workload_size(g):
    import torch
    xd = dev_normal(41, (B, 112, 112, 64))
    xd = (torch.round(xd.float() * 4) / 4).to(torch.bfloat16)        # ties inside windows
    x = back(xd)
    yo, arg = cnn.maxpool_fwd(x)
    y = torch.empty(B, 56, 56, 64, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_maxpool_fwd_bf16, g.ptr(xd), g.ptr(y), B, 112, 112, 64, g.stream_ptr())
    assert np.array_equal(back(y), yo)
    dyd = dev_normal(42, (B, 56, 56, 64))
    dx = torch.empty(B, 112, 112, 64, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_maxpool_bwd_bf16, g.ptr(xd), g.ptr(dyd), g.ptr(dx), B, 112, 112, 64, g.stream_ptr())
    ref = cnn.maxpool_bwd(back(dyd), arg, x.shape)
    got = back(dx)
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref))
    assert np.array_equal(got != 0, ref != 0)
