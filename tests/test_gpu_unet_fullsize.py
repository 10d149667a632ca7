"""Kernels of the fully convolutional workload at the size `bench.py --config 7` runs them (batch 16,
512x512 images, 64..1024 channels), in the launch configurations the step uses: whole images of
the forward result and of the input gradient against the fp64 oracle (they depend on their image
only), whole weight gradients (reductions over up to four million pixels, split over the chip), the
up-convolutions, the 2x2 pooling and the per-pixel softmax cross entropy over four million rows."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import cnn, unet
from test_gpu_bf16_kernels import back
from test_gpu_cnn_fullsize import close, dev_normal, splitk_ws

B = 16
IMAGES = (0, 7, B - 1)
# (name, H, Cin, Cout): 3x3, stride 1, padding 1
LAYERS = [("level0_from_image", 512, 8, 64), ("level0", 512, 64, 64), ("level1_expansive_half", 256, 128, 128),
          ("level3", 64, 512, 512), ("level4", 32, 1024, 1024)]


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


@pytest.mark.parametrize("name,h,ci,co", LAYERS, ids=[l[0] for l in LAYERS])
def test_unet_convolution_at_workload_size(g, name, h, ci, co):
    import torch
    lib = K.lib()
    sh = K.ConvShape(B, h, h, ci, co, 3, 3, 1, 1)
    x = dev_normal(51, (B, h, h, ci), zero_from_channel=1 if ci == 8 else None)
    w = dev_normal(52, (co, 3, 3, ci), (2.0 / (9 * co)) ** 0.5)
    # the expansive path's first convolution adds the result of its other half
    res = dev_normal(53, (B, h, h, co)) if name.endswith("half") else None
    y = torch.empty(B, h, h, co, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_fwd_add_bf16, g.ptr(x), g.ptr(w), g.ptr(res) if res is not None else None, g.ptr(y), C.byref(sh),
           g.stream_ptr())
    wh = back(w)
    for n in IMAGES:
        ref = cnn.conv2d_fwd(back(x[n:n + 1]), wh, 1, 1)[0]
        close(back(y[n]), ref + (back(res[n]) if res is not None else 0))
    del res, y

    dy = dev_normal(54, (B, h, h, co))
    if ci > 8:
        wt_ws = torch.empty(9 * ci * co + 8, dtype=torch.bfloat16, device="cuda")
        dx = torch.empty(B, h, h, ci, dtype=torch.bfloat16, device="cuda")
        g.call(lib.karma_k_conv2d_dgrad_bf16, g.ptr(dy), g.ptr(w), g.ptr(wt_ws), None, g.ptr(dx), C.byref(sh), g.stream_ptr())
        for n in IMAGES:
            dxo, _ = cnn.conv2d_bwd(back(x[n:n + 1]), wh, back(dy[n:n + 1]), 1, 1)
            close(back(dx[n]), dxo[0])
        del dx

    ws = splitk_ws(co, 9 * max(ci, co))
    dw = torch.empty(co, 3, 3, ci, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_wgrad_bf16, g.ptr(dy), g.ptr(x), g.ptr(dw), g.ptr(ws), C.c_uint64(ws.numel() * 4), C.byref(sh),
           g.stream_ptr())
    dwo = np.zeros((co, 3, 3, ci))
    for n in range(B):               # the oracle image by image (memory), summed in fp64
        dwo += cnn.conv2d_bwd(back(x[n:n + 1]), wh, back(dy[n:n + 1]), 1, 1)[1]
    if ci == 8:                      # channels 1..7 of the stored image are zero: so is their gradient
        assert np.all(back(dw)[..., 1:] == 0)
    close(back(dw), dwo)


@pytest.mark.parametrize("name,h,ci,co", [("to_level0", 256, 128, 64), ("to_level3", 32, 1024, 512)])
def test_unet_upconvolution_at_workload_size(g, name, h, ci, co):
    """coarse grid h x h with ci channels -> fine grid 2h x 2h with co channels, and both gradients."""
    import torch
    lib = K.lib()
    sh = K.ConvShape(B, 2 * h, 2 * h, co, ci, 2, 2, 2, 0)
    x = dev_normal(61, (B, h, h, ci))
    w = dev_normal(62, (ci, 2, 2, co), (2.0 / (4 * co)) ** 0.5)
    y = torch.empty(B, 2 * h, 2 * h, co, dtype=torch.bfloat16, device="cuda")
    wt_ws = torch.empty(4 * ci * co + 8, dtype=torch.bfloat16, device="cuda")
    ws = splitk_ws(ci, 4 * co)
    g.call(lib.karma_k_conv2d_dgrad_bf16, g.ptr(x), g.ptr(w), g.ptr(wt_ws), None, g.ptr(y), C.byref(sh), g.stream_ptr())
    wh = back(w)
    for n in IMAGES:
        close(back(y[n]), unet.upconv2x2_fwd(back(x[n:n + 1]), wh)[0])
    del y
    dy = dev_normal(63, (B, 2 * h, 2 * h, co))
    dx = torch.empty(B, h, h, ci, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_fwd_bf16, g.ptr(dy), g.ptr(w), g.ptr(dx), C.byref(sh), g.stream_ptr())
    dw = torch.empty(ci, 2, 2, co, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_conv2d_wgrad_bf16, g.ptr(x), g.ptr(dy), g.ptr(dw), g.ptr(ws), C.c_uint64(ws.numel() * 4), C.byref(sh),
           g.stream_ptr())
    dwo = np.zeros((ci, 2, 2, co))
    for n in range(B):
        dxo, dwn = unet.upconv2x2_bwd(back(x[n:n + 1]), wh, back(dy[n:n + 1]))
        dwo += dwn
        if n in IMAGES:
            close(back(dx[n]), dxo[0])
    close(back(dw), dwo)


def test_unet_pooling_at_workload_size(g):
    import torch
    h, c = 512, 64
    x = torch.relu(dev_normal(71, (B, h, h, c)))
    dy = dev_normal(72, (B, h // 2, h // 2, c))
    y = torch.empty(B, h // 2, h // 2, c, dtype=torch.bfloat16, device="cuda")
    dx = torch.empty(B, h, h, c, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_maxpool2_fwd_bf16, g.ptr(x), g.ptr(y), B, h, h, c, g.stream_ptr())
    g.call(K.lib().karma_k_maxpool2_bwd_bf16, g.ptr(x), g.ptr(dy), g.ptr(dx), B, h, h, c, g.stream_ptr())
    for n in IMAGES:
        yo, arg = cnn.maxpool_fwd(back(x[n:n + 1]), 2, 2, 0)
        assert np.array_equal(back(y[n]), yo[0])
        assert np.array_equal(back(dx[n]), cnn.maxpool_bwd(back(dy[n:n + 1]), arg, (1, h, h, c), 2, 2, 0)[0])


def test_unet_pixel_cross_entropy_at_workload_size(g):
    import torch
    rows, cols = B * 512 * 512, 8
    z = dev_normal(81, (rows, cols), 2.0)
    z[:, 2:] = -30000.0
    lab = torch.from_numpy(si_labels(rows)).cuda()
    zin = z.clone()
    rowloss = torch.empty(rows, dtype=torch.float32, device="cuda")
    scale = 1.0 / rows
    g.call(K.lib().karma_k_softmax_ce_bf16, g.ptr(z), g.ptr(lab), g.ptr(rowloss), rows, cols, C.c_float(scale), g.stream_ptr())
    pick = np.concatenate([np.arange(0, 4096), np.arange(rows // 2, rows // 2 + 4096), np.arange(rows - 4096, rows)])
    zi = back(zin[pick])
    lb = lab[pick].cpu().numpy()
    m = zi.max(axis=1, keepdims=True)
    lse = (m + np.log(np.exp(zi - m).sum(axis=1, keepdims=True)))[:, 0]
    want = lse - zi[np.arange(len(pick)), lb]
    p = np.exp(zi - lse[:, None])
    p[np.arange(len(pick)), lb] -= 1
    assert np.all(np.abs(rowloss[pick].cpu().numpy() - want) <= 1e-5 * (1 + np.abs(want)))
    got = back(z[pick])
    assert np.all(np.abs(got - p * scale) <= (2.0 ** -8 * np.abs(p) + 1e-6) * scale)
    # the mean loss over all rows against the fp64 sum of the kernel's own per-row values (the reduction kernel)
    total = torch.empty(1, dtype=torch.float32, device="cuda")
    part = torch.empty(1024, dtype=torch.float32, device="cuda")
    g.call(K.lib().karma_k_sum_f32, g.ptr(rowloss), g.ptr(total), g.ptr(part), C.c_uint64(rows), C.c_float(scale), g.stream_ptr())
    assert abs(float(total[0]) - rowloss.double().sum().item() * scale) <= 1e-5 * abs(float(total[0]))


def si_labels(rows):
    import synth_inputs as si
    return si.randint(82, (rows,), 2).astype(np.int32)
