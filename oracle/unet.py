"""Numerical oracle for the fully convolutional network (TEST INFRASTRUCTURE ONLY).

The U-Net row of KARMA's Table III and the model Sec. III-F.3 names for connections from
the contracting to the expansive path, composed from the plain fp64 layer definitions of
`oracle/cnn.py` (Sec. III-C: convolution, batch normalisation, ReLU, pooling, softmax) plus
the one layer they lack, the 2x2 up-convolution, written out from its definition below.
Nothing is blocked, fused or reordered.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this file; the product library never does and shares no code
with it.

The paper names the model and its dataset (30 grey-scale 512x512 sections, two classes)
and nothing more.  Readings used here (the HIP path uses the same ones): `depth` levels of
contraction; level l works on width << l channels at image >> l pixels a side.  A level is
two 3x3 convolutions (padding 1, so that the contracting path's tensors need no cropping
before they are concatenated), each followed by batch normalisation (training mode over
(N, H, W), biased variance, eps 1e-5) and ReLU, as current implementations of the model do;
convolutions and up-convolutions carry no bias.  Contracting level l >= 1 starts with 2x2
max pooling (stride 2) of the level above; expansive level l starts with the 2x2 stride-2
up-convolution of the level below to width << l channels, concatenated BEHIND the
contracting path's output of the same level (channels [0, C) = that output, [C, 2C) = the
up-convolution); a 1x1 convolution with bias to the classes and the mean over all pixels of
the cross entropy close the network.
"""
import numpy as np

from oracle.cnn import batchnorm_bwd, batchnorm_fwd, conv2d_bwd, conv2d_fwd, maxpool_bwd, maxpool_fwd
from oracle.nn import cross_entropy_fwd_bwd, linear_bwd, linear_fwd

LEVEL_TENSORS = ("w1", "g1", "b1", "w2", "g2", "b2")       # contracting levels and the lowest one
UP_TENSORS = ("wu",) + LEVEL_TENSORS                        # expansive levels (w1 reads 2C channels)


def upconv2x2_fwd(x, w):
    """2x2 up-convolution with stride 2: every input pixel spreads over its own 2x2 patch of the
    output, y[n, 2h+a, 2w+b, co] = sum_ci x[n,h,w,ci] * w[ci,a,b,co].  x [N,H,W,Ci], w [Ci,2,2,Co]."""
    n, h, wd, _ = x.shape
    co = w.shape[3]
    y = np.zeros((n, 2 * h, 2 * wd, co))
    for a in range(2):
        for b in range(2):
            y[:, a::2, b::2, :] = x @ w[:, a, b, :]
    return y


def upconv2x2_bwd(x, w, dy):
    """Gradients of upconv2x2_fwd: dx (shape of x) and dw (shape of w)."""
    dx = np.zeros_like(x, dtype=np.float64)
    dw = np.zeros_like(w, dtype=np.float64)
    for a in range(2):
        for b in range(2):
            g = dy[:, a::2, b::2, :]
            dx += g @ w[:, a, b, :].T
            dw[:, a, b, :] = x.reshape(-1, x.shape[3]).T @ g.reshape(-1, g.shape[3])   # sum over (n, h, w)
    return dx, dw


def double_conv_fwd(p, x):
    c1 = conv2d_fwd(x, p["w1"], 1, 1)
    n1, bc1 = batchnorm_fwd(c1, p["g1"], p["b1"])
    a1 = np.maximum(n1, 0)
    c2 = conv2d_fwd(a1, p["w2"], 1, 1)
    n2, bc2 = batchnorm_fwd(c2, p["g2"], p["b2"])
    return np.maximum(n2, 0), (x, n1, a1, bc1, n2, bc2)


def double_conv_bwd(p, cache, dy):
    x, n1, a1, bc1, n2, bc2 = cache
    g = {}
    dc2, g["g2"], g["b2"] = batchnorm_bwd(dy * (n2 > 0), p["g2"], bc2)
    da1, g["w2"] = conv2d_bwd(a1, p["w2"], dc2, 1, 1)
    dc1, g["g1"], g["b1"] = batchnorm_bwd(da1 * (n1 > 0), p["g1"], bc1)
    dx, g["w1"] = conv2d_bwd(x, p["w1"], dc1, 1, 1)
    return dx, g


def unet_step(params, images, labels):
    """One training step: loss and gradients.  params: down: depth + 1 dicts (LEVEL_TENSORS; the
    last is the lowest level), up: depth dicts (UP_TENSORS), the first being the deepest expansive
    level; head {w [classes, C], bias [classes]}.  images [N,S,S,Cimg]; labels [N,S,S] ints."""
    depth = len(params["up"])
    outs, caches, pools = [], [], []
    x = images
    for l, p in enumerate(params["down"]):
        if l:
            x, arg = maxpool_fwd(x, 2, 2, 0)
            pools.append((arg, outs[-1].shape))
        x, c = double_conv_fwd(p, x)
        outs.append(x)
        caches.append(c)
    up_caches = []
    for j, p in enumerate(params["up"]):
        l = depth - 1 - j
        u = upconv2x2_fwd(x, p["wu"])
        cat = np.concatenate([outs[l], u], axis=3)
        below = x
        x, c = double_conv_fwd(p, cat)
        up_caches.append((below, c))
    hd = params["head"]
    n, s, _, ch = x.shape
    logits = linear_fwd(x.reshape(-1, ch), hd["w"], hd["bias"])
    loss, dlogits = cross_entropy_fwd_bwd(logits, labels.reshape(-1))
    grads = {"down": [None] * (depth + 1), "up": [None] * depth, "head": {}}
    dflat, grads["head"]["w"], grads["head"]["bias"] = linear_bwd(x.reshape(-1, ch), hd["w"], dlogits)
    dx = dflat.reshape(x.shape)
    dskip = [None] * depth                     # what the expansive path leaves for the contracting outputs
    for j in range(depth - 1, -1, -1):
        l = depth - 1 - j
        p = params["up"][j]
        below, c = up_caches[j]
        dcat, g = double_conv_bwd(p, c, dx)
        cl = outs[l].shape[3]
        dskip[l] = dcat[..., :cl]
        dx, g["wu"] = upconv2x2_bwd(below, p["wu"], dcat[..., cl:])
        grads["up"][j] = g
    for l in range(depth, -1, -1):
        if l < depth:
            dx = dx + dskip[l]
        dx, grads["down"][l] = double_conv_bwd(params["down"][l], caches[l], dx)
        if l:
            arg, shape = pools[l - 1]
            dx = maxpool_bwd(dx, arg, shape, 2, 2, 0)
    return loss, grads
