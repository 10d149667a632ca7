"""Numerical oracle for the convolutional workload (TEST INFRASTRUCTURE ONLY).

Plain definitions, in float64 numpy, of the layers of a bottleneck residual network
(KARMA Sec. III-C: convolution layer, ReLU layer, pooling layer, batch normalisation
layer, fully connected layer, softmax; the ResNet-200 row of Table III).  Activations are
NHWC, convolution weights [C_out][K][K][C_in].  `numpy.matmul`/`tensordot` is the only
library primitive used as a step: a convolution is written as the sum over its K*K taps of
a matrix product between the shifted input and that tap's [C_out][C_in] slice, which is
the direct convolution of Sec. III-C with the loops over pixels and channels handed to the
matrix product; nothing is blocked, fused or reordered beyond that.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import this file; the product library never
does and shares no code with it.

The paper names the layers and fixes none of their constants.  Readings used here (the HIP
kernels use the same ones): batch normalisation in training mode with statistics over
(N, H, W), biased variance, eps 1e-5; bottleneck = 1x1 conv, 3x3 conv (carrying the
stride), 1x1 conv, each followed by batch normalisation, ReLU after the first two and
after the residual sum; projection shortcut (1x1 conv with the block's stride + batch
normalisation) wherever the shape changes; stem 7x7 stride 2 pad 3 + batch norm + ReLU +
3x3 max pooling stride 2 pad 1 (the first maximum in row-major window order takes the
gradient); global average pooling, fully connected layer, mean cross entropy; convolutions
carry no bias.
"""
import numpy as np

from oracle.nn import cross_entropy_fwd_bwd, linear_bwd, linear_fwd

BN_EPS = 1e-5


def conv_out(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


def conv2d_fwd(x, w, stride, pad):
    """y[n,ho,wo,co] = sum_{r,s,ci} x[n, ho*stride - pad + r, wo*stride - pad + s, ci] * w[co,r,s,ci],
    out-of-range input positions counting as zero (Sec. III-C convolution layer)."""
    N, H, W, Ci = x.shape
    Co, R, S, _ = w.shape
    Ho, Wo = conv_out(H, R, stride, pad), conv_out(W, S, stride, pad)
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, Ci), dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    y = np.zeros((N, Ho, Wo, Co), dtype=x.dtype)
    for r in range(R):
        for s in range(S):
            xs = xp[:, r:r + stride * (Ho - 1) + 1:stride, s:s + stride * (Wo - 1) + 1:stride, :]
            y += xs @ w[:, r, s, :].T
    return y


def conv2d_bwd(x, w, dy, stride, pad):
    """Gradients of conv2d_fwd: dx (same shape as x) and dw (same shape as w)."""
    N, H, W, Ci = x.shape
    Co, R, S, _ = w.shape
    _, Ho, Wo, _ = dy.shape
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, Ci), dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    dy2 = dy.reshape(-1, Co)
    for r in range(R):
        for s in range(S):
            sl = (slice(None), slice(r, r + stride * (Ho - 1) + 1, stride), slice(s, s + stride * (Wo - 1) + 1, stride))
            dw[:, r, s, :] = dy2.T @ xp[sl].reshape(-1, Ci)
            dxp[sl] += dy @ w[:, r, s, :]
    return dxp[:, pad:pad + H, pad:pad + W, :], dw


def batchnorm_fwd(x, g, b):
    """Training-mode batch normalisation over (N, H, W) per channel (Sec. III-C batch
    normalisation layer: mini-batch mean, mini-batch variance, normalise, scale and shift)."""
    mu = x.mean(axis=(0, 1, 2))
    var = ((x - mu) ** 2).mean(axis=(0, 1, 2))
    rstd = 1.0 / np.sqrt(var + BN_EPS)
    xh = (x - mu) * rstd
    return xh * g + b, (xh, rstd)


def batchnorm_bwd(dy, g, cache):
    xh, rstd = cache
    m = dy.shape[0] * dy.shape[1] * dy.shape[2]
    dg = (dy * xh).sum(axis=(0, 1, 2))
    db = dy.sum(axis=(0, 1, 2))
    dx = g * rstd * (dy - db / m - xh * dg / m)
    return dx, dg, db


def maxpool_fwd(x, k=3, stride=2, pad=1):
    """Max pooling (Sec. III-C pooling layer); padding never wins.  Returns y and, per
    output element, the flat index (r*k + s) of the first maximum in row-major window order."""
    N, H, W, C = x.shape
    Ho, Wo = conv_out(H, k, stride, pad), conv_out(W, k, stride, pad)
    xp = np.full((N, H + 2 * pad, W + 2 * pad, C), -np.inf, dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    y = np.full((N, Ho, Wo, C), -np.inf, dtype=x.dtype)
    arg = np.zeros((N, Ho, Wo, C), dtype=np.int64)
    for r in range(k):
        for s in range(k):
            xs = xp[:, r:r + stride * (Ho - 1) + 1:stride, s:s + stride * (Wo - 1) + 1:stride, :]
            better = xs > y
            y = np.where(better, xs, y)
            arg = np.where(better, r * k + s, arg)
    return y, arg


def maxpool_bwd(dy, arg, in_shape, k=3, stride=2, pad=1):
    N, H, W, C = in_shape
    _, Ho, Wo, _ = dy.shape
    dxp = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=dy.dtype)
    for r in range(k):
        for s in range(k):
            dxp[:, r:r + stride * (Ho - 1) + 1:stride, s:s + stride * (Wo - 1) + 1:stride, :] += np.where(arg == r * k + s, dy, 0)
    return dxp[:, pad:pad + H, pad:pad + W, :]


def avgpool_fwd(x):
    return x.mean(axis=(1, 2))


def avgpool_bwd(dy, in_shape):
    N, H, W, C = in_shape
    return np.broadcast_to(dy[:, None, None, :] / (H * W), in_shape).copy()


# ----------------------------------------------------------------- bottleneck block
BOTTLENECK_TENSORS = ("w1", "g1", "b1", "w2", "g2", "b2", "w3", "g3", "b3", "wp", "gp", "bp")


def bottleneck_fwd(p, x, stride):
    """p: dict with w1 [mid,1,1,cin], w2 [mid,3,3,mid], w3 [cout,1,1,mid] and the batch-norm
    gains/shifts g*, b*; wp/gp/bp (projection shortcut) present iff the shape changes."""
    c1 = conv2d_fwd(x, p["w1"], 1, 0)
    n1, bc1 = batchnorm_fwd(c1, p["g1"], p["b1"])
    a1 = np.maximum(n1, 0)
    c2 = conv2d_fwd(a1, p["w2"], stride, 1)
    n2, bc2 = batchnorm_fwd(c2, p["g2"], p["b2"])
    a2 = np.maximum(n2, 0)
    c3 = conv2d_fwd(a2, p["w3"], 1, 0)
    n3, bc3 = batchnorm_fwd(c3, p["g3"], p["b3"])
    if "wp" in p:
        cp = conv2d_fwd(x, p["wp"], stride, 0)
        sc, bcp = batchnorm_fwd(cp, p["gp"], p["bp"])
    else:
        sc, bcp = x, None
    z = n3 + sc
    y = np.maximum(z, 0)
    return y, (x, n1, a1, bc1, n2, a2, bc2, bc3, bcp, z)


def bottleneck_bwd(p, cache, dy, stride):
    x, n1, a1, bc1, n2, a2, bc2, bc3, bcp, z = cache
    g = {}
    dz = dy * (z > 0)
    dc3, g["g3"], g["b3"] = batchnorm_bwd(dz, p["g3"], bc3)
    da2, g["w3"] = conv2d_bwd(a2, p["w3"], dc3, 1, 0)
    dc2, g["g2"], g["b2"] = batchnorm_bwd(da2 * (n2 > 0), p["g2"], bc2)
    da1, g["w2"] = conv2d_bwd(a1, p["w2"], dc2, stride, 1)
    dc1, g["g1"], g["b1"] = batchnorm_bwd(da1 * (n1 > 0), p["g1"], bc1)
    dx, g["w1"] = conv2d_bwd(x, p["w1"], dc1, 1, 0)
    if "wp" in p:
        dcp, g["gp"], g["bp"] = batchnorm_bwd(dz, p["gp"], bcp)
        dxp, g["wp"] = conv2d_bwd(x, p["wp"], dcp, stride, 0)
        dx = dx + dxp
    else:
        dx = dx + dz
    return dx, g


def resnet_step(params, images, labels):
    """One training step of the bottleneck network: loss and gradients.
    params: stem {w, g, b}; blocks: list of (dict, stride); head {w [classes, C], b}."""
    st = params["stem"]
    c0 = conv2d_fwd(images, st["w"], 2, 3)
    n0, bc0 = batchnorm_fwd(c0, st["g"], st["b"])
    a0 = np.maximum(n0, 0)
    x, arg = maxpool_fwd(a0)
    caches = []
    for p, stride in params["blocks"]:
        x, c = bottleneck_fwd(p, x, stride)
        caches.append(c)
    feat = avgpool_fwd(x)
    logits = linear_fwd(feat, params["head"]["w"], params["head"]["b"])
    loss, dlogits = cross_entropy_fwd_bwd(logits, labels)
    grads = {"blocks": [None] * len(params["blocks"]), "head": {}, "stem": {}}
    dfeat, grads["head"]["w"], grads["head"]["b"] = linear_bwd(feat, params["head"]["w"], dlogits)
    dx = avgpool_bwd(dfeat, x.shape)
    for i in range(len(params["blocks"]) - 1, -1, -1):
        p, stride = params["blocks"][i]
        dx, grads["blocks"][i] = bottleneck_bwd(p, caches[i], dx, stride)
    da0 = maxpool_bwd(dx, arg, a0.shape)
    dc0, grads["stem"]["g"], grads["stem"]["b"] = batchnorm_bwd(da0 * (n0 > 0), st["g"], bc0)
    _, grads["stem"]["w"] = conv2d_bwd(images, st["w"], dc0, 2, 3)
    return loss, grads
