"""Numerical oracle for the wide residual network (TEST INFRASTRUCTURE ONLY).

The WRN-28-10 row of KARMA's Table III, composed from the plain fp64 layer definitions of
`oracle/cnn.py` (Sec. III-C: convolution, batch normalisation, ReLU, pooling, fully
connected layer, softmax); nothing is blocked, fused or reordered.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import this file; the product library never
does and shares no code with it.

The paper names the model and its dataset (CIFAR-10, 32x32 images) and nothing more.
Readings used here (the HIP path uses the same ones): depth 28 and widening factor 10 mean
a 3x3 convolution to 16 channels, then three groups of (28 - 4) / 6 = 4 basic blocks of 160,
320 and 640 channels, the second and third group starting with stride 2, then batch
normalisation, ReLU, global average pooling and a fully connected layer.  A basic block is
pre-activated: o = ReLU(BN1(x)); y = conv3x3(ReLU(BN2(conv3x3(o, stride)))) + shortcut,
the shortcut being x itself when the shape is kept and a 1x1 convolution of o with the
block's stride when it changes.  Batch normalisation in training mode over (N, H, W),
biased variance, eps 1e-5; convolutions carry no bias; no dropout between the two
convolutions (the variant of the model without it); mean cross entropy.
"""
import numpy as np

from oracle.cnn import avgpool_bwd, avgpool_fwd, batchnorm_bwd, batchnorm_fwd, conv2d_bwd, conv2d_fwd
from oracle.nn import cross_entropy_fwd_bwd, linear_bwd, linear_fwd

BASIC_TENSORS = ("g1", "b1", "w1", "g2", "b2", "w2", "ws")


def basic_fwd(p, x, stride):
    """p: g1, b1 [cin]; w1 [cout,3,3,cin]; g2, b2 [cout]; w2 [cout,3,3,cout]; ws [cout,1,1,cin]
    (the shortcut convolution) present iff the block changes the shape."""
    n1, bc1 = batchnorm_fwd(x, p["g1"], p["b1"])
    o1 = np.maximum(n1, 0)
    c1 = conv2d_fwd(o1, p["w1"], stride, 1)
    n2, bc2 = batchnorm_fwd(c1, p["g2"], p["b2"])
    o2 = np.maximum(n2, 0)
    c2 = conv2d_fwd(o2, p["w2"], 1, 1)
    sc = conv2d_fwd(o1, p["ws"], stride, 0) if "ws" in p else x
    return c2 + sc, (n1, o1, bc1, n2, o2, bc2)


def basic_bwd(p, cache, dy, stride):
    n1, o1, bc1, n2, o2, bc2 = cache
    g = {}
    do2, g["w2"] = conv2d_bwd(o2, p["w2"], dy, 1, 1)
    dc1, g["g2"], g["b2"] = batchnorm_bwd(do2 * (n2 > 0), p["g2"], bc2)
    do1, g["w1"] = conv2d_bwd(o1, p["w1"], dc1, stride, 1)
    if "ws" in p:
        dos, g["ws"] = conv2d_bwd(o1, p["ws"], dy, stride, 0)
        do1 = do1 + dos
    dx, g["g1"], g["b1"] = batchnorm_bwd(do1 * (n1 > 0), p["g1"], bc1)
    if "ws" not in p:
        dx = dx + dy
    return dx, g


def wrn_step(params, images, labels):
    """One training step: loss and gradients.  params: stem {w [16,3,3,3]}; blocks: list of
    (dict, stride); head {g, b [C], w [classes, C], bias [classes]}."""
    x = conv2d_fwd(images, params["stem"]["w"], 1, 1)
    caches = []
    for p, stride in params["blocks"]:
        x, c = basic_fwd(p, x, stride)
        caches.append(c)
    hd = params["head"]
    n, bc = batchnorm_fwd(x, hd["g"], hd["b"])
    o = np.maximum(n, 0)
    feat = avgpool_fwd(o)
    logits = linear_fwd(feat, hd["w"], hd["bias"])
    loss, dlogits = cross_entropy_fwd_bwd(logits, labels)
    grads = {"blocks": [None] * len(params["blocks"]), "head": {}, "stem": {}}
    dfeat, grads["head"]["w"], grads["head"]["bias"] = linear_bwd(feat, hd["w"], dlogits)
    do = avgpool_bwd(dfeat, o.shape)
    dx, grads["head"]["g"], grads["head"]["b"] = batchnorm_bwd(do * (n > 0), hd["g"], bc)
    for i in range(len(params["blocks"]) - 1, -1, -1):
        p, stride = params["blocks"][i]
        dx, grads["blocks"][i] = basic_bwd(p, caches[i], dx, stride)
    _, grads["stem"]["w"] = conv2d_bwd(images, params["stem"]["w"], dx, 1, 1)
    return loss, grads
