"""A bottleneck-network step that keeps its tensors in bf16 (TEST HELPER, not the oracle).

The oracle (`oracle/cnn.py`) is the plain fp64 definition and rounds nowhere.  This file
composes the oracle's layer functions into the same step, but rounds to bf16 every tensor
that a bf16 training step writes to memory between two operations: convolution outputs,
ReLU outputs, the shortcut, pooled features, logits and every gradient tensor handed from
one layer to the next; arithmetic inside a layer stays fp64.  It answers one question on
the CPU: how far does bf16 storage alone move the gradients of this network away from the
plain definition?  `tests/test_cnn_bf16_floor.py` measures that distance (the floor under
any bf16 implementation), and the GPU whole-step test sets its tolerance from it.
"""
import numpy as np

from oracle import cnn, nn


def q(a):
    """Round to nearest-even bf16, returned as float64."""
    return nn.bf16_round(np.asarray(a, np.float32)).astype(np.float64)


def _block_fwd(p, x, stride):
    c1 = q(cnn.conv2d_fwd(x, p["w1"], 1, 0))
    n1, s1 = cnn.batchnorm_fwd(c1, p["g1"], p["b1"])
    a1 = q(np.maximum(n1, 0))
    c2 = q(cnn.conv2d_fwd(a1, p["w2"], stride, 1))
    n2, s2 = cnn.batchnorm_fwd(c2, p["g2"], p["b2"])
    a2 = q(np.maximum(n2, 0))
    c3 = q(cnn.conv2d_fwd(a2, p["w3"], 1, 0))
    n3, s3 = cnn.batchnorm_fwd(c3, p["g3"], p["b3"])
    if "wp" in p:
        cp = q(cnn.conv2d_fwd(x, p["wp"], stride, 0))
        sc, sp = cnn.batchnorm_fwd(cp, p["gp"], p["bp"])
        sc = q(sc)
    else:
        sc, sp = x, None
    z = n3 + sc
    return q(np.maximum(z, 0)), (x, n1, a1, s1, n2, a2, s2, s3, sp, z)


def _block_bwd(p, saved, dy, stride):
    x, n1, a1, s1, n2, a2, s2, s3, sp, z = saved
    g = {}
    dz = dy * (z > 0)
    dc3, g["g3"], g["b3"] = cnn.batchnorm_bwd(dz, p["g3"], s3)
    da2, g["w3"] = cnn.conv2d_bwd(a2, p["w3"], q(dc3), 1, 0)
    dc2, g["g2"], g["b2"] = cnn.batchnorm_bwd(q(da2) * (n2 > 0), p["g2"], s2)
    da1, g["w2"] = cnn.conv2d_bwd(a1, p["w2"], q(dc2), stride, 1)
    dc1, g["g1"], g["b1"] = cnn.batchnorm_bwd(q(da1) * (n1 > 0), p["g1"], s1)
    dx, g["w1"] = cnn.conv2d_bwd(x, p["w1"], q(dc1), 1, 0)
    if "wp" in p:
        dcp, g["gp"], g["bp"] = cnn.batchnorm_bwd(dz, p["gp"], sp)
        dxp, g["wp"] = cnn.conv2d_bwd(x, p["wp"], q(dcp), stride, 0)
        dx = dx + q(dxp)
    else:
        dx = dx + dz
    return q(dx), g


def resnet_step_bf16_storage(params, images, labels):
    """Same signature and result layout as `oracle.cnn.resnet_step`."""
    st = params["stem"]
    c0 = q(cnn.conv2d_fwd(images, st["w"], 2, 3))
    n0, s0 = cnn.batchnorm_fwd(c0, st["g"], st["b"])
    a0 = q(np.maximum(n0, 0))
    x, arg = cnn.maxpool_fwd(a0)
    saved = []
    for p, stride in params["blocks"]:
        x, s = _block_fwd(p, x, stride)
        saved.append(s)
    feat = q(cnn.avgpool_fwd(x))
    logits = q(nn.linear_fwd(feat, params["head"]["w"], params["head"]["b"]))
    loss, dlogits = nn.cross_entropy_fwd_bwd(logits, labels)
    grads = {"blocks": [None] * len(params["blocks"]), "head": {}, "stem": {}}
    dfeat, grads["head"]["w"], grads["head"]["b"] = nn.linear_bwd(feat, params["head"]["w"], q(dlogits))
    dx = q(cnn.avgpool_bwd(q(dfeat), x.shape))
    for i in range(len(params["blocks"]) - 1, -1, -1):
        p, stride = params["blocks"][i]
        dx, grads["blocks"][i] = _block_bwd(p, saved[i], dx, stride)
    da0 = q(cnn.maxpool_bwd(dx, arg, a0.shape))
    dc0, grads["stem"]["g"], grads["stem"]["b"] = cnn.batchnorm_bwd(da0 * (n0 > 0), st["g"], s0)
    _, grads["stem"]["w"] = cnn.conv2d_bwd(images, st["w"], q(dc0), 2, 3)
    return loss, grads


# ------------------------------------------------------------------ shared by the floor test and the GPU test
SMALL = dict(width=8, stage_blocks=(1, 2, 1, 1), image=64, batch=4, classes=16)
SHALLOW = dict(width=8, stage_blocks=(1, 1, 0, 0), image=64, batch=4, classes=16)
SHIFT_PARAMS = ("b1", "b2", "b3", "bp")


def rounded_params(params):
    return dict(stem={k: q(v) for k, v in params["stem"].items()},
                blocks=[({k: q(v) for k, v in p.items()}, s) for p, s in params["blocks"]],
                head={k: q(v) for k, v in params["head"].items()})


def problem(dims, shift, seed=2008114203):
    """Seeded network and batch; every batch-norm shift raised by `shift`; images on the bf16 grid."""
    import synth_inputs as si
    params, images, labels = si.cnn_problem(seed=seed, bn_jitter=0.1, **dims)
    params["stem"]["b"] = params["stem"]["b"] + shift
    for p, _ in params["blocks"]:
        for k in SHIFT_PARAMS:
            if k in p:
                p[k] = p[k] + shift
    return params, q(images), labels.astype(np.int32)


def flat(grads):
    out = {"stem." + k: v for k, v in grads["stem"].items()}
    out.update({"head." + k: v for k, v in grads["head"].items()})
    for i, gb in enumerate(grads["blocks"]):
        for k, v in gb.items():
            out["b%d.%s" % (i, k)] = v
    return out


def scale_of(name, want):
    """Norm a tensor's error is measured against: its own, except for the shift of a batch
    norm that feeds a convolution + batch norm.  That shift has (almost) no gradient (the
    next normalisation removes a constant), so its error is measured against the gradient
    of the gain beside it."""
    s = np.linalg.norm(want[name])
    leaf = name.split(".")[-1]
    if leaf in SHIFT_PARAMS:
        s = max(s, np.linalg.norm(want[name[:-2] + "g" + name[-1:]]))
    elif name == "stem.b":
        s = max(s, np.linalg.norm(want["stem.g"]))
    return s


def distances(got, want):
    """Per tensor: ||got - want|| / scale_of(want)."""
    return {k: float(np.linalg.norm(np.asarray(got[k], np.float64).reshape(-1) - want[k].reshape(-1)) / scale_of(k, want))
            for k in want}


# ------------------------------------------------------------------ wide residual network
def _basic_fwd(p, x, stride):
    n1, s1 = cnn.batchnorm_fwd(x, p["g1"], p["b1"])
    o1 = q(np.maximum(n1, 0))
    c1 = q(cnn.conv2d_fwd(o1, p["w1"], stride, 1))
    n2, s2 = cnn.batchnorm_fwd(c1, p["g2"], p["b2"])
    o2 = q(np.maximum(n2, 0))
    sc = q(cnn.conv2d_fwd(o1, p["ws"], stride, 0)) if "ws" in p else x
    return q(cnn.conv2d_fwd(o2, p["w2"], 1, 1) + sc), (n1, o1, s1, n2, o2, s2)


def _basic_bwd(p, saved, dy, stride):
    n1, o1, s1, n2, o2, s2 = saved
    g = {}
    do2, g["w2"] = cnn.conv2d_bwd(o2, p["w2"], dy, 1, 1)
    dc1, g["g2"], g["b2"] = cnn.batchnorm_bwd(q(do2) * (n2 > 0), p["g2"], s2)
    do1, g["w1"] = cnn.conv2d_bwd(o1, p["w1"], q(dc1), stride, 1)
    if "ws" in p:
        dos, g["ws"] = cnn.conv2d_bwd(o1, p["ws"], dy, stride, 0)
        do1 = do1 + q(dos)
    dx, g["g1"], g["b1"] = cnn.batchnorm_bwd(q(do1) * (n1 > 0), p["g1"], s1)
    if "ws" not in p:
        dx = dx + dy
    return q(dx), g


def wrn_step_bf16_storage(params, images, labels):
    """Same signature and result layout as `oracle.wrn.wrn_step`, tensors between operations rounded to bf16."""
    x = q(cnn.conv2d_fwd(images, params["stem"]["w"], 1, 1))
    saved = []
    for p, stride in params["blocks"]:
        x, s = _basic_fwd(p, x, stride)
        saved.append(s)
    hd = params["head"]
    n, sh = cnn.batchnorm_fwd(x, hd["g"], hd["b"])
    o = q(np.maximum(n, 0))
    feat = q(cnn.avgpool_fwd(o))
    logits = q(nn.linear_fwd(feat, hd["w"], hd["bias"]))
    loss, dlogits = nn.cross_entropy_fwd_bwd(logits, labels)
    grads = {"blocks": [None] * len(params["blocks"]), "head": {}, "stem": {}}
    dfeat, grads["head"]["w"], grads["head"]["bias"] = nn.linear_bwd(feat, hd["w"], q(dlogits))
    do = q(cnn.avgpool_bwd(q(dfeat), o.shape))
    dx, grads["head"]["g"], grads["head"]["b"] = cnn.batchnorm_bwd(do * (n > 0), hd["g"], sh)
    dx = q(dx)
    for i in range(len(params["blocks"]) - 1, -1, -1):
        p, stride = params["blocks"][i]
        dx, grads["blocks"][i] = _basic_bwd(p, saved[i], dx, stride)
    _, grads["stem"]["w"] = cnn.conv2d_bwd(images, params["stem"]["w"], dx, 1, 1)
    return loss, grads


WRN_SMALL = dict(width=16, group_blocks=(1, 2, 1), image=16, batch=4, classes=16)


def wrn_problem(dims, shift, seed=2008114204):
    """Seeded wide residual network and batch; every batch-norm shift raised by `shift`; images on the bf16 grid."""
    import synth_inputs as si
    params, images, labels = si.wrn_problem(seed=seed, bn_jitter=0.1, **dims)
    for p, _ in params["blocks"]:
        p["b1"] = p["b1"] + shift
        p["b2"] = p["b2"] + shift
    params["head"]["b"] = params["head"]["b"] + shift
    return params, q(images), labels.astype(np.int32)


# ------------------------------------------------------------------ fully convolutional network
def _double_conv_fwd(p, x, x2=None):
    """x2: second half of the concatenated input (the convolution over the concatenation is computed as the
    sum of one convolution per half, the first half's result stored in between)."""
    if x2 is None:
        c1 = q(cnn.conv2d_fwd(x, p["w1"], 1, 1))
    else:
        c = x.shape[3]
        half = q(cnn.conv2d_fwd(x, p["w1"][..., :c], 1, 1))
        c1 = q(cnn.conv2d_fwd(x2, p["w1"][..., c:], 1, 1) + half)
    n1, s1 = cnn.batchnorm_fwd(c1, p["g1"], p["b1"])
    a1 = q(np.maximum(n1, 0))
    c2 = q(cnn.conv2d_fwd(a1, p["w2"], 1, 1))
    n2, s2 = cnn.batchnorm_fwd(c2, p["g2"], p["b2"])
    return q(np.maximum(n2, 0)), (x, x2, n1, a1, s1, n2, s2)


def _double_conv_bwd(p, saved, dy):
    x, x2, n1, a1, s1, n2, s2 = saved
    g = {}
    dc2, g["g2"], g["b2"] = cnn.batchnorm_bwd(dy * (n2 > 0), p["g2"], s2)
    da1, g["w2"] = cnn.conv2d_bwd(a1, p["w2"], q(dc2), 1, 1)
    dc1, g["g1"], g["b1"] = cnn.batchnorm_bwd(q(da1) * (n1 > 0), p["g1"], s1)
    dc1 = q(dc1)
    if x2 is None:
        dx, g["w1"] = cnn.conv2d_bwd(x, p["w1"], dc1, 1, 1)
        return q(dx), None, g
    c = x.shape[3]
    dx, gw_a = cnn.conv2d_bwd(x, p["w1"][..., :c], dc1, 1, 1)
    dx2, gw_b = cnn.conv2d_bwd(x2, p["w1"][..., c:], dc1, 1, 1)
    g["w1"] = np.concatenate([gw_a, gw_b], axis=3)
    return q(dx), q(dx2), g


def unet_step_bf16_storage(params, images, labels):
    """Same signature and result layout as `oracle.unet.unet_step`, tensors between operations rounded to bf16."""
    from oracle import unet
    depth = len(params["up"])
    outs, saved, pools = [], [], []
    x = images
    for l, p in enumerate(params["down"]):
        if l:
            x, arg = cnn.maxpool_fwd(x, 2, 2, 0)
            pools.append((arg, outs[-1].shape))
        x, s = _double_conv_fwd(p, x)
        outs.append(x)
        saved.append(s)
    up_saved = []
    for j, p in enumerate(params["up"]):
        l = depth - 1 - j
        u = q(unet.upconv2x2_fwd(x, p["wu"]))
        below = x
        x, s = _double_conv_fwd(p, outs[l], u)
        up_saved.append((below, s))
    hd = params["head"]
    ch = x.shape[3]
    flatx = x.reshape(-1, ch)
    logits = q(nn.linear_fwd(flatx, hd["w"], hd["bias"]))
    loss, dlogits = nn.cross_entropy_fwd_bwd(logits, labels.reshape(-1))
    grads = {"down": [None] * (depth + 1), "up": [None] * depth, "head": {}}
    dflat, grads["head"]["w"], grads["head"]["bias"] = nn.linear_bwd(flatx, hd["w"], q(dlogits))
    dx = q(dflat).reshape(x.shape)
    dskip = [None] * depth
    for j in range(depth - 1, -1, -1):
        l = depth - 1 - j
        p = params["up"][j]
        below, s = up_saved[j]
        dskip[l], du, g = _double_conv_bwd(p, s, dx)
        dxb, g["wu"] = unet.upconv2x2_bwd(below, p["wu"], du)
        dx = q(dxb)
        grads["up"][j] = g
    for l in range(depth, -1, -1):
        if l < depth:
            dx = q(dx + dskip[l])
        dx, _, grads["down"][l] = _double_conv_bwd(params["down"][l], saved[l], dx)
        if l:
            arg, shape = pools[l - 1]
            dx = cnn.maxpool_bwd(dx, arg, shape, 2, 2, 0)
    return loss, grads


UNET_SMALL = dict(width=8, depth=2, image=32, batch=2, classes=2)


def unet_problem(dims, shift, seed=2008114205):
    """Seeded fully convolutional network and batch; every batch-norm shift raised by `shift`; images on the bf16 grid."""
    import synth_inputs as si
    params, images, labels = si.unet_problem(seed=seed, bn_jitter=0.1, **dims)
    params["head"]["w"] = si.normal(seed + 99, params["head"]["w"].shape, 0.3)   # a classifier that already discriminates
    for p in params["down"] + params["up"]:
        p["b1"] = p["b1"] + shift
        p["b2"] = p["b2"] + shift
    return params, q(images), labels.astype(np.int32)


def unet_rounded_params(params):
    return dict(down=[{k: q(v) for k, v in p.items()} for p in params["down"]],
                up=[{k: q(v) for k, v in p.items()} for p in params["up"]],
                head={k: q(v) for k, v in params["head"].items()})


def unet_flat(grads):
    out = {"head." + k: v for k, v in grads["head"].items()}
    for l, gl in enumerate(grads["down"]):
        for k, v in gl.items():
            out["d%d.%s" % (l, k)] = v
    for j, gl in enumerate(grads["up"]):
        for k, v in gl.items():
            out["u%d.%s" % (j, k)] = v
    return out
