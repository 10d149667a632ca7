"""Pins of the fully convolutional oracle (`oracle/unet.py`) against things other than itself:
the up-convolution against loops written from its definition, against the adjoint identity
with the (separately pinned) strided convolution and against finite differences; the whole
step against finite differences of its own loss through every kind of tensor (both halves of
the concatenation, the up-convolution, both paths into a contracting level), and against
special cases whose value is known (zero classifier: ln(classes); zero up-convolutions: the
expansive level sees the contracting output alone)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import cnn, unet


def test_upconv_is_its_definition_in_loops():
    x = si.normal(1, (2, 3, 2, 3))
    w = si.normal(2, (3, 2, 2, 4))
    y = unet.upconv2x2_fwd(x, w)
    assert y.shape == (2, 6, 4, 4)
    want = np.zeros_like(y)
    for n in range(2):
        for h in range(3):
            for v in range(2):
                for a in range(2):
                    for b in range(2):
                        for co in range(4):
                            want[n, 2 * h + a, 2 * v + b, co] = sum(x[n, h, v, ci] * w[ci, a, b, co] for ci in range(3))
    np.testing.assert_allclose(y, want, rtol=0, atol=1e-14)


def test_upconv_is_the_adjoint_of_the_strided_convolution():
    """<up(x, w), z> = <x, conv(z, w, stride 2)>: as a convolution weight [c_out][r][s][c_in] the same array
    maps the fine grid's channels back to the coarse grid's."""
    x = si.normal(3, (2, 4, 3, 5))
    w = si.normal(4, (5, 2, 2, 6))
    z = si.normal(5, (2, 8, 6, 6))
    lhs = np.sum(unet.upconv2x2_fwd(x, w) * z)
    rhs = np.sum(x * cnn.conv2d_fwd(z, w, 2, 0))
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)
    # and its gradients are that convolution's forward and weight gradient
    dx, dw = unet.upconv2x2_bwd(x, w, z)
    np.testing.assert_allclose(dx, cnn.conv2d_fwd(z, w, 2, 0), rtol=1e-12, atol=1e-12)
    _, dwk = cnn.conv2d_bwd(z, w, x, 2, 0)
    np.testing.assert_allclose(dw, dwk, rtol=1e-12, atol=1e-12)


def test_upconv_gradients_by_finite_differences():
    x = si.normal(6, (1, 2, 2, 3))
    w = si.normal(7, (3, 2, 2, 2))
    t = si.normal(8, (1, 4, 4, 2))
    f = lambda x_, w_: 0.5 * np.sum((unet.upconv2x2_fwd(x_, w_) - t) ** 2)
    dx, dw = unet.upconv2x2_bwd(x, w, unet.upconv2x2_fwd(x, w) - t)
    for arr, grad in ((x, dx), (w, dw)):
        for idx in [(0,) * arr.ndim, tuple(s - 1 for s in arr.shape), tuple(s // 2 for s in arr.shape)]:
            e = np.zeros_like(arr)
            e[idx] = 1e-6
            fd = (f(x + e, w) - f(x - e, w)) / 2e-6 if arr is x else (f(x, w + e) - f(x, w - e)) / 2e-6
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd))


def small(depth=2, **kw):
    return si.unet_problem(width=4, depth=depth, image=8, batch=2, bn_jitter=0.2, **kw)


def perturbed(params, where, idx, eps):
    import copy
    q = copy.deepcopy(params)
    part, k, name = where
    (q[part] if k is None else q[part][k])[name][idx] += eps
    return q


@pytest.mark.parametrize("where", [("down", 0, "w1"), ("down", 0, "g2"), ("down", 1, "w2"), ("down", 2, "b1"), ("up", 0, "wu"),
                                   ("up", 0, "w1"), ("up", 1, "w1"), ("up", 1, "g1"), ("head", None, "w"), ("head", None, "bias")])
def test_whole_step_gradients_by_finite_differences(where):
    params, images, labels = small()
    params["head"]["w"] = si.normal(77, params["head"]["w"].shape, 0.5)
    loss, grads = unet.unet_step(params, images, labels)
    part, k, name = where
    g = (grads[part] if k is None else grads[part][k])[name]
    arr = (params[part] if k is None else params[part][k])[name]
    picks = [(0,) * arr.ndim, tuple(s - 1 for s in arr.shape)]
    if name == "w1" and part == "up":       # one channel of each half of the concatenation
        c = arr.shape[3] // 2
        picks = [(1, 1, 1, c - 1), (1, 1, 1, c)]
    for idx in picks:
        lp = unet.unet_step(perturbed(params, where, idx, 1e-5), images, labels)[0]
        lm = unet.unet_step(perturbed(params, where, idx, -1e-5), images, labels)[0]
        fd = (lp - lm) / 2e-5
        assert abs(fd - g[idx]) <= 2e-5 * max(1e-3, abs(fd)) + 1e-9, (where, idx, fd, g[idx])


def test_zero_classifier_gives_ln_classes_and_no_gradient_below():
    params, images, labels = small(classes=3)
    params["head"]["w"][:] = 0
    loss, grads = unet.unet_step(params, images, labels)
    assert abs(loss - np.log(3)) < 1e-12
    assert all(np.all(v == 0) for lvl in grads["down"] + grads["up"] for v in lvl.values())
    # the bias gradient is (1/3 - class frequency)
    freq = np.bincount(labels.reshape(-1), minlength=3) / labels.size
    np.testing.assert_allclose(grads["head"]["bias"], 1 / 3 - freq, atol=1e-12)


def test_zero_upconvolution_leaves_the_contracting_half():
    """With the up-convolutions at zero an expansive level's first convolution sees [contracting output, 0]:
    the step equals depth-0-style stacking of double convolutions through the first C channels of w1."""
    params, images, labels = small(depth=1)
    params["head"]["w"] = si.normal(78, params["head"]["w"].shape, 0.5)
    params["up"][0]["wu"][:] = 0
    loss, grads = unet.unet_step(params, images, labels)
    # by hand: level 0, then the expansive level on its output alone
    x0, _ = unet.double_conv_fwd(params["down"][0], images)
    p = dict(params["up"][0])
    c = x0.shape[3]
    p["w1"] = p["w1"][..., :c]
    x1, _ = unet.double_conv_fwd(p, x0)
    from oracle import nn
    logits = nn.linear_fwd(x1.reshape(-1, c), params["head"]["w"], params["head"]["bias"])
    want, _ = nn.cross_entropy_fwd_bwd(logits, labels.reshape(-1))
    assert abs(loss - want) <= 1e-13 * abs(want)
    # the lowest level still receives no gradient through the silent up-convolution ...
    assert all(np.all(v == 0) for v in grads["down"][1].values())
    # ... but the up-convolution's own weight does
    assert np.abs(grads["up"][0]["wu"]).max() > 0


def test_shapes_and_parameter_count_of_the_full_model():
    """width 64, depth 4, one input channel, two classes: the model the paper lists with 'more than 31M'
    parameters."""
    params, _, _ = si.unet_problem(image=16, batch=1)
    n = sum(v.size for lvl in params["down"] + params["up"] for v in lvl.values()) + sum(v.size for v in params["head"].values())
    assert 31.0e6 < n < 31.1e6
    convs = 2 * 5 + 2 * 4 + 4 + 1      # 3x3 convolutions, up-convolutions, classifier
    assert convs == 23
