"""Pins for the convolutional oracle: the direct convolution written as seven loops, the
1x1 case that is a fully connected layer over pixels, central finite differences, the
invariants of batch normalisation, brute-force pooling."""
import numpy as np
import pytest

from oracle import cnn, nn
import synth_inputs as si


def direct_conv(x, w, stride, pad):
    """Sec. III-C direct convolution: K*K*C_in multiply-adds per output element."""
    N, H, W, Ci = x.shape
    Co, R, S, _ = w.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, Ho, Wo, Co))
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Co):
                    acc = 0.0
                    for r in range(R):
                        for s in range(S):
                            hi, wi = ho * stride - pad + r, wo * stride - pad + s
                            if 0 <= hi < H and 0 <= wi < W:
                                for ci in range(Ci):
                                    acc += x[n, hi, wi, ci] * w[co, r, s, ci]
                    y[n, ho, wo, co] = acc
    return y


@pytest.mark.parametrize("H,W,R,stride,pad", [(5, 5, 3, 1, 1), (6, 5, 3, 2, 1), (7, 7, 7, 2, 3), (4, 6, 1, 2, 0), (5, 4, 1, 1, 0)])
def test_conv_against_seven_loops(H, W, R, stride, pad):
    x = si.normal(1, (2, H, W, 3))
    w = si.normal(2, (4, R, R, 3))
    assert np.allclose(cnn.conv2d_fwd(x, w, stride, pad), direct_conv(x, w, stride, pad), rtol=0, atol=1e-12)


def test_conv1x1_is_a_linear_layer_over_pixels():
    x = si.normal(3, (2, 4, 5, 6))
    w = si.normal(4, (7, 1, 1, 6))
    dy = si.normal(5, (2, 4, 5, 7))
    y = cnn.conv2d_fwd(x, w, 1, 0)
    assert np.allclose(y.reshape(-1, 7), nn.linear_fwd(x.reshape(-1, 6), w.reshape(7, 6), 0.0), atol=1e-13)
    dx, dw = cnn.conv2d_bwd(x, w, dy, 1, 0)
    dxl, dwl, _ = nn.linear_bwd(x.reshape(-1, 6), w.reshape(7, 6), dy.reshape(-1, 7))
    assert np.allclose(dx.reshape(-1, 6), dxl, atol=1e-13) and np.allclose(dw.reshape(7, 6), dwl, atol=1e-13)


def fd(f, a, idx, h=1e-5):
    old = a[idx]
    a[idx] = old + h
    up = f()
    a[idx] = old - h
    dn = f()
    a[idx] = old
    return (up - dn) / (2 * h)


@pytest.mark.parametrize("stride,pad,R", [(1, 1, 3), (2, 1, 3), (2, 0, 1), (2, 3, 7)])
def test_conv_backward_by_finite_differences(stride, pad, R):
    x = si.normal(6, (2, 7, 6, 3))
    w = si.normal(7, (4, R, R, 3))
    y = cnn.conv2d_fwd(x, w, stride, pad)
    t = si.normal(8, y.shape)
    loss = lambda: float((cnn.conv2d_fwd(x, w, stride, pad) * t).sum())
    dx, dw = cnn.conv2d_bwd(x, w, t, stride, pad)
    for idx in [(0, 0, 0, 0), (1, 6, 5, 2), (0, 3, 2, 1), (1, 2, 4, 0)]:
        assert abs(fd(loss, x, idx) - dx[idx]) <= 1e-6 * max(1.0, abs(dx[idx]))
    for idx in [(0, 0, 0, 0), (3, R - 1, R - 1, 2), (2, R // 2, 0, 1)]:
        assert abs(fd(loss, w, idx) - dw[idx]) <= 1e-6 * max(1.0, abs(dw[idx]))


def test_batchnorm_statistics_invariants_and_finite_differences():
    x = si.normal(9, (3, 4, 5, 6)) * 2.5 + 1.0
    g = 1.0 + si.normal(10, (6,), 0.3)
    b = si.normal(11, (6,), 0.3)
    y, cache = cnn.batchnorm_fwd(x, np.ones(6), np.zeros(6))
    assert np.allclose(y.mean(axis=(0, 1, 2)), 0, atol=1e-12)
    assert np.allclose(y.var(axis=(0, 1, 2)), 1, atol=1e-4)          # eps keeps it just below 1
    y, cache = cnn.batchnorm_fwd(x, g, b)
    dy = si.normal(12, x.shape)
    dx, dg, db = cnn.batchnorm_bwd(dy, g, cache)
    assert np.allclose(dx.sum(axis=(0, 1, 2)), 0, atol=1e-11)         # shifting a channel changes nothing
    assert np.allclose((dx * cache[0]).sum(axis=(0, 1, 2)), 0, atol=1e-4)   # nor does scaling it (up to eps)
    loss = lambda: float((cnn.batchnorm_fwd(x, g, b)[0] * dy).sum())
    for idx in [(0, 0, 0, 0), (2, 3, 4, 5), (1, 2, 0, 3)]:
        assert abs(fd(loss, x, idx) - dx[idx]) <= 1e-6
    for c in (0, 5):
        assert abs(fd(loss, g, (c,)) - dg[c]) <= 1e-6 and abs(fd(loss, b, (c,)) - db[c]) <= 1e-6


def test_maxpool_brute_force_and_ties():
    x = si.normal(13, (2, 7, 6, 3))
    x[0, 0, 0, 0] = x[0, 0, 1, 0] = x[0, 1, 0, 0] = 9.0      # a tie inside the first window
    y, arg = cnn.maxpool_fwd(x)
    N, H, W, C = x.shape
    Ho, Wo = y.shape[1:3]
    assert (Ho, Wo) == (4, 3)
    dy = si.normal(14, y.shape)
    want = np.zeros_like(x)
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for c in range(C):
                    best, where = -np.inf, None
                    for r in range(3):
                        for s in range(3):
                            hi, wi = 2 * ho - 1 + r, 2 * wo - 1 + s
                            if 0 <= hi < H and 0 <= wi < W and x[n, hi, wi, c] > best:
                                best, where = x[n, hi, wi, c], r * 3 + s
                    assert y[n, ho, wo, c] == best and arg[n, ho, wo, c] == where
                    want[n, 2 * ho - 1 + where // 3, 2 * wo - 1 + where % 3, c] += dy[n, ho, wo, c]
    assert arg[0, 0, 0, 0] == 1 * 3 + 1                       # first maximum in row-major order: (0,0) of the image
    dx = cnn.maxpool_bwd(dy, arg, x.shape)
    assert np.isclose(dx.sum(), dy.sum()) and np.allclose(dx, want, atol=1e-15)
    loss = lambda: float((cnn.maxpool_fwd(x)[0] * dy).sum())
    for idx in [(1, 3, 3, 1), (0, 6, 5, 2), (1, 0, 0, 0)]:
        assert abs(fd(loss, x, idx, 1e-6) - dx[idx]) <= 1e-6


def test_avgpool():
    x = si.normal(15, (2, 3, 4, 5))
    assert np.allclose(cnn.avgpool_fwd(x), x.reshape(2, 12, 5).sum(axis=1) / 12)
    dy = si.normal(16, (2, 5))
    dx = cnn.avgpool_bwd(dy, x.shape)
    assert np.allclose(dx[1, 2, 3], dy[1] / 12) and np.isclose(dx.sum(), dy.sum())


def tiny_resnet(seed=21):
    def w(k, shape, s=0.3):
        return si.normal(seed + k, shape, s)
    def bn(k, c):
        return 1.0 + w(k, (c,), 0.1), w(k + 1, (c,), 0.1)
    def block(k, cin, mid, cout, proj):
        p = dict(w1=w(k, (mid, 1, 1, cin)), w2=w(k + 1, (mid, 3, 3, mid)), w3=w(k + 2, (cout, 1, 1, mid)))
        p["g1"], p["b1"] = bn(k + 3, mid); p["g2"], p["b2"] = bn(k + 5, mid); p["g3"], p["b3"] = bn(k + 7, cout)
        if proj:
            p["wp"] = w(k + 9, (cout, 1, 1, cin)); p["gp"], p["bp"] = bn(k + 10, cout)
        return p
    g, b = bn(1, 4)
    params = dict(stem=dict(w=w(0, (4, 7, 7, 3), 0.1), g=g, b=b),
                  blocks=[(block(10, 4, 2, 8, True), 1), (block(30, 8, 2, 8, False), 1), (block(50, 8, 4, 16, True), 2)],
                  head=dict(w=w(70, (5, 16)), b=w(71, (5,), 0.1)))
    images = si.normal(seed + 100, (2, 16, 16, 3))
    labels = np.array([1, 4])
    return params, images, labels


def test_resnet_step_by_finite_differences():
    params, images, labels = tiny_resnet()
    loss, grads = cnn.resnet_step(params, images, labels)
    assert np.isfinite(loss)
    f = lambda: cnn.resnet_step(params, images, labels)[0]
    checks = [(params["stem"]["w"], grads["stem"]["w"], (1, 3, 4, 2)), (params["stem"]["g"], grads["stem"]["g"], (2,)),
              (params["blocks"][0][0]["w2"], grads["blocks"][0]["w2"], (1, 2, 0, 1)),
              (params["blocks"][0][0]["wp"], grads["blocks"][0]["wp"], (5, 0, 0, 3)),
              (params["blocks"][1][0]["w1"], grads["blocks"][1]["w1"], (0, 0, 0, 6)),
              (params["blocks"][1][0]["b3"], grads["blocks"][1]["b3"], (7,)),
              (params["blocks"][2][0]["w3"], grads["blocks"][2]["w3"], (11, 0, 0, 2)),
              (params["blocks"][2][0]["gp"], grads["blocks"][2]["gp"], (4,)),
              (params["head"]["w"], grads["head"]["w"], (3, 9)), (params["head"]["b"], grads["head"]["b"], (0,))]
    for a, ga, idx in checks:
        num = fd(f, a, idx, 1e-5)
        assert abs(num - ga[idx]) <= 2e-6 * max(1.0, abs(ga[idx])), (idx, num, ga[idx])
