"""Pins of the wide-residual-network oracle: its layer functions are pinned in
test_oracle_cnn.py; here the composition (pre-activated basic block, shortcut from the
activated input, head) is checked by finite differences of the loss, by the identities the
architecture implies, and by the parameter count the paper's Table III quotes."""
import numpy as np

from oracle import cnn, wrn
import synth_inputs as si
from test_oracle_cnn import fd


def tiny(seed=31):
    def w(k, shape, s=0.3):
        return si.normal(seed + k, shape, s)
    def bn(k, c):
        return 1.0 + w(k, (c,), 0.1), w(k + 1, (c,), 0.1)
    def block(k, cin, cout):
        p = {}
        p["g1"], p["b1"] = bn(k, cin)
        p["w1"] = w(k + 2, (cout, 3, 3, cin))
        p["g2"], p["b2"] = bn(k + 3, cout)
        p["w2"] = w(k + 5, (cout, 3, 3, cout))
        if cin != cout:
            p["ws"] = w(k + 6, (cout, 1, 1, cin))
        return p
    g, b = bn(90, 8)
    params = dict(stem=dict(w=w(0, (3, 3, 3, 3), 0.2)),
                  blocks=[(block(10, 3, 4), 1), (block(20, 4, 4), 1), (block(30, 4, 8), 2), (block(40, 8, 8), 1)],
                  head=dict(g=g, b=b, w=w(70, (5, 8)), bias=w(71, (5,), 0.1)))
    images = si.normal(seed + 100, (3, 8, 8, 3))
    labels = np.array([1, 4, 0])
    return params, images, labels


def test_wrn_step_by_finite_differences():
    params, images, labels = tiny()
    loss, grads = wrn.wrn_step(params, images, labels)
    assert np.isfinite(loss)
    f = lambda: wrn.wrn_step(params, images, labels)[0]
    B, G = params["blocks"], grads["blocks"]
    checks = [(params["stem"]["w"], grads["stem"]["w"], (1, 2, 0, 2)),
              (B[0][0]["g1"], G[0]["g1"], (2,)), (B[0][0]["w1"], G[0]["w1"], (3, 1, 2, 0)), (B[0][0]["ws"], G[0]["ws"], (2, 0, 0, 1)),
              (B[1][0]["b1"], G[1]["b1"], (3,)), (B[1][0]["w2"], G[1]["w2"], (0, 2, 1, 3)), (B[1][0]["g2"], G[1]["g2"], (1,)),
              (B[2][0]["w1"], G[2]["w1"], (6, 0, 0, 2)), (B[2][0]["ws"], G[2]["ws"], (7, 0, 0, 3)), (B[2][0]["b2"], G[2]["b2"], (5,)),
              (B[3][0]["w2"], G[3]["w2"], (4, 1, 1, 7)), (B[3][0]["g1"], G[3]["g1"], (0,)),
              (params["head"]["g"], grads["head"]["g"], (6,)), (params["head"]["b"], grads["head"]["b"], (2,)),
              (params["head"]["w"], grads["head"]["w"], (3, 5)), (params["head"]["bias"], grads["head"]["bias"], (0,))]
    for a, ga, idx in checks:
        num = fd(f, a, idx, 1e-5)
        assert abs(num - ga[idx]) <= 2e-6 * max(1.0, abs(ga[idx])), (idx, num, ga[idx])
    assert sorted(G[0]) == sorted(B[0][0]) and "ws" not in G[1]


def test_identity_shortcut_passes_the_gradient_and_the_input_through():
    """With a zero second convolution a shape-keeping block is the identity, forward and backward;
    with a shortcut convolution it is that convolution of the activated input."""
    params, images, _ = tiny()
    x = si.normal(5, (2, 6, 6, 4))
    p = dict(params["blocks"][1][0])
    p["w2"] = np.zeros_like(p["w2"])
    y, cache = wrn.basic_fwd(p, x, 1)
    assert np.array_equal(y, x)
    dy = si.normal(6, y.shape)
    dx, g = wrn.basic_bwd(p, cache, dy, 1)
    assert np.allclose(dx, dy) and not g["w1"].any() and g["w2"].any()
    q = dict(params["blocks"][2][0])
    q["w2"] = np.zeros_like(q["w2"])
    y, cache = wrn.basic_fwd(q, x, 2)
    o1 = np.maximum(cnn.batchnorm_fwd(x, q["g1"], q["b1"])[0], 0)
    assert y.shape == (2, 3, 3, 8) and np.allclose(y, cnn.conv2d_fwd(o1, q["ws"], 2, 0))


def test_default_shapes_are_wrn_28_10():
    """36.5 M parameters (Table III: "> 36M"); 28 convolutions: the first, two per basic block and
    the three shortcut convolutions (depth = 6 * 4 + 4)."""
    shapes = []
    cin = 16
    n_conv = 1
    total = 16 * 27
    for gi in range(3):
        cout = 160 << gi
        for j in range(4):
            total += 2 * cin + cout * 9 * cin + 2 * cout + cout * 9 * cout + (cout * cin if cin != cout else 0)
            n_conv += 2
            cin = cout
    total += 2 * 640 + 640 * 10 + 10
    assert n_conv + 3 == 28
    assert 36.4e6 < total < 36.6e6
    params, images, labels = si.wrn_problem(batch=2, width=8, stem=8)       # same builder, narrow
    assert len(params["blocks"]) == 12 and [s for _, s in params["blocks"]] == [1, 1, 1, 1, 2, 1, 1, 1, 2, 1, 1, 1]
    assert [("ws" in p) for p, _ in params["blocks"]] == [False, False, False, False, True, False, False, False, True, False, False, False]
    assert images.shape == (2, 32, 32, 3) and params["head"]["w"].shape == (10, 32)
    full = si.wrn_problem.__defaults__
    assert full[1:6] == (160, (4, 4, 4), 32, 128, 10)
