"""Pins for the numerical oracle: central finite differences in fp64, closed forms,
invariants and special cases.  None of them calls the oracle to check the oracle."""
import math

import numpy as np
import pytest

from oracle import nn
import synth_inputs as si


def fd_check(f, arrays, grads, rng, n_probe=12, h=1e-5, tol=1e-6):
    """f() -> scalar using the arrays in place; compares analytic grads with central
    differences on a few random coordinates of every array."""
    for a, g in zip(arrays, grads):
        assert a.shape == g.shape
        flat = a.reshape(-1)
        for idx in rng.choice(flat.size, size=min(n_probe, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + h
            fp = f()
            flat[idx] = old - h
            fm = f()
            flat[idx] = old
            num = (fp - fm) / (2 * h)
            ana = g.reshape(-1)[idx]
            assert abs(num - ana) <= tol * max(1.0, abs(num), abs(ana)), (idx, num, ana)


def test_linear_closed_form_and_fd():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7)); W = rng.standard_normal((3, 7)); b = rng.standard_normal(3)
    y = nn.linear_fwd(x, W, b)
    # closed form written out with loops
    for m in range(5):
        for n in range(3):
            assert math.isclose(y[m, n], sum(x[m, k] * W[n, k] for k in range(7)) + b[n], rel_tol=1e-12)
    dy = rng.standard_normal((5, 3))
    dx, dW, db = nn.linear_bwd(x, W, dy)
    assert np.allclose(dW, np.einsum("mn,mk->nk", dy, x))
    assert np.allclose(dx, np.einsum("mn,nk->mk", dy, W))
    assert np.allclose(db, dy.sum(0))
    f = lambda: float((nn.linear_fwd(x, W, b) * dy).sum())
    fd_check(f, [x, W, b], [dx, dW, db], rng)


def test_mse_closed_form():
    y = np.array([[1.0, 2.0], [3.0, 5.0]]); t = np.array([[0.0, 2.0], [1.0, 1.0]])
    loss, d = nn.mse_fwd_bwd(y, t)
    assert loss == pytest.approx((1 + 0 + 4 + 16) / 4)
    assert np.allclose(d, 2 * (y - t) / 4)


def test_layernorm_fd_and_invariants():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 16)); g = rng.standard_normal(16); b = rng.standard_normal(16)
    w = rng.standard_normal((4, 16))
    y, cache = nn.layernorm_fwd(x, g, b)
    # normalised rows have zero mean and unit (biased) variance up to eps
    xhat = cache[0]
    assert np.allclose(xhat.mean(-1), 0, atol=1e-12)
    assert np.allclose((xhat ** 2).mean(-1), 1, atol=1e-4)
    dx, dg, db = nn.layernorm_bwd(w, g, cache)
    assert np.allclose(dx.sum(-1), 0, atol=1e-12)
    assert np.allclose((dx * xhat).sum(-1), 0, atol=1e-4)     # exact up to the eps in the variance
    f = lambda: float((nn.layernorm_fwd(x, g, b)[0] * w).sum())
    fd_check(f, [x, g, b], [dx, dg, db], rng)


def test_gelu_values_and_fd():
    # tanh-form GELU: odd part is x/2, known points
    x = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    y = nn.gelu_fwd(x)
    assert y[2] == 0.0
    assert np.allclose(nn.gelu_fwd(x) - nn.gelu_fwd(-x), x)        # g(x) - g(-x) = x
    assert y[4] == pytest.approx(0.5 * 2 * (1 + math.tanh(math.sqrt(2 / math.pi) * (2 + 0.044715 * 8))))
    rng = np.random.default_rng(2)
    w = rng.standard_normal(5)
    d = nn.gelu_bwd(x, w)
    f = lambda: float((nn.gelu_fwd(x) * w).sum())
    fd_check(f, [x], [d], rng)


def test_attention_special_cases():
    rng = np.random.default_rng(3)
    # S = 1: output is V
    q, k, v = (rng.standard_normal((1, 8)) for _ in range(3))
    o, p = nn.attention_fwd(q, k, v)
    assert np.allclose(o, v) and np.allclose(p, 1)
    # causal: row 0 attends only to itself; rows of P sum to 1; strictly upper part zero
    q, k, v = (rng.standard_normal((6, 4)) for _ in range(3))
    o, p = nn.attention_fwd(q, k, v)
    assert np.allclose(o[0], v[0])
    assert np.allclose(p.sum(-1), 1) and np.allclose(np.triu(p, 1), 0)
    # equal keys: uniform attention over the causal prefix -> running mean of V
    o2, _ = nn.attention_fwd(q, np.ones((6, 4)), v)
    assert np.allclose(o2, np.cumsum(v, 0) / np.arange(1, 7)[:, None])
    # brute-force loops for one row
    i = 4
    s = np.array([sum(q[i, c] * k[j, c] for c in range(4)) / 2.0 for j in range(i + 1)])
    e = np.exp(s - s.max()); e /= e.sum()
    assert np.allclose(o[i], sum(e[j] * v[j] for j in range(i + 1)))


def test_attention_fd():
    rng = np.random.default_rng(4)
    q, k, v = (rng.standard_normal((5, 4)) for _ in range(3))
    w = rng.standard_normal((5, 4))
    o, p = nn.attention_fwd(q, k, v)
    dq, dk, dv = nn.attention_bwd(q, k, v, p, w)
    f = lambda: float((nn.attention_fwd(q, k, v)[0] * w).sum())
    fd_check(f, [q, k, v], [dq, dk, dv], rng, n_probe=20)


def test_cross_entropy_identities():
    rng = np.random.default_rng(5)
    V = 32000
    loss, d = nn.cross_entropy_fwd_bwd(np.zeros((3, V)), np.array([0, 5, V - 1]))
    assert loss == pytest.approx(math.log(V))          # uniform logits -> ln V = 10.373...
    assert loss == pytest.approx(10.3735, abs=1e-4)
    assert nn.cross_entropy_fwd_bwd(np.zeros((2, 51200)), np.array([1, 2]))[0] == pytest.approx(10.8435, abs=1e-4)
    lg = rng.standard_normal((4, 9)); lab = np.array([0, 3, 8, 3])
    loss, d = nn.cross_entropy_fwd_bwd(lg, lab)
    assert np.allclose(d.sum(-1), 0, atol=1e-15)
    p = np.exp(lg) / np.exp(lg).sum(-1, keepdims=True)
    oh = np.eye(9)[lab]
    assert np.allclose(d, (p - oh) / 4)
    f = lambda: nn.cross_entropy_fwd_bwd(lg, lab)[0]
    fd_check(f, [lg], [d], rng)


def test_mlp_step_fd():
    Ws, bs, x, t = si.mlp_problem(seed=7, n_layers=3, width=6, batch=4)
    bs = [b + 0.1 for b in bs]
    loss, dWs, dbs, _ = nn.mlp_step(Ws, bs, x, t)
    rng = np.random.default_rng(6)
    f = lambda: nn.mlp_step(Ws, bs, x, t)[0]
    fd_check(f, Ws + bs, dWs + dbs, rng, h=1e-6, tol=1e-5)


def _flat_params(params):
    arrs = [params["wte"], params["wpe"], params["lnf_g"], params["lnf_b"]]
    for b in params["blocks"]:
        arrs += [b[k] for k in nn.BLOCK_TENSORS]
    return arrs


def _flat_grads(g):
    arrs = [g["wte"], g["wpe"], g["lnf_g"], g["lnf_b"]]
    for b in g["blocks"]:
        arrs += [b[k] for k in nn.BLOCK_TENSORS]
    return arrs


def test_gpt_step_fd():
    params, ids, labels = si.gpt_problem(seed=11, n_layers=2, hidden=8, ffn=16, vocab=13,
                                         seq=5, batch=2, std=0.3, bias_std=0.2)
    ids[0, 1] = ids[0, 0]          # a repeated token exercises the scatter-add
    loss, grads, hs, dhs = nn.gpt_step(params, ids, labels, n_heads=2)
    rng = np.random.default_rng(7)
    f = lambda: nn.gpt_step(params, ids, labels, 2)[0]
    fd_check(f, _flat_params(params), _flat_grads(grads), rng, n_probe=6, h=1e-6, tol=2e-5)


def test_gpt_zero_weights_loss_is_ln_vocab():
    params, ids, labels = si.gpt_problem(seed=12, n_layers=1, hidden=8, ffn=16, vocab=50,
                                         seq=4, batch=2, std=0.3)
    params["wte"][:] = 0
    loss = nn.gpt_step(params, ids, labels, 2)[0]
    assert loss == pytest.approx(math.log(50))


def test_block_samples_independent():
    """A transformer block treats batch entries independently: the basis of the sampled
    full-size parity checks."""
    params, ids, labels = si.gpt_problem(seed=13, n_layers=1, hidden=8, ffn=16, vocab=20,
                                         seq=6, batch=3, std=0.3, bias_std=0.1)
    x = si.normal(5, (3, 6, 8))
    y, _ = nn.block_fwd(params["blocks"][0], x, 2)
    y1, _ = nn.block_fwd(params["blocks"][0], x[1:2], 2)
    assert np.allclose(y[1:2], y1, atol=1e-14)


def test_optimisers():
    w = np.array([1.0, -2.0, 3.0]); g = np.array([0.5, -0.25, 4.0])
    assert np.allclose(nn.sgd_update(w, g, 0.1), [0.95, -1.975, 2.6])
    w2, buf = nn.sgd_momentum_update(w, np.array([1.0, 1.0, 1.0]), g, 0.1, 0.9)
    assert np.allclose(buf, [1.4, 0.65, 4.9]) and np.allclose(w2, w - 0.1 * buf)
    # the first bias-corrected Adam step moves every weight by lr*sign(g) (up to eps)
    w3, m, v = nn.adam_update(w, np.zeros(3), np.zeros(3), g, 1, 1e-3)
    assert np.allclose(w3, w - 1e-3 * np.sign(g), atol=1e-9)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)
    # second step against the recurrences written out
    g2 = np.array([-1.0, 0.5, 2.0])
    w4, m2, v2 = nn.adam_update(w3, m, v, g2, 2, 1e-3)
    mm = 0.9 * 0.1 * g + 0.1 * g2; vv = 0.999 * 0.001 * g * g + 0.001 * g2 * g2
    assert np.allclose(w4, w3 - 1e-3 * (mm / (1 - 0.81)) / (np.sqrt(vv / (1 - 0.999 ** 2)) + 1e-8))


def test_bf16_round():
    a = np.array([1.0, 1.00390625, 1.01171875, 3.140625, -2.5, 0.0], dtype=np.float32)
    r = nn.bf16_round(a)
    # bf16 has 8 significant bits: 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> 1 + 2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625)
    assert r[3] == np.float32(3.140625) and r[4] == -2.5 and r[5] == 0.0
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
