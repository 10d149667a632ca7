"""Numerical oracle for the training step (TEST INFRASTRUCTURE ONLY).

Swapping and recomputation leave the mathematics of a step untouched (KARMA, Sec. IV-C:
neither the shape nor the hyper-parameters of the model change), so the reference for
every out-of-core step is the in-core step by its textbook definition.  This file writes
that definition out with numpy: forward, reverse-mode backward, loss and one optimiser
update, for the layer types the paper lists in Sec. III-C (fully connected, ReLU,
softmax, self-attention `Softmax(QK^T/sqrt(d_k))V`) plus the ones a GPT-style block
needs.  `numpy.matmul` is the only library primitive used as a step; nothing is fused,
blocked or reordered.  Default precision is float64; pass dtype=np.float32 for the fp32
variant.  Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this file; the product library never does and shares no code with it.

The paper names the layers but fixes none of their constants.  Readings used here (the
HIP kernels use the same ones): pre-LN GPT block `x += Proj(Attn(LN1(x)))`,
`x += FC2(GELU(FC1(LN2(x))))`; causal mask; scale 1/sqrt(d_head); tanh-form GELU;
LayerNorm eps 1e-5 with biased variance; LM head tied to the token embedding; losses
are means over all elements (MSE) or all tokens (cross entropy); Adam is bias-corrected
with no weight decay.
"""
import numpy as np

LN_EPS = 1e-5
GELU_C = 0.7978845608028654   # sqrt(2/pi)
GELU_A = 0.044715


# ----------------------------------------------------------------- elementary layers
def linear_fwd(x, W, b):
    """y = x W^T + b with W stored [out, in] (Sec. III-C fully-connected layer)."""
    return x @ W.T + b


def linear_bwd(x, W, dy):
    """Returns dx, dW, db."""
    return dy @ W, dy.T @ x, dy.sum(axis=0)


def relu_fwd(z):
    return np.maximum(z, 0)


def relu_bwd(z, dy):
    return dy * (z > 0)


def mse_fwd_bwd(y, t):
    """Mean over every element of (y - t)^2 and its gradient w.r.t. y."""
    d = y - t
    return float(np.mean(d * d)), 2.0 * d / d.size


def layernorm_fwd(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_bwd(dy, g, cache):
    xhat, rstd = cache
    dg = (dy * xhat).sum(axis=0)
    db = dy.sum(axis=0)
    dxhat = dy * g
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def gelu_fwd(x):
    u = GELU_C * (x + GELU_A * x ** 3)
    return 0.5 * x * (1.0 + np.tanh(u))


def gelu_bwd(x, dy):
    u = GELU_C * (x + GELU_A * x ** 3)
    th = np.tanh(u)
    du = GELU_C * (1.0 + 3.0 * GELU_A * x * x)
    return dy * (0.5 * (1.0 + th) + 0.5 * x * (1.0 - th * th) * du)


def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention_fwd(q, k, v):
    """Causal scaled dot-product attention for one head; q, k, v are [S, d]."""
    S, d = q.shape
    s = (q @ k.T) / np.sqrt(d)
    mask = np.triu(np.ones((S, S), dtype=bool), 1)
    s = np.where(mask, -np.inf, s)
    p = softmax_rows(s)
    return p @ v, p


def attention_bwd(q, k, v, p, do):
    S, d = q.shape
    dv = p.T @ do
    dp = do @ v.T
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    ds = ds / np.sqrt(d)
    return ds @ k, ds.T @ q, dv


def mha_fwd(qkv, n_heads):
    """qkv [B, S, 3h] with q | k | v in thirds, head j in columns j*d..(j+1)*d of each
    third.  Returns context [B, S, h] and the per-head probabilities."""
    B, S, h3 = qkv.shape
    h = h3 // 3
    d = h // n_heads
    ctx = np.empty((B, S, h), dtype=qkv.dtype)
    probs = {}
    for b in range(B):
        for j in range(n_heads):
            q = qkv[b, :, j * d:(j + 1) * d]
            k = qkv[b, :, h + j * d:h + (j + 1) * d]
            v = qkv[b, :, 2 * h + j * d:2 * h + (j + 1) * d]
            o, p = attention_fwd(q, k, v)
            ctx[b, :, j * d:(j + 1) * d] = o
            probs[b, j] = p
    return ctx, probs


def mha_bwd(qkv, n_heads, probs, dctx):
    B, S, h3 = qkv.shape
    h = h3 // 3
    d = h // n_heads
    dqkv = np.empty_like(qkv)
    for b in range(B):
        for j in range(n_heads):
            sl = [slice(c * h + j * d, c * h + (j + 1) * d) for c in range(3)]
            dq, dk, dv = attention_bwd(qkv[b, :, sl[0]], qkv[b, :, sl[1]], qkv[b, :, sl[2]],
                                       probs[b, j], dctx[b, :, sl[0]])
            dqkv[b, :, sl[0]] = dq
            dqkv[b, :, sl[1]] = dk
            dqkv[b, :, sl[2]] = dv
    return dqkv


def cross_entropy_fwd_bwd(logits, labels):
    """Mean over rows of -log softmax(logits)[label]; gradient (p - onehot)/rows."""
    n = logits.shape[0]
    m = logits.max(axis=-1, keepdims=True)
    z = logits - m
    lse = np.log(np.exp(z).sum(axis=-1, keepdims=True))
    logp = z - lse
    loss = float(-logp[np.arange(n), labels].mean())
    d = np.exp(logp)
    d[np.arange(n), labels] -= 1.0
    return loss, d / n


# ----------------------------------------------------------------- MLP (config 1)
def mlp_step(Ws, bs, x, target):
    """L x (Linear + ReLU), MSE loss.  Returns loss, dWs, dbs, activations list."""
    acts = [x]
    zs = []
    for W, b in zip(Ws, bs):
        z = linear_fwd(acts[-1], W, b)
        zs.append(z)
        acts.append(relu_fwd(z))
    loss, dy = mse_fwd_bwd(acts[-1], target)
    dWs, dbs = [None] * len(Ws), [None] * len(Ws)
    for i in range(len(Ws) - 1, -1, -1):
        dz = relu_bwd(zs[i], dy)
        dy, dWs[i], dbs[i] = linear_bwd(acts[i], Ws[i], dz)
    return loss, dWs, dbs, acts


# ----------------------------------------------------------------- GPT (configs 2, 4, 5)
BLOCK_TENSORS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
                 "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def block_fwd(p, x, n_heads):
    """x [B, S, h].  Returns y and a cache for backward."""
    B, S, h = x.shape
    x2 = x.reshape(B * S, h)
    a, c1 = layernorm_fwd(x2, p["ln1_g"], p["ln1_b"])
    qkv = linear_fwd(a, p["wqkv"], p["bqkv"])
    ctx, probs = mha_fwd(qkv.reshape(B, S, 3 * h), n_heads)
    ctx2 = ctx.reshape(B * S, h)
    r1 = x2 + linear_fwd(ctx2, p["wo"], p["bo"])
    m, c2 = layernorm_fwd(r1, p["ln2_g"], p["ln2_b"])
    f1 = linear_fwd(m, p["w1"], p["b1"])
    g = gelu_fwd(f1)
    y = r1 + linear_fwd(g, p["w2"], p["b2"])
    cache = dict(c1=c1, a=a, qkv=qkv, probs=probs, ctx=ctx2, r1=r1, c2=c2, m=m, f1=f1, g=g)
    return y.reshape(B, S, h), cache


def block_bwd(p, cache, dy, n_heads):
    B, S, h = dy.shape
    dy2 = dy.reshape(B * S, h)
    grads = {}
    dg, grads["w2"], grads["b2"] = linear_bwd(cache["g"], p["w2"], dy2)
    df1 = gelu_bwd(cache["f1"], dg)
    dm, grads["w1"], grads["b1"] = linear_bwd(cache["m"], p["w1"], df1)
    dr1, grads["ln2_g"], grads["ln2_b"] = layernorm_bwd(dm, p["ln2_g"], cache["c2"])
    dr1 = dr1 + dy2
    dctx, grads["wo"], grads["bo"] = linear_bwd(cache["ctx"], p["wo"], dr1)
    dqkv = mha_bwd(cache["qkv"].reshape(B, S, 3 * h), n_heads, cache["probs"],
                   dctx.reshape(B, S, h))
    da, grads["wqkv"], grads["bqkv"] = linear_bwd(cache["a"], p["wqkv"], dqkv.reshape(B * S, 3 * h))
    dx, grads["ln1_g"], grads["ln1_b"] = layernorm_bwd(da, p["ln1_g"], cache["c1"])
    return (dx + dr1).reshape(B, S, h), grads


def gpt_step(params, ids, labels, n_heads):
    """params: dict(wte [V,h], wpe [S,h], blocks [list of dict], lnf_g, lnf_b).
    ids, labels: int arrays [B, S].  Returns loss, grads (same structure), and the
    list of block inputs/outputs (hidden states)."""
    B, S = ids.shape
    wte, wpe = params["wte"], params["wpe"]
    h = wte.shape[1]
    x = wte[ids] + wpe[np.arange(S)][None, :, :]
    hs = [x]
    caches = []
    for bp in params["blocks"]:
        x, c = block_fwd(bp, x, n_heads)
        caches.append(c)
        hs.append(x)
    xf, cf = layernorm_fwd(x.reshape(B * S, h), params["lnf_g"], params["lnf_b"])
    logits = xf @ wte.T
    loss, dlogits = cross_entropy_fwd_bwd(logits, labels.reshape(-1))
    dwte = dlogits.T @ xf
    dxf = dlogits @ wte
    dx, dlnf_g, dlnf_b = layernorm_bwd(dxf, params["lnf_g"], cf)
    dx = dx.reshape(B, S, h)
    gblocks = [None] * len(params["blocks"])
    dhs = [None] * (len(params["blocks"]) + 1)
    dhs[-1] = dx
    for i in range(len(params["blocks"]) - 1, -1, -1):
        dx, gblocks[i] = block_bwd(params["blocks"][i], caches[i], dx, n_heads)
        dhs[i] = dx
    dwpe = dx.sum(axis=0)
    np.add.at(dwte, ids.reshape(-1), dx.reshape(B * S, h))
    grads = dict(wte=dwte, wpe=dwpe, blocks=gblocks, lnf_g=dlnf_g, lnf_b=dlnf_b)
    return loss, grads, hs, dhs


# ----------------------------------------------------------------- host optimisers
def sgd_update(w, g, lr):
    return w - lr * g


def sgd_momentum_update(w, buf, g, lr, mu):
    """No dampening, no Nesterov: buf = mu*buf + g; w -= lr*buf."""
    buf = mu * buf + g
    return w - lr * buf, buf


def adam_update(w, m, v, g, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """Bias-corrected Adam, no weight decay.  step counts from 1."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return w - lr * mhat / (np.sqrt(vhat) + eps), m, v


def bf16_round(a):
    """Round-to-nearest-even to bfloat16, returned as float32 (the conversion applied
    to the fp32 master weights before they are sent to the device)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32)
    return np.where(np.isnan(a), a, out).reshape(a.shape)
