"""Parity at the benchmark's full sizes (configs[1]: 32768 tokens, hidden 1024, FFN 4096,
vocabulary 32000, 16 heads), in the launch configurations bench.py times.  The oracle
cannot compute whole results at these sizes in seconds, so it computes sampled outputs
one by one (rows, heads, entries) from the same seeded inputs."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import nn
import synth_inputs as si
from test_gpu_bf16_kernels import TOL_ATTN, TOL_BF16, TOL_F32, back

T, H, FFN, V, HEADS, S, B = 32768, 1024, 4096, 32000, 16, 1024, 32


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def dev_normal(seed, shape, std=1.0):
    """Large seeded bf16 tensor: generated on the host in fp32, rounded to bf16."""
    import torch
    a = si.normal(seed, shape, std).astype(np.float32)
    t = torch.from_numpy(a).to(torch.bfloat16).cuda()
    return t


def rows_of(t, idx):
    return t[idx].float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("m,n,k,flags,use_ws", [(T, FFN, H, 0, False), (T, H, FFN, K.GEMM_B_STRIDED, False),
                                                (FFN, H, T, K.GEMM_A_STRIDED | K.GEMM_B_STRIDED, True),
                                                (4096, V, H, 0, False)])
def test_gemm_full_size_sampled_entries(g, m, n, k, flags, use_ws):
    import torch
    a = dev_normal(101, (k, m) if flags & K.GEMM_A_STRIDED else (m, k))
    b = dev_normal(102, (k, n) if flags & K.GEMM_B_STRIDED else (n, k))
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(8 * m * n, dtype=torch.float32, device="cuda") if use_ws else None
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(a), g.ptr(b), g.ptr(c), None, None, m, n, k, flags,
           g.ptr(ws) if use_ws else None, C.c_uint64(ws.numel() * 4 if use_ws else 0), g.stream_ptr())
    rng = np.random.default_rng(5)
    ms = np.r_[0, m - 1, rng.integers(0, m, 30)]
    ns = np.r_[0, n - 1, rng.integers(0, n, 30)]
    A = (a[:, ms].t() if flags & K.GEMM_A_STRIDED else a[ms]).float().cpu().numpy().astype(np.float64)   # [32, k]
    Bm = (b[:, ns].t() if flags & K.GEMM_B_STRIDED else b[ns]).float().cpu().numpy().astype(np.float64)
    ref = A @ Bm.T
    got = c[ms][:, ns].float().cpu().numpy()
    assert g.rel_l2(got, ref) <= TOL_BF16
    assert np.all(np.abs(got - ref) <= 2.0 ** -7 * (np.abs(A) @ np.abs(Bm.T)) / np.sqrt(k) * 8 + 1e-6)


def test_gemm_with_gelu_full_size_sampled_entries(g):
    """The feed-forward products as the benchmark step launches them: FC1 with GELU written beside the
    pre-activation, and dY W2 multiplied by GELU' of the stored pre-activation."""
    import torch
    m, n, k = T, FFN, H
    a = dev_normal(111, (m, k), 0.5)
    w = dev_normal(112, (n, k), 0.05)
    bias = dev_normal(113, (n,), 0.5)
    pre = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    act = torch.empty_like(pre)
    g.call(K.lib().karma_k_gemm_gelu_bf16, g.ptr(a), g.ptr(w), g.ptr(pre), g.ptr(bias), g.ptr(act), m, n, k, 0,
           K.GEMM_GELU_FWD, g.stream_ptr())
    rng = np.random.default_rng(6)
    ms = np.r_[0, m - 1, rng.integers(0, m, 30)]
    ns = np.r_[0, n - 1, rng.integers(0, n, 30)]
    A = rows_of(a, ms)
    W = rows_of(w, ns)
    ref = A @ W.T + bias[ns].float().cpu().numpy().astype(np.float64)
    got_pre = pre[ms][:, ns].float().cpu().numpy().astype(np.float64)
    got_act = act[ms][:, ns].float().cpu().numpy().astype(np.float64)
    assert g.rel_l2(got_pre, ref) <= TOL_BF16
    assert g.rel_l2(got_act, nn.gelu_fwd(got_pre)) <= TOL_BF16
    # backward: dy [m][k] times W2 stored [k][n] (strided operand), times GELU'(pre)
    w2 = dev_normal(114, (k, n), 0.05)
    dx = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_gemm_gelu_bf16, g.ptr(a), g.ptr(w2), g.ptr(dx), None, g.ptr(pre), m, n, k, K.GEMM_B_STRIDED,
           K.GEMM_GELU_BWD, g.stream_ptr())
    W2 = w2[:, ns].t().float().cpu().numpy().astype(np.float64)
    ref_dx = nn.gelu_bwd(got_pre, A @ W2.T)
    assert g.rel_l2(dx[ms][:, ns].float().cpu().numpy(), ref_dx) <= TOL_BF16
    # the same launch leaving the column sums of dx (FC1's bias gradient): three columns summed over all rows
    dx3 = torch.empty_like(dx)
    sums = torch.empty(n, device="cuda")
    nws = (m // 64) * n
    ws = torch.empty(nws, device="cuda")
    g.call(K.lib().karma_k_gemm_gelu_bwd_colsum_bf16, g.ptr(a), g.ptr(w2), g.ptr(dx3), g.ptr(pre), g.ptr(sums), g.ptr(ws),
           C.c_uint64(nws * 4), m, n, k, g.stream_ptr())
    assert torch.equal(dx3, dx)
    cols = [0, 1777, n - 1]
    a_all = a.float().cpu().numpy().astype(np.float64)
    pre_c = pre[:, cols].float().cpu().numpy().astype(np.float64)
    w2_c = w2[:, cols].float().cpu().numpy().astype(np.float64)
    ref_sum = nn.gelu_bwd(pre_c, a_all @ w2_c).sum(0)
    assert g.rel_l2(sums[cols].cpu().numpy(), ref_sum) <= TOL_BF16


def test_attention_full_size_sampled_heads(g):
    import torch
    qkv = dev_normal(111, (B, S, 3 * H), 1.2)
    dctx = dev_normal(112, (B, S, H))
    ctx = torch.empty(B, S, H, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(B, HEADS, S, device="cuda")
    dqkv = torch.empty_like(qkv)
    delta = torch.empty(B, HEADS, S, device="cuda")
    lib = K.lib()
    g.call(lib.karma_k_attention_fwd_bf16, g.ptr(qkv), g.ptr(ctx), g.ptr(lse), B, S, HEADS, 64, g.stream_ptr())
    g.call(lib.karma_k_attention_bwd_bf16, g.ptr(qkv), g.ptr(ctx), g.ptr(dctx), g.ptr(lse), g.ptr(delta), g.ptr(dqkv),
           B, S, HEADS, 64, g.stream_ptr())
    for (b, hd) in [(0, 0), (31, 15), (7, 9)]:
        sl = [slice(c * H + hd * 64, c * H + (hd + 1) * 64) for c in range(3)]
        q, k, v = (qkv[b, :, s_].float().cpu().numpy().astype(np.float64) for s_ in sl)
        do = dctx[b, :, sl[0]].float().cpu().numpy().astype(np.float64)
        o, p = nn.attention_fwd(q, k, v)
        assert g.rel_l2(back(ctx[b, :, sl[0]]), o) <= TOL_ATTN
        ratio = g.elem_ratio(back(ctx[b, :, sl[0]]), o, 1, 2.0 ** -6)
        assert ratio <= 1, (ratio, (b, hd))
        dq, dk, dv = nn.attention_bwd(q, k, v, p, do)
        for name, ref, s_ in (("dq", dq, sl[0]), ("dk", dk, sl[1]), ("dv", dv, sl[2])):
            assert g.rel_l2(back(dqkv[b, :, s_]), ref) <= TOL_ATTN, (b, hd, name)
            ratio = g.elem_ratio(back(dqkv[b, :, s_]), ref, 1, 2.0 ** -4, axis=None)
            assert ratio <= 1, (ratio, (b, hd, name))


def test_attention_head_dimension_152_full_shape_sampled_heads(g):
    """The attention shape of the 17B-parameter configuration: batch 4, 28 heads of 152, 1024 tokens."""
    import torch
    b_, heads, d = 4, 28, 152
    h = heads * d
    qkv = dev_normal(113, (b_, S, 3 * h), 1.2)
    dctx = dev_normal(114, (b_, S, h))
    ctx = torch.empty(b_, S, h, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(b_, heads, S, device="cuda")
    dqkv = torch.empty_like(qkv)
    delta = torch.empty(b_, heads, S, device="cuda")
    lib = K.lib()
    g.call(lib.karma_k_attention_fwd_bf16, g.ptr(qkv), g.ptr(ctx), g.ptr(lse), b_, S, heads, d, g.stream_ptr())
    g.call(lib.karma_k_attention_bwd_bf16, g.ptr(qkv), g.ptr(ctx), g.ptr(dctx), g.ptr(lse), g.ptr(delta), g.ptr(dqkv),
           b_, S, heads, d, g.stream_ptr())
    for (b, hd) in [(0, 0), (3, 27), (2, 13)]:
        sl = [slice(c * h + hd * d, c * h + (hd + 1) * d) for c in range(3)]
        q, k, v = (qkv[b, :, s_].float().cpu().numpy().astype(np.float64) for s_ in sl)
        do = dctx[b, :, sl[0]].float().cpu().numpy().astype(np.float64)
        o, p = nn.attention_fwd(q, k, v)
        assert g.rel_l2(back(ctx[b, :, sl[0]]), o) <= TOL_ATTN
        ratio = g.elem_ratio(back(ctx[b, :, sl[0]]), o, 1, 2.0 ** -6)
        assert ratio <= 1, (ratio, (b, hd))
        dq, dk, dv = nn.attention_bwd(q, k, v, p, do)
        for name, ref, s_ in (("dq", dq, sl[0]), ("dk", dk, sl[1]), ("dv", dv, sl[2])):
            assert g.rel_l2(back(dqkv[b, :, s_]), ref) <= TOL_ATTN, (b, hd, name)
            ratio = g.elem_ratio(back(dqkv[b, :, s_]), ref, 1, 2.0 ** -4, axis=None)
            assert ratio <= 1, (ratio, (b, hd, name))


def test_rowwise_kernels_full_size_sampled_rows(g):
    import torch
    lib = K.lib()
    rng = np.random.default_rng(9)
    rows = np.r_[0, T - 1, rng.integers(0, T, 14)]
    # LayerNorm forward / backward
    x = dev_normal(121, (T, H), 2.0)
    gam = dev_normal(122, (H,), 0.2) + 1
    bet = dev_normal(123, (H,), 0.2)
    dy = dev_normal(124, (T, H))
    y = torch.empty_like(x); dx = torch.empty_like(x)
    stats = torch.empty(T, 2, device="cuda")
    dg = torch.empty(H, device="cuda"); db = torch.empty(H, device="cuda")
    nws = (T // 64) * 3 * H
    ws = torch.empty(nws, device="cuda")
    g.call(lib.karma_k_layernorm_fwd_bf16, g.ptr(x), g.ptr(gam), g.ptr(bet), g.ptr(y), g.ptr(stats), T, H, g.stream_ptr())
    g.call(lib.karma_k_layernorm_bwd_bf16, g.ptr(dy), g.ptr(x), g.ptr(stats), g.ptr(gam), None, g.ptr(dx), g.ptr(dg),
           g.ptr(db), g.ptr(ws), C.c_uint64(nws * 4), T, H, g.stream_ptr())
    xo, go, bo, dyo = rows_of(x, rows), back(gam), back(bet), rows_of(dy, rows)
    yo, cache = nn.layernorm_fwd(xo, go, bo)
    assert g.rel_l2(rows_of(y, rows), yo) <= TOL_BF16
    ratio = g.elem_ratio(rows_of(y, rows), yo, 1, 1e-3)
    assert ratio <= 1, ratio
    dxo, _, _ = nn.layernorm_bwd(dyo, go, cache)
    assert g.rel_l2(rows_of(dx, rows), dxo) <= TOL_BF16
    ratio = g.elem_ratio(rows_of(dx, rows), dxo, 1, 1e-3)
    assert ratio <= 1, ratio
    # the column reductions over all 32768 rows: a few columns in full
    cols = [0, 17, H - 1]
    xc = x[:, cols].float().cpu().numpy().astype(np.float64); dyc = dy[:, cols].float().cpu().numpy().astype(np.float64)
    st = stats.cpu().numpy().astype(np.float64)
    xhat = (xc - st[:, :1]) * st[:, 1:]
    assert g.rel_l2(dg[cols].cpu().numpy(), (dyc * xhat).sum(0)) <= 1e-3
    assert g.rel_l2(db[cols].cpu().numpy(), dyc.sum(0)) <= TOL_F32
    # the variant the transformer block launches: the residual branch's gradient is added to dx and its column
    # sums (a bias gradient) come out of the same pass
    add = dev_normal(125, (T, H))
    dx2 = torch.empty_like(x)
    dg2 = torch.empty(H, device="cuda"); db2 = torch.empty(H, device="cuda"); asum = torch.empty(H, device="cuda")
    g.call(lib.karma_k_layernorm_bwd_addsum_bf16, g.ptr(dy), g.ptr(x), g.ptr(stats), g.ptr(gam), g.ptr(add), g.ptr(dx2),
           g.ptr(dg2), g.ptr(db2), g.ptr(asum), g.ptr(ws), C.c_uint64(nws * 4), T, H, g.stream_ptr())
    assert g.rel_l2(rows_of(dx2, rows), dxo + rows_of(add, rows)) <= TOL_BF16
    assert torch.equal(dg2, dg) and torch.equal(db2, db)
    assert g.rel_l2(asum[cols].cpu().numpy(), add[:, cols].float().cpu().numpy().astype(np.float64).sum(0)) <= TOL_F32
    # GELU on the FFN activation
    f = dev_normal(131, (T, FFN), 1.5)
    gy = torch.empty_like(f)
    g.call(lib.karma_k_gelu_fwd_bf16, g.ptr(f), g.ptr(gy), C.c_uint64(T * FFN), g.stream_ptr())
    assert g.rel_l2(rows_of(gy, rows), nn.gelu_fwd(rows_of(f, rows))) <= TOL_BF16
    ratio = g.elem_ratio(rows_of(gy, rows), nn.gelu_fwd(rows_of(f, rows)), 1, 1e-4)
    assert ratio <= 1, ratio
    # softmax cross-entropy on one head chunk (4096 x 32000)
    z = dev_normal(141, (4096, V), 2.0)
    zr = rows_of(z, rows % 4096)
    labels = si.randint(142, (4096,), V).astype(np.int32)
    labd = g.dev(labels)
    rowloss = torch.empty(4096, device="cuda")
    g.call(lib.karma_k_softmax_ce_bf16, g.ptr(z), g.ptr(labd), g.ptr(rowloss), 4096, V, C.c_float(1.0 / T), g.stream_ptr())
    rr = rows % 4096
    for j, r in enumerate(rr):
        loss, d = nn.cross_entropy_fwd_bwd(zr[j:j + 1], labels[r:r + 1])
        assert abs(rowloss[r].item() - loss) <= 1e-4 * abs(loss) + 1e-5
        assert g.rel_l2(rows_of(z, [r]), d / T) <= TOL_BF16
        ratio = g.elem_ratio(rows_of(z, [r]), d / T, 1, 1e-3)
        assert ratio <= 1, ratio
