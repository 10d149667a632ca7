"""bf16 kernels against the oracle, element by element, at sizes that span several
tiles and ragged tails.  Inputs are rounded to bf16 first (that is what the device
holds); the oracle then works in fp64.  Tolerances: a bf16 result carries one
round-to-nearest-even (relative error <= 2^-9 per element, so relative L2 <= 2^-8 with
margin for fp32 accumulation); an fp32 result only carries accumulation error (1e-4)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import nn
import synth_inputs as si

TOL_BF16 = 2.0 ** -8
TOL_F32 = 1e-4


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def bf(a):
    """Round to bf16, return (float64 view of rounded values, torch bf16 device tensor)."""
    import torch
    r = nn.bf16_round(np.asarray(a, dtype=np.float32))
    return r.astype(np.float64), torch.from_numpy(r).to(torch.bfloat16).cuda()


def back(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("m,n,k", [(256, 256, 128), (200, 136, 72), (4, 8, 8), (384, 520, 1032), (1024, 1024, 1024)])
@pytest.mark.parametrize("flags", [0, K.GEMM_A_STRIDED, K.GEMM_B_STRIDED, K.GEMM_A_STRIDED | K.GEMM_B_STRIDED])
def test_gemm_layouts(g, m, n, k, flags):
    import torch
    a, ad = bf(si.normal(1, (m, k)))
    b, bd = bf(si.normal(2, (n, k)))
    ref = a @ b.T
    if flags & K.GEMM_A_STRIDED:
        ad = ad.t().contiguous()
    if flags & K.GEMM_B_STRIDED:
        bd = bd.t().contiguous()
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c), None, None, m, n, k, flags, None, 0, g.stream_ptr())
    assert g.rel_l2(back(c), ref) <= TOL_BF16
    c32 = torch.empty(m, n, dtype=torch.float32, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c32), None, None, m, n, k, flags | K.GEMM_OUT_F32,
           None, 0, g.stream_ptr())
    assert g.rel_l2(back(c32), ref) <= TOL_F32
    # element-wise bound as well: no single entry may be off by more than a few ulps of bf16
    scale = np.abs(a) @ np.abs(b.T)
    assert np.all(np.abs(back(c32) - ref) <= 1e-5 * scale + 1e-30)


@pytest.mark.parametrize("m,n,k", [(256, 256, 64), (4096, 4352, 64), (4096, 4352, 128), (2048, 8704, 192), (128, 256, 32),
                                   (4096, 4352, 32), (8192, 4352, 96), (384, 768, 160)])
@pytest.mark.parametrize("flags", [0, K.GEMM_B_STRIDED, K.GEMM_A_STRIDED | K.GEMM_B_STRIDED])
def test_gemm_whole_tile_shapes_with_few_k_tiles(g, m, n, k, flags):
    """Shapes made of whole 256x256x64 tiles take the direct-to-LDS kernel; with one to three k-tiles
    per output tile and more output tiles than workgroups (272 > 256) its tile stream crosses from one
    work item into the next after every one, two or three tiles.  Reductions that are no multiple of 64 (32, 96,
    160) and row counts that are no multiple of 256 take the register-staged kernel on the same data."""
    import torch
    a, ad = bf(si.normal(11, (m, k)))
    b, bd = bf(si.normal(12, (n, k)))
    ref = a @ b.T
    if flags & K.GEMM_A_STRIDED:
        ad = ad.t().contiguous()
    if flags & K.GEMM_B_STRIDED:
        bd = bd.t().contiguous()
    c32 = torch.empty(m, n, dtype=torch.float32, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c32), None, None, m, n, k, flags | K.GEMM_OUT_F32,
           None, 0, g.stream_ptr())
    assert g.rel_l2(back(c32), ref) <= TOL_F32
    scale = np.abs(a) @ np.abs(b.T)
    assert np.all(np.abs(back(c32) - ref) <= 1e-5 * scale + 1e-30)


def test_gemm_epilogues(g):
    import torch
    m, n, k = 200, 136, 72
    a, ad = bf(si.normal(3, (m, k)))
    b, bd = bf(si.normal(4, (n, k)))
    bias, biasd = bf(si.normal(5, (n,)))
    res, resd = bf(si.normal(6, (m, n)))
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c), g.ptr(biasd), g.ptr(resd), m, n, k, 0, None, 0, g.stream_ptr())
    assert g.rel_l2(back(c), a @ b.T + bias + res) <= TOL_BF16
    acc0 = si.normal(7, (m, n)).astype(np.float32)
    c32 = torch.from_numpy(acc0).cuda()
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c32), None, None, m, n, k,
           K.GEMM_OUT_F32 | K.GEMM_ACCUMULATE, None, 0, g.stream_ptr())
    assert g.rel_l2(back(c32), acc0.astype(np.float64) + a @ b.T) <= TOL_F32


@pytest.mark.parametrize("m,n,k,flags", [(512, 256, 8192, 3), (200, 136, 4096 + 72, 0), (1024, 1024, 32768, 3), (384, 264, 2048, 2)])
def test_gemm_split_k(g, m, n, k, flags):
    """With a workspace the reduction is split over workgroups and summed in a fixed order:
    same tolerance, bit-identical from run to run, epilogues still applied."""
    import torch
    a, ad = bf(si.normal(8, (m, k)))
    b, bd = bf(si.normal(9, (n, k)))
    ref = a @ b.T
    if flags & K.GEMM_A_STRIDED:
        ad = ad.t().contiguous()
    if flags & K.GEMM_B_STRIDED:
        bd = bd.t().contiguous()
    ws = torch.empty(16 * m * n, dtype=torch.float32, device="cuda")
    outs = []
    for _ in range(2):
        c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
        g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c), None, None, m, n, k, flags, g.ptr(ws),
               C.c_uint64(ws.numel() * 4), g.stream_ptr())
        outs.append(c)
    assert g.rel_l2(back(outs[0]), ref) <= TOL_BF16
    assert torch.equal(outs[0], outs[1])
    acc0 = si.normal(7, (m, n)).astype(np.float32)
    c32 = torch.from_numpy(acc0).cuda()
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c32), None, None, m, n, k,
           flags | K.GEMM_OUT_F32 | K.GEMM_ACCUMULATE, g.ptr(ws), C.c_uint64(ws.numel() * 4), g.stream_ptr())
    assert g.rel_l2(back(c32), acc0.astype(np.float64) + ref) <= TOL_F32
    # a workspace that is too small for any split still gives the right answer
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_gemm_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c), None, None, m, n, k, flags, g.ptr(ws),
           C.c_uint64(1024), g.stream_ptr())
    assert g.rel_l2(back(c), ref) <= TOL_BF16


@pytest.mark.parametrize("m,n,k", [(512, 512, 256), (200, 136, 72), (1024, 768, 1024)])
def test_gemm_with_gelu_output_stage(g, m, n, k):
    """The feed-forward products with GELU folded into the kernel's output stage: forward writes the
    pre-activation and its GELU; backward multiplies the product by GELU' of a stored pre-activation."""
    import torch
    a, ad = bf(si.normal(41, (m, k), 0.5))
    b, bd = bf(si.normal(42, (n, k), 0.1))
    bias, biasd = bf(si.normal(43, (n,)))
    pre = a @ b.T + bias
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    act = torch.empty_like(c)
    g.call(K.lib().karma_k_gemm_gelu_bf16, g.ptr(ad), g.ptr(bd), g.ptr(c), g.ptr(biasd), g.ptr(act), m, n, k, 0,
           K.GEMM_GELU_FWD, g.stream_ptr())
    assert g.rel_l2(back(c), pre) <= TOL_BF16
    # the activation is taken of the value as stored (one rounding away from the exact pre-activation)
    assert g.rel_l2(back(act), nn.gelu_fwd(back(c))) <= TOL_BF16
    assert g.rel_l2(back(act), nn.gelu_fwd(pre)) <= 2 * TOL_BF16
    # backward: dy [m][k2] times w [k2][n] (strided operand, as in dX = dY W), times GELU'(pre)
    x, xd = bf(si.normal(44, (m, n), 2.0))
    w, wd = bf(si.normal(45, (n, k), 0.1))      # [n][k] -> product over k of a[m][k] w[n][k]
    wt = wd.t().contiguous()                     # stored [k][n]: strided B operand
    dx = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_gemm_gelu_bf16, g.ptr(ad), g.ptr(wt), g.ptr(dx), None, g.ptr(xd), m, n, k, K.GEMM_B_STRIDED,
           K.GEMM_GELU_BWD, g.stream_ptr())
    assert g.rel_l2(back(dx), nn.gelu_bwd(x, a @ w.T)) <= TOL_BF16
    lib = K.lib()
    assert lib.karma_k_gemm_gelu_bf16(g.ptr(ad), g.ptr(bd), g.ptr(c), None, None, m, n, k, 0, K.GEMM_GELU_FWD, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_gelu_bf16(g.ptr(ad), g.ptr(bd), g.ptr(c), None, g.ptr(act), m, n, k, 0, 3, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_gelu_bf16(g.ptr(ad), g.ptr(bd), g.ptr(c), None, g.ptr(act), m, n, k, K.GEMM_OUT_F32, 1, g.stream_ptr()) == K.E_INVAL


def test_gemm_rejects_bad_shapes(g):
    import torch
    t = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    lib = K.lib()
    assert lib.karma_k_gemm_bf16(g.ptr(t), g.ptr(t), g.ptr(t), None, None, 8, 8, 12, 0, None, 0, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_bf16(g.ptr(t), g.ptr(t), g.ptr(t), None, None, 6, 8, 8, K.GEMM_A_STRIDED, None, 0, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_bf16(g.ptr(t), g.ptr(t), g.ptr(t), None, None, 8, 8, 8, K.GEMM_ACCUMULATE, None, 0, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_gemm_bf16(None, g.ptr(t), g.ptr(t), None, None, 8, 8, 8, 0, None, 0, g.stream_ptr()) == K.E_INVAL


TOL_ATTN = 1e-2   # three chained bf16 roundings (probabilities, dS, result), each <= 2^-9


@pytest.mark.parametrize("m,n,k", [(512, 512, 256), (768, 256, 128), (200, 136, 72)])
def test_gemm_gelu_backward_with_column_sums(g, m, n, k):
    """dX = (dY W) * GELU'(pre) with the column sums of dX (the bias gradient of the layer before the GELU) taken
    in the same launch where the shape is made of whole tiles, by a pass over the result otherwise."""
    import torch
    a, ad = bf(si.normal(46, (m, k), 0.5))
    w, wd = bf(si.normal(47, (n, k), 0.1))
    x, xd = bf(si.normal(48, (m, n), 2.0))
    wt = wd.t().contiguous()
    dx = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    sums = torch.empty(n, device="cuda")
    nws = ((m + 63) // 64) * n
    ws = torch.empty(nws, device="cuda")
    lib = K.lib()
    g.call(lib.karma_k_gemm_gelu_bwd_colsum_bf16, g.ptr(ad), g.ptr(wt), g.ptr(dx), g.ptr(xd), g.ptr(sums), g.ptr(ws),
           C.c_uint64(nws * 4), m, n, k, g.stream_ptr())
    ref = nn.gelu_bwd(x, a @ w.T)
    assert g.rel_l2(back(dx), ref) <= TOL_BF16
    # a sum of m values each carrying up to one bf16 rounding (only when the result was stored before summing)
    assert g.rel_l2(sums.cpu().numpy(), ref.sum(0)) <= TOL_BF16
    # the same bits as the plain entry point gives for dX
    dx2 = torch.empty_like(dx)
    g.call(lib.karma_k_gemm_gelu_bf16, g.ptr(ad), g.ptr(wt), g.ptr(dx2), None, g.ptr(xd), m, n, k, K.GEMM_B_STRIDED,
           K.GEMM_GELU_BWD, g.stream_ptr())
    assert torch.equal(dx, dx2)
    assert lib.karma_k_gemm_gelu_bwd_colsum_bf16(g.ptr(ad), g.ptr(wt), g.ptr(dx), g.ptr(xd), g.ptr(sums), g.ptr(ws),
                                                 C.c_uint64(16), m, n, k, g.stream_ptr()) == K.E_OOM


@pytest.mark.parametrize("rows,h", [(64, 1024), (37, 256), (5, 3072), (130, 4256), (3, 8)])
def test_layernorm(g, rows, h):
    import torch
    x, xd = bf(si.normal(11, (rows, h), 2.0) + 0.5)
    gam, gd = bf(1.0 + si.normal(12, (h,), 0.2))
    bet, bd = bf(si.normal(13, (h,), 0.2))
    dy, dyd = bf(si.normal(14, (rows, h)))
    add, addd = bf(si.normal(15, (rows, h)))
    y = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    stats = torch.empty(rows, 2, device="cuda")
    lib = K.lib()
    g.call(lib.karma_k_layernorm_fwd_bf16, g.ptr(xd), g.ptr(gd), g.ptr(bd), g.ptr(y), g.ptr(stats), rows, h, g.stream_ptr())
    yo, cache = nn.layernorm_fwd(x, gam, bet)
    assert g.rel_l2(back(y), yo) <= TOL_BF16
    ratio = g.elem_ratio(back(y), yo, 1, 1e-3)
    assert ratio <= 1, ratio
    assert g.rel_l2(stats[:, 0].cpu().numpy(), x.mean(-1)) <= TOL_F32 + 1e-6
    assert g.rel_l2(stats[:, 1].cpu().numpy(), cache[1].reshape(-1)) <= TOL_F32
    dx = torch.empty_like(y)
    dg = torch.empty(h, device="cuda"); db = torch.empty(h, device="cuda")
    nws = ((rows + 63) // 64) * 3 * h
    ws = torch.empty(nws, device="cuda")
    for use_add in (False, True):
        g.call(lib.karma_k_layernorm_bwd_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), g.ptr(addd) if use_add else None,
               g.ptr(dx), g.ptr(dg), g.ptr(db), g.ptr(ws), C.c_uint64(nws * 4), rows, h, g.stream_ptr())
        dxo, dgo, dbo = nn.layernorm_bwd(dy, gam, cache)
        if use_add:
            dxo = dxo + add
        assert g.rel_l2(back(dx), dxo) <= TOL_BF16
        ratio = g.elem_ratio(back(dx), dxo, 1, 1e-3)
        assert ratio <= 1, (ratio, use_add)
        assert g.rel_l2(dg.cpu().numpy(), dgo) <= TOL_F32 * 10
        assert g.rel_l2(db.cpu().numpy(), dbo) <= TOL_F32
    # the variant that also sums the added tensor's columns (a bias gradient) in the same pass
    dx2 = torch.empty_like(y)
    dg2 = torch.empty(h, device="cuda"); db2 = torch.empty(h, device="cuda"); asum = torch.empty(h, device="cuda")
    g.call(lib.karma_k_layernorm_bwd_addsum_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), g.ptr(addd), g.ptr(dx2),
           g.ptr(dg2), g.ptr(db2), g.ptr(asum), g.ptr(ws), C.c_uint64(nws * 4), rows, h, g.stream_ptr())
    assert torch.equal(dx2, dx) and torch.equal(dg2, dg) and torch.equal(db2, db)
    assert g.rel_l2(asum.cpu().numpy(), add.sum(0)) <= TOL_F32
    assert lib.karma_k_layernorm_bwd_addsum_bf16(g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), None, g.ptr(dx2), g.ptr(dg2),
                                                 g.ptr(db2), g.ptr(asum), g.ptr(ws), C.c_uint64(nws * 4), rows, h,
                                                 g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_layernorm_bwd_bf16(g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), None, g.ptr(dx), g.ptr(dg),
                                          g.ptr(db), g.ptr(ws), C.c_uint64(8), rows, h, g.stream_ptr()) == K.E_OOM


@pytest.mark.parametrize("rows,cols", [(1000, 4096), (129, 24), (1, 8), (300, 2056)])
def test_colsum(g, rows, cols):
    import torch
    x, xd = bf(si.normal(21, (rows, cols)))
    out = torch.empty(cols, device="cuda")
    nws = ((rows + 63) // 64) * cols
    ws = torch.empty(nws, device="cuda")
    g.call(K.lib().karma_k_colsum_bf16, g.ptr(xd), g.ptr(out), g.ptr(ws), C.c_uint64(nws * 4), rows, cols, g.stream_ptr())
    assert g.rel_l2(out.cpu().numpy(), x.sum(0)) <= TOL_F32


@pytest.mark.parametrize("n", [8, 4096 * 33, 1000 * 8])
def test_gelu(g, n):
    import torch
    x, xd = bf(si.normal(31, (n,), 2.0))
    dy, dyd = bf(si.normal(32, (n,)))
    y = torch.empty(n, dtype=torch.bfloat16, device="cuda"); dx = torch.empty_like(y)
    g.call(K.lib().karma_k_gelu_fwd_bf16, g.ptr(xd), g.ptr(y), C.c_uint64(n), g.stream_ptr())
    g.call(K.lib().karma_k_gelu_bwd_bf16, g.ptr(xd), g.ptr(dyd), g.ptr(dx), C.c_uint64(n), g.stream_ptr())
    assert g.rel_l2(back(y), nn.gelu_fwd(x)) <= TOL_BF16
    assert g.rel_l2(back(dx), nn.gelu_bwd(x, dy)) <= TOL_BF16
    # element by element: one bf16 rounding, plus the hardware exponential's error where the result is a
    # small difference (1e-4 of a typical element)
    ratio = g.elem_ratio(back(y), nn.gelu_fwd(x), 1, 1e-4, axis=None)
    assert ratio <= 1, ratio
    ratio = g.elem_ratio(back(dx), nn.gelu_bwd(x, dy), 1, 1e-4, axis=None)
    assert ratio <= 1, ratio


def sort_tokens(ids):
    """Host-side preparation the step does for the embedding gradient: stable sort of
    token positions by id and the run boundaries."""
    flat = ids.reshape(-1)
    order = np.argsort(flat, kind="stable").astype(np.int32)
    sid = flat[order]
    starts = np.flatnonzero(np.r_[True, sid[1:] != sid[:-1]]).astype(np.int32)
    return order, np.r_[starts, len(flat)].astype(np.int32), sid[starts].astype(np.int32)


def test_embedding(g):
    import torch
    B, S, h, V = 3, 16, 64, 50
    wte, wted = bf(si.normal(41, (V, h)))
    wpe, wped = bf(si.normal(42, (S, h)))
    ids = si.randint(43, (B, S), V).astype(np.int32)
    ids[0, :5] = 7
    out = torch.empty(B * S, h, dtype=torch.bfloat16, device="cuda")
    idd = g.dev(ids.reshape(-1))
    g.call(K.lib().karma_k_embed_fwd_bf16, g.ptr(idd), g.ptr(wted), g.ptr(wped), g.ptr(out), B * S, S, h, g.stream_ptr())
    ref = wte[ids] + wpe[np.arange(S)][None]
    assert g.rel_l2(back(out), ref.reshape(B * S, h)) <= TOL_BF16
    dx, dxd = bf(si.normal(44, (B * S, h)))
    order, starts, segid = sort_tokens(ids)
    base = si.normal(45, (V, h)).astype(np.float32)
    dwte = torch.from_numpy(base.copy()).cuda()
    dwpe = torch.empty(S, h, dtype=torch.bfloat16, device="cuda")
    od, sd, gd = g.dev(order), g.dev(starts), g.dev(segid)     # keep the device copies alive
    g.call(K.lib().karma_k_embed_bwd_bf16, g.ptr(dxd), g.ptr(od), g.ptr(sd), g.ptr(gd),
           len(segid), g.ptr(dwte), g.ptr(dwpe), B, S, h, g.stream_ptr())
    refw = base.astype(np.float64)
    np.add.at(refw, ids.reshape(-1), dx)
    assert g.rel_l2(dwte.cpu().numpy(), refw) <= TOL_F32
    assert g.rel_l2(back(dwpe), dx.reshape(B, S, h).sum(0)) <= TOL_BF16


@pytest.mark.parametrize("rows,cols", [(7, 32000), (300, 51200), (5, 8), (64, 1000)])
def test_softmax_cross_entropy(g, rows, cols):
    import torch
    z, zd = bf(si.normal(51, (rows, cols), 3.0))
    labels = si.randint(52, (rows,), cols).astype(np.int32)
    rowloss = torch.empty(rows, device="cuda")
    scale = 1.0 / rows
    labd = g.dev(labels)
    g.call(K.lib().karma_k_softmax_ce_bf16, g.ptr(zd), g.ptr(labd), g.ptr(rowloss), rows, cols, C.c_float(scale),
           g.stream_ptr())
    loss, d = nn.cross_entropy_fwd_bwd(z, labels)
    out = torch.zeros(1, device="cuda"); ws = torch.empty(1024, device="cuda")
    g.call(K.lib().karma_k_sum_f32, g.ptr(rowloss), g.ptr(out), g.ptr(ws), C.c_uint64(rows), C.c_float(scale), g.stream_ptr())
    assert abs(out.item() - loss) <= TOL_F32 * abs(loss)
    assert g.rel_l2(back(zd), d) <= TOL_BF16
    # every gradient entry: one bf16 rounding of a probability (the label's entry is p - 1: a difference)
    ratio = g.elem_ratio(back(zd), d, 1, 1e-3)
    assert ratio <= 1, ratio
    # uniform logits: loss ln(cols), gradient rows sum to ~0
    zd.zero_()
    g.call(K.lib().karma_k_softmax_ce_bf16, g.ptr(zd), g.ptr(labd), g.ptr(rowloss), rows, cols, C.c_float(1.0),
           g.stream_ptr())
    assert np.allclose(rowloss.cpu().numpy(), np.log(cols), rtol=1e-5)


@pytest.mark.parametrize("B,S,H,D", [(2, 256, 3, 64), (1, 128, 1, 64), (1, 384, 2, 128), (2, 1024, 2, 64),
                                     (1, 384, 2, 152), (2, 256, 3, 152)])
def test_attention(g, B, S, H, D):
    import torch
    h = H * D
    qkv, qkvd = bf(si.normal(61, (B, S, 3 * h), 1.5))
    dctx, dctxd = bf(si.normal(62, (B, S, h)))
    ctx = torch.empty(B, S, h, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(B, H, S, device="cuda")
    lib = K.lib()
    g.call(lib.karma_k_attention_fwd_bf16, g.ptr(qkvd), g.ptr(ctx), g.ptr(lse), B, S, H, D, g.stream_ptr())
    ctxo, probs = nn.mha_fwd(qkv, H)
    assert g.rel_l2(back(ctx), ctxo) <= TOL_ATTN
    # every entry of every query row: the result's own rounding plus the probabilities' (2^-9 each,
    # weighted by |v|, which does not cancel: a share of the row's size)
    ratio = g.elem_ratio(back(ctx), ctxo, 1, 2.0 ** -6)
    assert ratio <= 1, ratio
    # lse in the base-2 domain of the scaled scores
    q = qkv[0, :, :D]; k = qkv[0, :, h:h + D]
    s = (q @ k.T) / np.sqrt(D)
    s[np.triu(np.ones((S, S), bool), 1)] = -np.inf
    lse_ref = (np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)) / np.log(2)
    assert np.allclose(lse[0, 0].cpu().numpy(), lse_ref, rtol=1e-4, atol=1e-4)
    dqkv = torch.zeros(B, S, 3 * h, dtype=torch.bfloat16, device="cuda")
    delta = torch.empty(B, H, S, device="cuda")
    g.call(lib.karma_k_attention_bwd_bf16, g.ptr(qkvd), g.ptr(ctx), g.ptr(dctxd), g.ptr(lse), g.ptr(delta), g.ptr(dqkv),
           B, S, H, D, g.stream_ptr())
    dqkvo = nn.mha_bwd(qkv, H, probs, dctx)
    got = back(dqkv)
    for name, sl in (("dq", slice(0, h)), ("dk", slice(h, 2 * h)), ("dv", slice(2 * h, 3 * h))):
        assert g.rel_l2(got[:, :, sl], dqkvo[:, :, sl]) <= TOL_ATTN, name
        # per head, every element against the size of that head's gradient (the rounding of the stored
        # context enters every row through delta = rowsum(dO * O), whatever the row's own size): a wrong
        # row cannot hide in the norm.  Three chained roundings leave errors of about 1 % of the head's
        # size (the relative L2 above); the largest of 10^5..10^6 of them reaches 5 %, the bound is 2^-4
        for hd in range(H):
            a, b = got[:, :, sl][:, :, hd * D:(hd + 1) * D], dqkvo[:, :, sl][:, :, hd * D:(hd + 1) * D]
            ratio = g.elem_ratio(a, b, 1, 2.0 ** -4, axis=(1, 2))
            assert ratio <= 1, (ratio, (name, hd))
    # a second run gives the same bits (no atomics)
    dqkv2 = torch.zeros_like(dqkv)
    g.call(lib.karma_k_attention_bwd_bf16, g.ptr(qkvd), g.ptr(ctx), g.ptr(dctxd), g.ptr(lse), g.ptr(delta), g.ptr(dqkv2),
           B, S, H, D, g.stream_ptr())
    assert torch.equal(dqkv, dqkv2)


@pytest.mark.parametrize("B,S,H,D", [(2, 256, 3, 64), (1, 1024, 2, 64), (1, 256, 2, 128)])
def test_attention_backward_with_qkv_bias_gradient(g, B, S, H, D):
    """The backward pass also delivering the column sums of dqkv over all tokens (the QKV bias gradient): inside the
    kernels for head dimension 64, by a pass over dqkv otherwise; dqkv itself is unchanged."""
    import torch
    h = H * D
    qkv, qkvd = bf(si.normal(63, (B, S, 3 * h), 1.5))
    dctx, dctxd = bf(si.normal(64, (B, S, h)))
    ctx = torch.empty(B, S, h, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(B, H, S, device="cuda")
    lib = K.lib()
    g.call(lib.karma_k_attention_fwd_bf16, g.ptr(qkvd), g.ptr(ctx), g.ptr(lse), B, S, H, D, g.stream_ptr())
    delta = torch.empty(B, H, S, device="cuda")
    ref = torch.zeros(B, S, 3 * h, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_attention_bwd_bf16, g.ptr(qkvd), g.ptr(ctx), g.ptr(dctxd), g.ptr(lse), g.ptr(delta), g.ptr(ref),
           B, S, H, D, g.stream_ptr())
    dqkv = torch.zeros_like(ref)
    sums = torch.empty(3 * h, device="cuda")
    nws = max(B * S // 32, (B * S + 63) // 64) * 3 * h
    ws = torch.empty(nws, device="cuda")
    g.call(lib.karma_k_attention_bwd_colsum_bf16, g.ptr(qkvd), g.ptr(ctx), g.ptr(dctxd), g.ptr(lse), g.ptr(delta), g.ptr(dqkv),
           g.ptr(sums), g.ptr(ws), C.c_uint64(nws * 4), B, S, H, D, g.stream_ptr())
    assert torch.equal(dqkv, ref)
    _, probs = nn.mha_fwd(qkv, H)
    want = nn.mha_bwd(qkv, H, probs, dctx).reshape(B * S, 3 * h).sum(0)
    assert g.rel_l2(sums.cpu().numpy(), want) <= TOL_ATTN
    assert lib.karma_k_attention_bwd_colsum_bf16(g.ptr(qkvd), g.ptr(ctx), g.ptr(dctxd), g.ptr(lse), g.ptr(delta), g.ptr(dqkv),
                                                 g.ptr(sums), g.ptr(ws), C.c_uint64(64), B, S, H, D, g.stream_ptr()) == K.E_OOM


def test_attention_rejects_unsupported(g):
    import torch
    t = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda"); f = torch.zeros(1 << 12, device="cuda")
    lib = K.lib()
    assert lib.karma_k_attention_fwd_bf16(g.ptr(t), g.ptr(t), g.ptr(f), 1, 100, 1, 64, g.stream_ptr()) == K.E_INVAL
    assert lib.karma_k_attention_fwd_bf16(g.ptr(t), g.ptr(t), g.ptr(f), 1, 128, 1, 96, g.stream_ptr()) == K.E_INVAL
