"""Wide residual network (the WRN-28-10 row of Table III) on the GPU: a small network of
the same structure through the whole step against the oracle, out-of-core plans
bit-identical to the in-core step, the planner's choice equal to the oracle planner's, and
the two kernel forms the pre-activated block adds (a convolution that adds a residual, a
batch-norm backward that adds a shortcut gradient) against the oracle element by element.
Tolerances of the whole step as for the bottleneck network: each gradient tensor within
FLOOR_FACTOR times the distance that bf16 storage alone puts between the plain fp64 oracle
and the same step with bf16 tensors (`tests/test_cnn_bf16_floor.py`), plus half the bar."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import cnn, wrn, planner as P
import synth_inputs as si

import cnn_bf16_storage as S
from test_gpu_bf16_kernels import back, bf

BAR = 2e-2
FLOOR_FACTOR = 2.0
DIMS = S.WRN_SMALL
BT = si.BASIC_TENSORS
TOL = 2.0 ** -8


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def make_ctx(dims, arena, lr=0.05, mu=0.9):
    desc = dict(kind=K.MODEL_WRN, n_layers=0, width=dims["width"], batch=dims["batch"], seq=dims["image"], n_heads=0, ffn=0,
                vocab=dims["classes"], stream_weights=0, stage_blocks=tuple(dims["group_blocks"]) + (0,))
    cfg = dict(optimizer=K.OPT_SGD_MOMENTUM, lr=lr, beta1=mu, beta2=0.0, eps=0.0, host_threads=8)
    return K.Context(desc, cfg, arena)


def pad_stem(w):
    out = np.zeros(w.shape[:3] + (8,), dtype=np.float64)
    out[..., :3] = w
    return out


def load_params(ctx, params):
    ctx.karma_set_param(0, 0, pad_stem(params["stem"]["w"]))
    for i, (p, _) in enumerate(params["blocks"]):
        for t, name in enumerate(BT):
            if name in p:
                ctx.karma_set_param(i + 1, t, p[name])
    L = len(params["blocks"]) + 1
    for t, name in enumerate(("g", "b", "w", "bias")):
        ctx.karma_set_param(L, t, params["head"][name])


def all_grads(ctx, params):
    out = {"stem.w": ctx.karma_get_grad(0, 0)}
    for i, (p, _) in enumerate(params["blocks"]):
        for t, name in enumerate(BT):
            if name in p:
                out["b%d.%s" % (i, name)] = ctx.karma_get_grad(i + 1, t)
    L = len(params["blocks"]) + 1
    for t, name in enumerate(("g", "b", "w", "bias")):
        out["head." + name] = ctx.karma_get_grad(L, t)
    return out


def oracle_grads(grads):
    out = S.flat(grads)
    out["stem.w"] = pad_stem(out["stem.w"])
    return out


@pytest.mark.parametrize("shift", [3.0, 0.0])
def test_wrn_step_matches_oracle_and_plans_are_bit_identical(g, shift):
    params, images, labels = S.wrn_problem(DIMS, shift)
    arena = 256 << 20
    ctx = make_ctx(DIMS, arena)
    n = ctx.n_layers
    assert n == 5
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * n)
    loss = ctx.karma_step(images, labels)
    ref = all_grads(ctx, params)
    pr = S.rounded_params(params)
    lo, go = wrn.wrn_step(pr, images, labels)
    _, gs = S.wrn_step_bf16_storage(pr, images, labels)
    og, sg = oracle_grads(go), oracle_grads(gs)
    assert abs(loss - lo) <= 5e-3 * abs(lo), (loss, lo)
    floor = S.distances(sg, og)
    d = S.distances(ref, og)
    bad = {k: (d[k], floor[k]) for k in d if not d[k] <= 0.5 * BAR + FLOOR_FACTOR * floor[k]}
    assert not bad, bad
    assert np.median([d[k] / (floor[k] + 1e-3) for k in d]) <= 1.25
    assert np.all(ref["stem.w"].reshape(16, 3, 3, 8)[..., 3:] == 0)      # the padding channels see no gradient

    plans = [[K.SWAP] * n, [K.RC_KEEP] * n, [K.KEEP, K.RC_SWAP, K.RC_CHAIN, K.SWAP, K.RC_KEEP],
             [K.RC_KEEP] + [K.RC_CHAIN] * (n - 1), [K.SWAP, K.KEEP, K.RC_KEEP, K.SWAP, K.RC_SWAP]]
    for pl in plans:
        ctx.karma_set_plan(arena, pl)
        assert ctx.karma_step(images, labels) == loss, pl
        for name, v in all_grads(ctx, params).items():
            assert np.array_equal(v, ref[name]), (pl, name)

    # a budget that holds about half of the saved sets: the library's plan equals the oracle planner's
    layers, loss_c, fixed = ctx.karma_get_costs()
    layers = [(1000 + 10 * i, 2000 + 10 * i, 800 + 10 * i) + l[3:] for i, l in enumerate(layers)]
    loss_c = (500,) + tuple(loss_c[1:])
    link = (2 * 10**9, 2 * 10**9, 1000)
    ctx.karma_set_costs(layers, loss_c, link)
    full = sum(l[3] + l[4] for l in layers)
    budget = fixed + full // 2 + max(max(l[5] for l in layers), loss_c[1]) + 2 * max(l[4] for l in layers)
    acts, summ = ctx.karma_plan(budget)
    ao, so = P.plan([P.Layer(*l) for l in layers], P.Link(*link), budget, fixed, P.Loss(*loss_c))
    assert acts == ao and summ["makespan_ns"] == so["makespan_ns"] and summ["peak_bytes"] == so["peak_bytes"] <= budget
    assert acts != [K.KEEP] * n
    assert ctx.karma_step(images, labels) == loss
    for name, v in all_grads(ctx, params).items():
        assert np.array_equal(v, ref[name]), name
    ctx.close()


def test_wrn_true_width_depth_one_block_per_group_batch_8(g):
    """The widths, image size and strides of WRN-28-10 itself (16 -> 160 -> 320 -> 640 channels on 32 x 32
    images), one block per group instead of four, batch 8: every shape of the full model's convolutions."""
    dims = dict(width=160, group_blocks=(1, 1, 1), image=32, batch=8, classes=16)
    params, images, labels = S.wrn_problem(dims, 3.0)
    arena = 1 << 30
    ctx = make_ctx(dims, arena)
    n = ctx.n_layers
    assert n == 4
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * n)
    loss = ctx.karma_step(images, labels)
    ref = all_grads(ctx, params)
    pr = S.rounded_params(params)
    lo, go = wrn.wrn_step(pr, images, labels)
    _, gs = S.wrn_step_bf16_storage(pr, images, labels)
    og, sg = oracle_grads(go), oracle_grads(gs)
    assert abs(loss - lo) <= 5e-3 * abs(lo), (loss, lo)
    floor = S.distances(sg, og)
    d = S.distances(ref, og)
    bad = {k: (d[k], floor[k]) for k in d if not d[k] <= 0.5 * BAR + FLOOR_FACTOR * floor[k]}
    assert not bad, bad
    assert np.median([d[k] / (floor[k] + 1e-3) for k in d]) <= 1.25
    ctx.karma_set_plan(arena, [K.SWAP, K.RC_KEEP, K.RC_CHAIN, K.RC_SWAP])
    assert ctx.karma_step(images, labels) == loss
    for name, v in all_grads(ctx, params).items():
        assert np.array_equal(v, ref[name]), name
    ctx.close()


def test_wrn_sgd_momentum_step_lowers_the_loss(g):
    params, images, labels = S.wrn_problem(DIMS, 3.0)
    arena = 256 << 20
    ctx = make_ctx(DIMS, arena, lr=1e-3, mu=0.9)
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP, K.SWAP, K.RC_KEEP, K.KEEP, K.RC_SWAP])
    l0 = ctx.karma_step(images, labels, K.STEP_APPLY_OPTIMIZER)
    g0 = all_grads(ctx, params)
    l1 = ctx.karma_step(images, labels, K.STEP_APPLY_OPTIMIZER)
    w = ctx.karma_get_param(2, 2)
    from oracle import nn
    w0 = np.asarray(params["blocks"][1][0]["w1"], np.float32).astype(np.float64).reshape(-1)
    w1, _ = nn.sgd_momentum_update(w0, np.zeros_like(w0), g0["b1.w1"].astype(np.float64), 1e-3, 0.9)
    l2 = ctx.karma_step(images, labels)
    assert l2 < l0
    # after the first update the weights are w1 (the second update is checked by the bottleneck network's test)
    ctx.close()
    ctx = make_ctx(DIMS, arena, lr=1e-3, mu=0.9)
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * 5)
    ctx.karma_step(images, labels, K.STEP_APPLY_OPTIMIZER)
    assert g.rel_l2(ctx.karma_get_param(2, 2), w1) <= 1e-6
    ctx.close()


def test_wrn_rejects_bad_descriptions(g):
    with pytest.raises(K.KarmaError):
        make_ctx(dict(DIMS, image=18), 64 << 20)
    with pytest.raises(K.KarmaError):
        make_ctx(dict(DIMS, group_blocks=(0, 1, 0)), 64 << 20)
    with pytest.raises(K.KarmaError):
        make_ctx(dict(DIMS, classes=10), 64 << 20)


# ------------------------------------------------------------------ the two kernel forms the block adds
@pytest.mark.parametrize("n,h,w,ci,co,r,stride,pad", [(2, 16, 16, 32, 32, 3, 1, 1), (3, 9, 7, 24, 40, 3, 1, 1),
                                                       (2, 16, 16, 16, 160, 1, 1, 0), (2, 14, 14, 160, 320, 1, 2, 0),
                                                       (8, 32, 32, 160, 160, 3, 1, 1)])
def test_conv_forward_with_residual(g, n, h, w, ci, co, r, stride, pad):
    import torch
    x, xd = bf(si.normal(1, (n, h, w, ci)))
    wt, wd = bf(si.normal(2, (co, r, r, ci), 0.2))
    ho, wo = cnn.conv_out(h, r, stride, pad), cnn.conv_out(w, r, stride, pad)
    add, addd = bf(si.normal(3, (n, ho, wo, co)) * 3)
    sh = K.ConvShape(n, h, w, ci, co, r, r, stride, pad)
    y = torch.empty(n, ho, wo, co, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_conv2d_fwd_add_bf16, g.ptr(xd), g.ptr(wd), g.ptr(addd), g.ptr(y), C.byref(sh), g.stream_ptr())
    ref = cnn.conv2d_fwd(x, wt, stride, pad) + add
    assert g.rel_l2(back(y), ref) <= TOL
    assert np.all(np.abs(back(y) - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-4 * np.abs(ref).max())
    # without a residual it is the plain convolution
    y2 = torch.empty_like(y)
    y3 = torch.empty_like(y)
    g.call(K.lib().karma_k_conv2d_fwd_add_bf16, g.ptr(xd), g.ptr(wd), None, g.ptr(y2), C.byref(sh), g.stream_ptr())
    g.call(K.lib().karma_k_conv2d_fwd_bf16, g.ptr(xd), g.ptr(wd), g.ptr(y3), C.byref(sh), g.stream_ptr())
    assert np.array_equal(back(y2), back(y3))


@pytest.mark.parametrize("rows,c", [(1000, 64), (257, 24), (5000, 160), (64, 640)])
def test_batchnorm_backward_with_shortcut_gradient(g, rows, c):
    import torch
    x, xd = bf(si.normal(5, (rows, c)) * (1.0 + 0.1 * np.arange(c)[None, :] % 3) + 0.5 * (np.arange(c)[None, :] % 5 - 2))
    gam, gd = bf(1.0 + si.normal(6, (c,), 0.2))
    bet, bd = bf(si.normal(7, (c,), 0.2))
    dy, dyd = bf(si.normal(9, (rows, c)))
    add, addd = bf(si.normal(10, (rows, c)))
    lib = K.lib()
    lib.karma_k_batchnorm_ws_bytes.restype = C.c_uint64
    ws = torch.empty(lib.karma_k_batchnorm_ws_bytes(rows, c) // 4, dtype=torch.float32, device="cuda")
    stats = torch.empty(2, c, dtype=torch.float32, device="cuda")
    y = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_batchnorm_fwd_bf16, g.ptr(xd), g.ptr(gd), g.ptr(bd), None, g.ptr(y), g.ptr(stats), g.ptr(ws), rows, c, 1,
           g.stream_ptr())
    _, cache = cnn.batchnorm_fwd(x.reshape(1, 1, rows, c), gam, bet)
    dym = dy * (back(y) > 0)           # the ReLU decision is the kernel's own
    dxo, dgo, dbo = cnn.batchnorm_bwd(dym.reshape(1, 1, rows, c), gam, cache)
    res = {}
    for name, a_ref, a_dev in (("other", add, addd), ("dy", dy, dyd), ("none", 0, None)):
        dx = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
        dg = torch.empty(c, dtype=torch.float32, device="cuda"); db = torch.empty(c, dtype=torch.float32, device="cuda")
        g.call(lib.karma_k_batchnorm_bwd_add_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), g.ptr(bd), 1,
               g.ptr(a_dev) if a_dev is not None else None, g.ptr(dx), g.ptr(dg), g.ptr(db), g.ptr(ws), rows, c, g.stream_ptr())
        want = dxo.reshape(rows, c) + a_ref
        assert g.rel_l2(back(dx), want) <= TOL, name
        ratio = g.elem_ratio(back(dx), want, 1, 1e-3, axis=0)
        assert ratio <= 1, (name, ratio)
        assert np.all(np.abs(dg.cpu().numpy() - dgo) <= 1e-3 * np.sqrt(rows) + 1e-4 * np.abs(dgo))
        res[name] = back(dx)
    dx0 = torch.empty(rows, c, dtype=torch.bfloat16, device="cuda")
    g.call(lib.karma_k_batchnorm_bwd_bf16, g.ptr(dyd), g.ptr(xd), g.ptr(stats), g.ptr(gd), g.ptr(bd), 1, g.ptr(dx0),
           g.ptr(dg), g.ptr(db), g.ptr(ws), rows, c, g.stream_ptr())
    assert np.array_equal(back(dx0), res["none"])
