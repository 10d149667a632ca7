"""Fully convolutional network (the U-Net row of Table III; Sec. III-F.3: connections from the
contracting to the expansive path) on the GPU.  A small network of the same structure goes
through the whole step against the oracle; out-of-core plans, among them plans that swap
out or recompute the contracting records whose outputs the expansive path reads again
(premature swap-in, held gradients), must be bit-identical to the in-core step; the
library's plan under a tight budget must equal the oracle planner's with the same
connections.  The kernels this model adds (2x2 pooling, the up-convolution as the input
gradient of a strided convolution, the in-place add, per-pixel softmax cross entropy) are
compared with the oracle element by element.  Tolerances of the whole step as for the
other convolutional networks: each gradient tensor within FLOOR_FACTOR times the distance
that bf16 storage alone puts between the plain fp64 oracle and the same step with bf16
tensors (`tests/test_cnn_bf16_floor.py`), plus half the bar."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import cnn, nn, unet, planner as P
import synth_inputs as si

import cnn_bf16_storage as S
from test_gpu_bf16_kernels import back, bf

BAR = 2e-2
FLOOR_FACTOR = 2.0
DIMS = S.UNET_SMALL
TOL = 2.0 ** -8
DOWN = si.LEVEL_TENSORS                                        # w1 g1 b1 w2 g2 b2
UP = ("wu", "w1s", "w1u", "g1", "b1", "w2", "g2", "b2")       # the library's tensors of an expansive record


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def make_ctx(dims, arena, lr=0.05, mu=0.9, classes=8):
    desc = dict(kind=K.MODEL_UNET, n_layers=dims["depth"], width=dims["width"], batch=dims["batch"], seq=dims["image"],
                n_heads=0, ffn=0, vocab=classes, stream_weights=0, stage_blocks=(0, 0, 0, 0))
    cfg = dict(optimizer=K.OPT_SGD_MOMENTUM, lr=lr, beta1=mu, beta2=0.0, eps=0.0, host_threads=8)
    return K.Context(desc, cfg, arena)


def pad_last(w, n):
    out = np.zeros(w.shape[:-1] + (n,), dtype=np.float64)
    out[..., :w.shape[-1]] = w
    return out


def up_tensors(p):
    c = p["w1"].shape[3] // 2
    d = dict(p)
    d["w1s"], d["w1u"] = p["w1"][..., :c], p["w1"][..., c:]
    return d


def load_params(ctx, params, classes=8):
    depth = len(params["up"])
    for l, p in enumerate(params["down"]):
        for t, name in enumerate(DOWN):
            ctx.karma_set_param(l, t, pad_last(p[name], 8) if (l == 0 and name == "w1") else p[name])
    for j, p in enumerate(params["up"]):
        d = up_tensors(p)
        for t, name in enumerate(UP):
            ctx.karma_set_param(depth + 1 + j, t, d[name])
    hd = params["head"]
    k = hd["w"].shape[0]
    w = np.zeros((classes, hd["w"].shape[1]))
    w[:k] = hd["w"]
    bias = np.full(classes, -30000.0)
    bias[:k] = hd["bias"]
    ctx.karma_set_param(2 * depth + 1, 0, w)
    ctx.karma_set_param(2 * depth + 1, 1, bias)


def all_grads(ctx, params):
    depth = len(params["up"])
    out = {}
    for l in range(depth + 1):
        for t, name in enumerate(DOWN):
            out["d%d.%s" % (l, name)] = ctx.karma_get_grad(l, t)
    for j in range(depth):
        for t, name in enumerate(UP):
            out["u%d.%s" % (j, name)] = ctx.karma_get_grad(depth + 1 + j, t)
    out["head.w"] = ctx.karma_get_grad(2 * depth + 1, 0)
    out["head.bias"] = ctx.karma_get_grad(2 * depth + 1, 1)
    return out


def as_library(flat, params, classes=8):
    """Oracle gradients in the library's tensor layout (split first weight, padded image channel and classes)."""
    out = {}
    for k, v in flat.items():
        if k.startswith("u") and k.endswith(".w1"):
            c = v.shape[3] // 2
            out[k + "s"], out[k + "u"] = v[..., :c], v[..., c:]
        elif k == "d0.w1":
            out[k] = pad_last(v, 8)
        elif k == "head.w":
            w = np.zeros((classes, v.shape[1]))
            w[:v.shape[0]] = v
            out[k] = w
        elif k == "head.bias":
            b = np.zeros(classes)
            b[:v.shape[0]] = v
            out[k] = b
        else:
            out[k] = v
    return out


def distances(got, want):
    """As `cnn_bf16_storage.distances`; the split halves of a first weight are measured against the whole weight."""
    d = {}
    for k in want:
        scale = S.scale_of(k, want) if not (k.endswith("w1s") or k.endswith("w1u")) else np.sqrt(
            np.linalg.norm(want[k[:-1] + "s"]) ** 2 + np.linalg.norm(want[k[:-1] + "u"]) ** 2)
        d[k] = float(np.linalg.norm(np.asarray(got[k], np.float64).reshape(-1) - np.asarray(want[k]).reshape(-1)) / scale)
    return d


def check_against_oracle(g, ctx, params, images, labels, loss):
    ref = all_grads(ctx, params)
    pr = S.unet_rounded_params(params)
    lo, go = unet.unet_step(pr, images, labels)
    _, gs = S.unet_step_bf16_storage(pr, images, labels)
    og, sg = as_library(S.unet_flat(go), params), as_library(S.unet_flat(gs), params)
    assert abs(loss - lo) <= 5e-3 * abs(lo), (loss, lo)
    floor = distances(sg, og)
    d = distances(ref, og)
    bad = {k: (d[k], floor[k]) for k in d if not d[k] <= 0.5 * BAR + FLOOR_FACTOR * floor[k]}
    assert not bad, bad
    assert np.median([d[k] / (floor[k] + 1e-3) for k in d]) <= 1.25
    return ref


@pytest.mark.parametrize("shift", [3.0, 0.0])
def test_unet_step_matches_oracle_and_plans_are_bit_identical(g, shift):
    params, images, labels = S.unet_problem(DIMS, shift)
    arena = 256 << 20
    ctx = make_ctx(DIMS, arena)
    n = ctx.n_layers
    assert n == 5 and K.karma_model_skips(ctx.desc) == [(0, 4), (1, 3)]
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * n)
    loss = ctx.karma_step(images[..., 0], labels)
    ref = check_against_oracle(g, ctx, params, images, labels, loss)
    assert np.all(ref["d0.w1"].reshape(-1, 8)[:, 1:] == 0)      # the padding channels see no gradient
    assert np.all(ref["head.w"][2 * DIMS["width"]:] == 0)       # nor do the padding classes

    # records 1 and 2 are the ones whose input the expansive path reads again: swapped out, they come back early
    plans = [[K.SWAP] * n, [K.RC_KEEP] * n, [K.RC_SWAP] * n, [K.KEEP, K.SWAP, K.KEEP, K.KEEP, K.KEEP],
             [K.KEEP, K.KEEP, K.RC_SWAP, K.KEEP, K.KEEP], [K.SWAP, K.RC_SWAP, K.SWAP, K.RC_KEEP, K.RC_CHAIN],
             [K.RC_KEEP, K.RC_KEEP, K.SWAP, K.SWAP, K.RC_SWAP], [K.KEEP, K.SWAP, K.RC_KEEP, K.RC_SWAP, K.RC_CHAIN]]
    for pl in plans:
        ctx.karma_set_plan(arena, pl)
        assert ctx.karma_step(images[..., 0], labels) == loss, pl
        for name, v in all_grads(ctx, params).items():
            assert np.array_equal(v, ref[name]), (pl, name)
    # a chained record cannot be one whose input is read again
    with pytest.raises(K.KarmaError):
        ctx.karma_set_plan(arena, [K.RC_KEEP, K.RC_CHAIN, K.KEEP, K.KEEP, K.KEEP])

    ctx.close()


def test_unet_planned_under_tight_budgets_equals_oracle_planner_and_in_core_step(g):
    """Budgets below what the in-core step needs, on a batch large enough for the saved tensors to outweigh the
    workspaces: the library's plan equals the oracle planner's given the same connections, swaps out records
    whose input the expansive path reads again, and the step stays bit-identical."""
    dims = dict(DIMS, image=128, batch=4)
    params, images, labels = S.unet_problem(dims, 3.0)
    arena = 256 << 20
    ctx = make_ctx(dims, arena)
    n = ctx.n_layers
    load_params(ctx, params)
    layers, loss_c, fixed = ctx.karma_get_costs()
    layers = [(100000 + 10 * i, 200000 + 10 * i, 80000 + 10 * i) + l[3:] for i, l in enumerate(layers)]
    loss_c = (50000,) + tuple(loss_c[1:])
    link = (50 * 10**9, 50 * 10**9, 1000)
    ctx.karma_set_costs(layers, loss_c, link)
    peak = ctx.karma_set_plan(arena, [K.KEEP] * n)["peak_bytes"]
    loss = ctx.karma_step(images[..., 0], labels)
    ref = all_grads(ctx, params)
    assert abs(loss - np.log(2)) < 0.5
    skips = K.karma_model_skips(ctx.desc)
    seen = set()
    for share in (0.9, 0.8, 0.75, 0.7, 0.65):
        budget = fixed + int((peak - fixed) * share)
        ao, so = P.plan([P.Layer(*l) for l in layers], P.Link(*link), budget, fixed, P.Loss(*loss_c), skips=skips)
        acts, summ = ctx.karma_plan(budget)
        assert acts == ao and summ["makespan_ns"] == so["makespan_ns"] and summ["peak_bytes"] == so["peak_bytes"] <= budget
        seen.add(tuple(acts))
        assert ctx.karma_step(images[..., 0], labels) == loss
        for name, v in all_grads(ctx, params).items():
            assert np.array_equal(v, ref[name]), (share, name)
    assert len(seen) >= 4 and any(a[1] == K.SWAP for a in seen) and any(a[1] == K.RC_KEEP for a in seen)
    with pytest.raises(K.KarmaError):
        ctx.karma_plan(fixed + int((peak - fixed) * 0.3))
    ctx.close()


def test_unet_true_widths_depth_4_image_64_batch_1(g):
    """The channel counts of the model itself (64 .. 1024, up-convolutions 1024 -> 512 .. 128 -> 64) on 64 x 64
    images, one image: every convolution shape of the full model except for the number of pixels."""
    dims = dict(width=64, depth=4, image=64, batch=1, classes=2)
    params, images, labels = S.unet_problem(dims, 3.0)
    arena = 2 << 30
    ctx = make_ctx(dims, arena)
    n = ctx.n_layers
    assert n == 9
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * n)
    loss = ctx.karma_step(images[..., 0], labels)
    ref = check_against_oracle(g, ctx, params, images, labels, loss)
    ctx.karma_set_plan(arena, [K.SWAP, K.RC_SWAP, K.SWAP, K.RC_KEEP, K.SWAP, K.RC_KEEP, K.RC_CHAIN, K.SWAP, K.RC_SWAP])
    assert ctx.karma_step(images[..., 0], labels) == loss
    for name, v in all_grads(ctx, params).items():
        assert np.array_equal(v, ref[name]), name
    ctx.close()


def test_unet_sgd_momentum_steps_lower_the_loss(g):
    params, images, labels = S.unet_problem(DIMS, 3.0)
    arena = 256 << 20
    ctx = make_ctx(DIMS, arena, lr=2e-2, mu=0.9)
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP, K.SWAP, K.RC_SWAP, K.KEEP, K.RC_KEEP])
    l0 = ctx.karma_step(images[..., 0], labels, K.STEP_APPLY_OPTIMIZER)
    g0 = all_grads(ctx, params)
    w_lib = ctx.karma_get_param(3, 0)
    w0 = np.asarray(params["up"][0]["wu"], np.float32).astype(np.float64).reshape(-1)
    w1, _ = nn.sgd_momentum_update(w0, np.zeros_like(w0), g0["u0.wu"].astype(np.float64), 2e-2, 0.9)
    assert g.rel_l2(w_lib, w1) <= 1e-6
    for _ in range(3):
        ctx.karma_step(images[..., 0], labels, K.STEP_APPLY_OPTIMIZER)
    assert ctx.karma_step(images[..., 0], labels) < l0
    ctx.close()


def test_unet_rejects_bad_descriptions(g):
    with pytest.raises(K.KarmaError):
        make_ctx(dict(DIMS, image=30), 64 << 20)          # not a multiple of 2^depth
    with pytest.raises(K.KarmaError):
        make_ctx(dict(DIMS, depth=0), 64 << 20)
    with pytest.raises(K.KarmaError):
        make_ctx(DIMS, 64 << 20, classes=2)               # classes are stored in multiples of 8
    ctx = make_ctx(DIMS, 64 << 20)
    ctx.karma_set_plan(64 << 20, [K.KEEP] * 5)
    with pytest.raises(K.KarmaError):                     # a label outside the classes
        ctx.karma_step(np.zeros((2, 32, 32), np.float32), np.full((2, 32, 32), 8, np.int32))
    ctx.close()


# ------------------------------------------------------------------ the kernels this model adds
@pytest.mark.parametrize("n,h,w,c", [(2, 8, 8, 8), (3, 6, 10, 24), (1, 64, 64, 64), (2, 32, 32, 128)])
def test_maxpool_2x2(g, n, h, w, c):
    import torch
    x, xd = bf(np.maximum(si.normal(11, (n, h, w, c)), 0))     # after a ReLU: many ties at zero
    dy, dyd = bf(si.normal(12, (n, h // 2, w // 2, c)))
    y = torch.empty(n, h // 2, w // 2, c, dtype=torch.bfloat16, device="cuda")
    dx = torch.full((n, h, w, c), 7.0, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_maxpool2_fwd_bf16, g.ptr(xd), g.ptr(y), n, h, w, c, g.stream_ptr())
    g.call(K.lib().karma_k_maxpool2_bwd_bf16, g.ptr(xd), g.ptr(dyd), g.ptr(dx), n, h, w, c, g.stream_ptr())
    yo, arg = cnn.maxpool_fwd(x, 2, 2, 0)
    assert np.array_equal(back(y), yo)
    assert np.array_equal(back(dx), cnn.maxpool_bwd(dy, arg, x.shape, 2, 2, 0))
    assert K.lib().karma_k_maxpool2_fwd_bf16(g.ptr(xd), g.ptr(y), n, h + 1, w, c, g.stream_ptr()) != 0


@pytest.mark.parametrize("n,h,w,ci,co", [(2, 4, 4, 16, 8), (1, 6, 10, 24, 40), (2, 8, 8, 256, 128), (4, 16, 16, 128, 64),
                                         (2, 32, 32, 1024, 512)])
def test_upconvolution_through_the_strided_convolution_kernels(g, n, h, w, ci, co):
    """Forward = input gradient of the 2x2 stride-2 convolution that maps the fine grid back; its gradients are
    that convolution's forward pass and weight gradient."""
    import torch
    x, xd = bf(si.normal(21, (n, h, w, ci)))
    wt, wd = bf(si.normal(22, (ci, 2, 2, co), 0.1))
    dy, dyd = bf(si.normal(23, (n, 2 * h, 2 * w, co)))
    sh = K.ConvShape(n, 2 * h, 2 * w, co, ci, 2, 2, 2, 0)
    y = torch.empty(n, 2 * h, 2 * w, co, dtype=torch.bfloat16, device="cuda")
    wt_ws = torch.empty(4 * ci * co, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_conv2d_dgrad_bf16, g.ptr(xd), g.ptr(wd), g.ptr(wt_ws), None, g.ptr(y), C.byref(sh), g.stream_ptr())
    ref = unet.upconv2x2_fwd(x, wt)
    assert g.rel_l2(back(y), ref) <= TOL
    assert np.all(np.abs(back(y) - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-4 * np.abs(ref).max())
    dxo, dwo = unet.upconv2x2_bwd(x, wt, dy)
    dx = torch.empty(n, h, w, ci, dtype=torch.bfloat16, device="cuda")
    g.call(K.lib().karma_k_conv2d_fwd_bf16, g.ptr(dyd), g.ptr(wd), g.ptr(dx), C.byref(sh), g.stream_ptr())
    assert g.rel_l2(back(dx), dxo) <= TOL
    dw = torch.empty(ci, 2, 2, co, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(16 * 4 * ci * co, dtype=torch.float32, device="cuda")
    g.call(K.lib().karma_k_conv2d_wgrad_bf16, g.ptr(xd), g.ptr(dyd), g.ptr(dw), g.ptr(ws), ws.numel() * 4, C.byref(sh),
           g.stream_ptr())
    assert g.rel_l2(back(dw), dwo) <= TOL
    assert g.elem_ratio(back(dw).reshape(ci, -1), dwo.reshape(ci, -1), 1, 2e-3) <= 1


@pytest.mark.parametrize("n", [8, 4096, 100000 * 8 + 8])
def test_add_in_place(g, n):
    a, ad = bf(si.normal(31, (n,)))
    b, bd = bf(si.normal(32, (n,)))
    g.call(K.lib().karma_k_add_inplace_bf16, g.ptr(ad), g.ptr(bd), n, g.stream_ptr())
    assert np.array_equal(back(ad), nn.bf16_round((a + b).astype(np.float32)).astype(np.float64))
    assert K.lib().karma_k_add_inplace_bf16(g.ptr(ad), g.ptr(bd), 12, g.stream_ptr()) != 0


@pytest.mark.parametrize("rows,cols", [(4096, 8), (70001, 8), (5000, 16), (100, 8)])
def test_softmax_cross_entropy_over_short_rows(g, rows, cols):
    """Millions of pixels with a handful of classes take a kernel with one thread per row (from 4096 rows on)."""
    import torch
    z, zd = bf(si.normal(41, (rows, cols)) * 3)
    z[:, cols - 3:] = -30000.0                            # padding classes
    zd = g.dev(z).to(torch.bfloat16)
    z = back(zd)
    lab = si.randint(42, (rows,), cols - 3).astype(np.int32)
    labd = g.dev(lab)
    rowloss = torch.empty(rows, dtype=torch.float32, device="cuda")
    scale = 1.0 / rows
    g.call(K.lib().karma_k_softmax_ce_bf16, g.ptr(zd), g.ptr(labd), g.ptr(rowloss), rows, cols, C.c_float(scale), g.stream_ptr())
    m = z.max(axis=1, keepdims=True)
    lse = (m + np.log(np.exp(z - m).sum(axis=1, keepdims=True)))[:, 0]
    want_loss = lse - z[np.arange(rows), lab]
    p = np.exp(z - lse[:, None])
    p[np.arange(rows), lab] -= 1
    assert np.all(np.abs(rowloss.cpu().numpy() - want_loss) <= 1e-5 * (1 + np.abs(want_loss)))
    got = back(zd)
    assert np.all(np.abs(got - p * scale) <= (2.0 ** -8 * np.abs(p) + 1e-6) * scale)
    assert np.all(got[:, cols - 3:] == 0)
