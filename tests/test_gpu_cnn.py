"""Bottleneck CNN workload on the GPU: a small residual network through the whole step
against the oracle (bf16 tolerance of the workload: relative L2 <= 2e-2), out-of-core
plans bit-identical to the in-core step, host SGD with momentum against the oracle's
update, streamed weights."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import cnn, nn, planner as P
import synth_inputs as si

import cnn_bf16_storage as S

BAR = 2e-2
# No step that keeps its tensors in bf16 comes within the workload's 2e-2 of the plain
# oracle on this kind of network: `tests/test_cnn_bf16_floor.py` measures, on the CPU, how
# far bf16 storage alone moves each gradient (3e-2 in the median, 15e-2 at worst, with
# stable ReLU masks; 15e-2 to 60e-2 when they flip).  So a gradient tensor passes when its
# distance from the PLAIN oracle is at most FLOOR_FACTOR times that tensor's own floor plus
# half the bar, the floor being recomputed here from the plain oracle and the storage
# variant.  The factor allows for the roundings a real kernel adds to the variant's: fp32
# instead of fp64 accumulation and statistics, bf16 weight gradients, bf16 sums on the
# shortcut (measured: at most 1.5 times the floor, 0.92 to 0.99 in the median).
FLOOR_FACTOR = 2.0
SMALL, SHALLOW = S.SMALL, S.SHALLOW
BT = cnn.BOTTLENECK_TENSORS


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def make_ctx(dims, arena, stream=0, lr=0.05, mu=0.9):
    desc = dict(kind=K.MODEL_CNN, n_layers=0, width=dims["width"], batch=dims["batch"], seq=dims["image"], n_heads=0, ffn=0,
                vocab=dims["classes"], stream_weights=stream, stage_blocks=dims["stage_blocks"])
    cfg = dict(optimizer=K.OPT_SGD_MOMENTUM, lr=lr, beta1=mu, beta2=0.0, eps=0.0, host_threads=8)
    return K.Context(desc, cfg, arena)


def pad_stem(w):
    out = np.zeros(w.shape[:3] + (8,), dtype=np.float64)
    out[..., :3] = w
    return out


def load_params(ctx, params):
    st = params["stem"]
    ctx.karma_set_param(0, 0, pad_stem(st["w"]))
    ctx.karma_set_param(0, 1, st["g"])
    ctx.karma_set_param(0, 2, st["b"])
    for i, (p, _) in enumerate(params["blocks"]):
        for t, name in enumerate(BT):
            if name in p:
                ctx.karma_set_param(i + 1, t, p[name])
    L = len(params["blocks"]) + 1
    ctx.karma_set_param(L, 0, params["head"]["w"])
    ctx.karma_set_param(L, 1, params["head"]["b"])


def all_grads(ctx, params):
    out = {"stem.w": ctx.karma_get_grad(0, 0), "stem.g": ctx.karma_get_grad(0, 1), "stem.b": ctx.karma_get_grad(0, 2)}
    for i, (p, _) in enumerate(params["blocks"]):
        for t, name in enumerate(BT):
            if name in p:
                out["b%d.%s" % (i, name)] = ctx.karma_get_grad(i + 1, t)
    L = len(params["blocks"]) + 1
    out["head.w"] = ctx.karma_get_grad(L, 0)
    out["head.b"] = ctx.karma_get_grad(L, 1)
    return out


def oracle_grads(grads):
    out = {"stem.w": pad_stem(grads["stem"]["w"]), "stem.g": grads["stem"]["g"], "stem.b": grads["stem"]["b"],
           "head.w": grads["head"]["w"], "head.b": grads["head"]["b"]}
    for i, gb in enumerate(grads["blocks"]):
        for name, v in gb.items():
            out["b%d.%s" % (i, name)] = v
    return out


def small_problem(shift=3.0, dims=None):
    """Batch-norm shifts are raised by `shift` (ReLU masks far from a flip: the comparison
    then measures arithmetic rather than flipped decisions; the masks themselves are checked
    exactly, decision by decision, in the kernel tests)."""
    return S.problem(dims or SMALL, shift)


def oracle_step(params, images, labels):
    """Loss and gradients of the plain fp64 oracle, and the gradients of the same step with
    bf16 storage (the floor under any bf16 implementation)."""
    pr = S.rounded_params(params)
    lo, go = cnn.resnet_step(pr, images, labels)
    _, gs = S.resnet_step_bf16_storage(pr, images, labels)
    return lo, oracle_grads(go), oracle_grads(gs)


def check_grads(got, plain, storage):
    floor = S.distances(storage, plain)
    d = S.distances(got, plain)
    bad = {k: (d[k], floor[k]) for k in d if not d[k] <= 0.5 * BAR + FLOOR_FACTOR * floor[k]}
    assert not bad, bad
    # taken together the device's gradients are about as far from the plain oracle as the
    # storage variant's are
    assert np.median([d[k] / (floor[k] + 1e-3) for k in d]) <= 1.25


@pytest.mark.parametrize("shift", [3.0, 0.0])
def test_cnn_shallow_step_matches_oracle(g, shift):
    params, images, labels = small_problem(shift=shift, dims=SHALLOW)
    arena = 256 << 20
    ctx = make_ctx(SHALLOW, arena)
    assert ctx.n_layers == 3
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * 3)
    loss = ctx.karma_step(images, labels)
    lo, og, sg = oracle_step(params, images, labels)
    assert abs(loss - lo) <= 5e-3 * abs(lo), (loss, lo)
    check_grads(all_grads(ctx, params), og, sg)
    ctx.karma_set_plan(arena, [K.SWAP, K.RC_KEEP, K.RC_CHAIN])
    assert ctx.karma_step(images, labels) == loss
    ctx.close()


@pytest.mark.parametrize("shift", [3.0, 0.0])
def test_cnn_step_matches_oracle_and_plans_are_bit_identical(g, shift):
    params, images, labels = small_problem(shift=shift)
    arena = 256 << 20
    ctx = make_ctx(SMALL, arena)
    n = ctx.n_layers
    assert n == 6
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * n)
    loss = ctx.karma_step(images, labels)
    ref = all_grads(ctx, params)
    lo, og, sg = oracle_step(params, images, labels)
    assert abs(loss - lo) <= 5e-3 * abs(lo), (loss, lo)
    check_grads(ref, og, sg)
    assert np.all(ref["stem.w"].reshape(8, 7, 7, 8)[..., 3:] == 0)      # the padding channels see no gradient

    plans = [[K.SWAP] * n, [K.RC_KEEP] * n, [K.KEEP, K.RC_SWAP, K.RC_CHAIN, K.SWAP, K.RC_KEEP, K.RC_CHAIN],
             [K.RC_KEEP] + [K.RC_CHAIN] * (n - 1), [K.SWAP, K.KEEP, K.RC_KEEP, K.SWAP, K.KEEP, K.RC_SWAP]]
    for pl in plans:
        ctx.karma_set_plan(arena, pl)
        assert ctx.karma_step(images, labels) == loss, pl
        for name, v in all_grads(ctx, params).items():
            assert np.array_equal(v, ref[name]), (pl, name)

    # a budget that holds about half of the saved sets: plan equals the oracle's plan
    layers, loss_c, fixed = ctx.karma_get_costs()
    layers = [(1000 + 10 * i, 2000 + 10 * i, 1000 + 10 * i) + l[3:] for i, l in enumerate(layers)]
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


def test_cnn_sgd_momentum_and_streamed_weights(g):
    params, images, labels = small_problem()
    arena = 256 << 20
    res = []
    for stream in (0, 1):
        ctx = make_ctx(SMALL, arena, stream=stream, lr=1e-3, mu=0.9)
        load_params(ctx, params)
        n = ctx.n_layers
        ctx.karma_set_plan(arena, [K.KEEP, K.SWAP, K.RC_KEEP, K.KEEP, K.RC_SWAP, K.KEEP], [0, 1, 0, 0, 1, 0] if stream else None)
        l0 = ctx.karma_step(images, labels, K.STEP_APPLY_OPTIMIZER)
        g0 = all_grads(ctx, params)
        l1 = ctx.karma_step(images, labels, K.STEP_APPLY_OPTIMIZER)
        g1 = all_grads(ctx, params)
        l2 = ctx.karma_step(images, labels)
        w = {"b1.w2": ctx.karma_get_param(2, 3), "stem.g": ctx.karma_get_param(0, 1), "head.w": ctx.karma_get_param(n, 0),
             "b3.wp": ctx.karma_get_param(4, 9)}
        res.append((l0, l1, l2, w))
        if stream == 0:
            # two steps of SGD with momentum 0.9 from the device gradients of those steps
            for key, before in (("b1.w2", params["blocks"][1][0]["w2"]), ("stem.g", params["stem"]["g"]),
                                ("head.w", params["head"]["w"]), ("b3.wp", params["blocks"][3][0]["wp"])):
                w0 = np.asarray(before, np.float32).astype(np.float64).reshape(-1)
                w1, buf = nn.sgd_momentum_update(w0, np.zeros_like(w0), g0[key].astype(np.float64), 1e-3, 0.9)
                w2, buf = nn.sgd_momentum_update(w1, buf, g1[key].astype(np.float64), 1e-3, 0.9)
                assert g.rel_l2(w[key], w2) <= 1e-6, key
            assert l2 < l0
        ctx.close()
    assert res[0][:3] == res[1][:3]
    for key in res[0][3]:
        assert np.array_equal(res[0][3][key], res[1][3][key]), key


def test_step_on_the_resident_batch_equals_the_step_with_inputs(g):
    params, images, labels = small_problem()
    arena = 256 << 20
    ctx = make_ctx(SMALL, arena)
    load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP, K.SWAP, K.RC_KEEP, K.KEEP, K.RC_SWAP, K.KEEP])
    with pytest.raises(K.KarmaError) as e:
        ctx.karma_step(None, None)              # nothing resident yet
    assert e.value.status == K.E_STATE
    loss = ctx.karma_step(images, labels)
    ref = all_grads(ctx, params)
    assert ctx.karma_step(None, None) == loss
    for name, v in all_grads(ctx, params).items():
        assert np.array_equal(v, ref[name]), name
    other = images[::-1].copy()
    l2 = ctx.karma_step(other, labels)
    assert l2 != loss and ctx.karma_step(None, None) == l2
    ctx.karma_measure(1)                        # profiling steps replace the batch
    ctx.karma_set_plan(arena, [K.KEEP] * 6)
    with pytest.raises(K.KarmaError) as e:
        ctx.karma_step(None, None)
    assert e.value.status == K.E_STATE
    ctx.close()


def test_cnn_rejects_bad_descriptions(g):
    with pytest.raises(K.KarmaError):
        make_ctx(dict(SMALL, image=60), 64 << 20)             # image size not a multiple of 32
    with pytest.raises(K.KarmaError):
        make_ctx(dict(SMALL, stage_blocks=(0, 1, 0, 0)), 64 << 20)
    ctx = make_ctx(SMALL, 256 << 20)
    ctx.karma_set_plan(256 << 20, [0] * 6)
    images = np.zeros((4, 64, 64, 3), np.float32)
    with pytest.raises(K.KarmaError) as e:
        ctx.karma_step(images, np.array([0, 1, 16, 2], np.int32))
    assert e.value.status == K.E_INVAL
    ctx.close()
