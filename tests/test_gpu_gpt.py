"""GPT workload on the GPU: a small pre-LN transformer through the whole step against the
oracle (bf16 tolerance of the workload: relative L2 <= 2e-2), out-of-core plans
bit-identical to the in-core step, host Adam against the oracle's update."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import nn, planner as P
import synth_inputs as si

TOL = 2e-2
BLOCK_T = nn.BLOCK_TENSORS


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


def make_ctx(n_layers, hidden, heads, ffn, vocab, seq, batch, arena, lr=1e-3, threads=8, device_update_first=0):
    desc = dict(kind=K.MODEL_GPT, n_layers=n_layers, width=hidden, batch=batch, seq=seq, n_heads=heads, ffn=ffn, vocab=vocab)
    cfg = dict(optimizer=K.OPT_ADAM, lr=lr, beta1=0.9, beta2=0.999, eps=1e-8, host_threads=threads,
               device_update_first=device_update_first)
    return K.Context(desc, cfg, arena)


def load_params(ctx, params):
    ctx.karma_set_param(0, 0, params["wte"])
    ctx.karma_set_param(0, 1, params["wpe"])
    for i, b in enumerate(params["blocks"]):
        for t, name in enumerate(BLOCK_T):
            ctx.karma_set_param(i + 1, t, b[name])
    L = len(params["blocks"]) + 1
    ctx.karma_set_param(L, 0, params["lnf_g"])
    ctx.karma_set_param(L, 1, params["lnf_b"])


def rounded(params):
    r = lambda a: nn.bf16_round(np.asarray(a, np.float32)).astype(np.float64)
    return dict(wte=r(params["wte"]), wpe=r(params["wpe"]), lnf_g=r(params["lnf_g"]), lnf_b=r(params["lnf_b"]),
                blocks=[{k: r(v) for k, v in b.items()} for b in params["blocks"]])


def all_grads(ctx, n_blocks):
    out = {"wte": ctx.karma_get_grad(0, 0), "wpe": ctx.karma_get_grad(0, 1)}
    for i in range(n_blocks):
        for t, name in enumerate(BLOCK_T):
            out["b%d.%s" % (i, name)] = ctx.karma_get_grad(i + 1, t)
    out["lnf_g"] = ctx.karma_get_grad(n_blocks + 1, 0)
    out["lnf_b"] = ctx.karma_get_grad(n_blocks + 1, 1)
    return out


def oracle_grads(grads):
    out = {"wte": grads["wte"], "wpe": grads["wpe"], "lnf_g": grads["lnf_g"], "lnf_b": grads["lnf_b"]}
    for i, b in enumerate(grads["blocks"]):
        for name in BLOCK_T:
            out["b%d.%s" % (i, name)] = b[name]
    return out


SMALL = dict(n_layers=3, hidden=128, heads=2, ffn=264, vocab=520, seq=128, batch=2)


def small_problem():
    p, ids, labels = si.gpt_problem(seed=2008114202, n_layers=SMALL["n_layers"], hidden=SMALL["hidden"], ffn=SMALL["ffn"],
                                    vocab=SMALL["vocab"], seq=SMALL["seq"], batch=SMALL["batch"], std=0.05, bias_std=0.05)
    ids[0, 3] = ids[0, 9] = ids[1, 100]     # repeated tokens exercise the ordered scatter-add
    return p, ids.astype(np.int32), labels.astype(np.int32)


def unit_costs(ctx):
    layers, loss, fixed = ctx.karma_get_costs()
    layers = [(1000 + 10 * i, 2000 + 10 * i, 1000 + 10 * i) + l[3:] for i, l in enumerate(layers)]
    return layers, (3000,) + tuple(loss[1:]), fixed


def test_gpt_step_matches_oracle_and_plans_are_bit_identical(g):
    params, ids, labels = small_problem()
    ctx = make_ctx(arena=512 << 20, **SMALL)
    load_params(ctx, params)
    layers, loss_c, fixed = unit_costs(ctx)
    link = (2 * 10**9, 2 * 10**9, 1000)
    ctx.karma_set_costs(layers, loss_c, link)
    big = 512 << 20
    acts, summ = ctx.karma_plan(big)
    assert acts == [K.KEEP] * 4
    loss = ctx.karma_step(ids, labels)
    ref = all_grads(ctx, 3)
    lo, go, _, _ = nn.gpt_step(rounded(params), ids, labels, SMALL["heads"])
    assert abs(loss - lo) <= 2e-3 * abs(lo), (loss, lo)
    og = oracle_grads(go)
    for name, v in ref.items():
        assert g.rel_l2(v, og[name]) <= TOL, (name, g.rel_l2(v, og[name]))
    # the same batch again, from where it already lies in HBM
    assert ctx.karma_step(None, None) == loss
    for name, v in all_grads(ctx, 3).items():
        assert np.array_equal(v, ref[name]), name

    plans = [[K.KEEP, K.SWAP, K.SWAP, K.SWAP], [K.KEEP, K.RC_KEEP, K.RC_KEEP, K.RC_KEEP], [K.SWAP, K.RC_SWAP, K.RC_CHAIN, K.KEEP],
             [K.RC_KEEP, K.RC_CHAIN, K.RC_CHAIN, K.RC_CHAIN], [K.KEEP, K.RC_SWAP, K.SWAP, K.RC_KEEP]]
    for pl in plans:
        ctx.karma_set_plan(big, pl)
        assert ctx.karma_step(ids, labels) == loss, pl
        for name, v in all_grads(ctx, 3).items():
            assert np.array_equal(v, ref[name]), (pl, name)

    # a budget that holds about half of the blocks' saved sets: plan equals the oracle's plan
    per_block = layers[1][3] + layers[1][4]
    budget = fixed + int(1.6 * per_block) + max(layers[1][5], loss_c[1]) + 2 * layers[1][4]
    acts, summ = ctx.karma_plan(budget)
    ao, so = P.plan([P.Layer(*l) for l in layers], P.Link(*link), budget, fixed, P.Loss(*loss_c))
    assert acts == ao and summ["makespan_ns"] == so["makespan_ns"] and summ["peak_bytes"] == so["peak_bytes"]
    assert acts != [K.KEEP] * 4 and summ["peak_bytes"] <= budget
    assert ctx.karma_step(ids, labels) == loss
    for name, v in all_grads(ctx, 3).items():
        assert np.array_equal(v, ref[name]), name
    ctx.close()


def test_gpt_head_dimension_152_and_ragged_widths(g):
    """Two blocks with heads of 152 (the 17B-parameter configuration's head size) and widths that are no
    multiple of the GEMM tiles: the step against the oracle, swap and recompute plans bit-identical."""
    dims = dict(n_layers=2, hidden=304, heads=2, ffn=600, vocab=520, seq=128, batch=2)
    params, ids, labels = si.gpt_problem(seed=2008114205, n_layers=2, hidden=304, ffn=600, vocab=520, seq=128, batch=2,
                                         std=0.05, bias_std=0.05)
    ids, labels = ids.astype(np.int32), labels.astype(np.int32)
    ctx = make_ctx(arena=512 << 20, **dims)
    load_params(ctx, params)
    big = 512 << 20
    ctx.karma_set_plan(big, [K.KEEP] * 3)
    loss = ctx.karma_step(ids, labels)
    ref = all_grads(ctx, 2)
    lo, go, _, _ = nn.gpt_step(rounded(params), ids, labels, dims["heads"])
    assert abs(loss - lo) <= 2e-3 * abs(lo), (loss, lo)
    og = oracle_grads(go)
    for name, v in ref.items():
        assert g.rel_l2(v, og[name]) <= TOL, (name, g.rel_l2(v, og[name]))
    for pl in ([K.SWAP, K.RC_SWAP, K.RC_CHAIN], [K.KEEP, K.SWAP, K.RC_KEEP]):
        ctx.karma_set_plan(big, pl)
        assert ctx.karma_step(ids, labels) == loss, pl
        for name, v in all_grads(ctx, 2).items():
            assert np.array_equal(v, ref[name]), (pl, name)
    ctx.close()


def split_ctx(arena, dims, lr=1e-3):
    desc = dict(kind=K.MODEL_GPT, n_layers=dims["n_layers"], width=dims["hidden"], batch=dims["batch"], seq=dims["seq"],
                n_heads=dims["heads"], ffn=dims["ffn"], vocab=dims["vocab"], split_blocks=1)
    cfg = dict(optimizer=K.OPT_ADAM, lr=lr, beta1=0.9, beta2=0.999, eps=1e-8, host_threads=8)
    return K.Context(desc, cfg, arena)


def split_slot(block, t):
    """(record, tensor) of block tensor t when every block is two records."""
    return (2 * block + 1, t) if t < 6 else (2 * block + 2, t - 6)


def load_params_split(ctx, params):
    ctx.karma_set_param(0, 0, params["wte"])
    ctx.karma_set_param(0, 1, params["wpe"])
    for i, b in enumerate(params["blocks"]):
        for t, name in enumerate(BLOCK_T):
            ctx.karma_set_param(*split_slot(i, t), b[name])
    L = 2 * len(params["blocks"]) + 1
    ctx.karma_set_param(L, 0, params["lnf_g"])
    ctx.karma_set_param(L, 1, params["lnf_b"])


def all_grads_split(ctx, n_blocks):
    out = {"wte": ctx.karma_get_grad(0, 0), "wpe": ctx.karma_get_grad(0, 1)}
    for i in range(n_blocks):
        for t, name in enumerate(BLOCK_T):
            out["b%d.%s" % (i, name)] = ctx.karma_get_grad(*split_slot(i, t))
    out["lnf_g"] = ctx.karma_get_grad(2 * n_blocks + 1, 0)
    out["lnf_b"] = ctx.karma_get_grad(2 * n_blocks + 1, 1)
    return out


def test_blocks_split_into_attention_and_feed_forward_records(g):
    """split_blocks: the planner sees two records per transformer block.  The same kernels run in the same
    order, so loss and gradients equal those of whole blocks bit for bit, under any plan over the seven
    records; the plan equals the oracle's plan on the context's cost records; Adam reaches the same weights."""
    params, ids, labels = small_problem()
    whole = make_ctx(arena=512 << 20, **SMALL)
    load_params(whole, params)
    whole.karma_set_plan(512 << 20, [K.KEEP] * 4)
    loss = whole.karma_step(ids, labels)
    ref = all_grads(whole, 3)

    ctx = split_ctx(512 << 20, SMALL)
    load_params_split(ctx, params)
    layers, loss_c, fixed = ctx.karma_get_costs()
    assert len(layers) == 7
    lw = whole.karma_get_costs()[0]
    # the halves' saved sets make up the block's but for r1, which is now the attention half's output
    assert layers[1][3] + layers[2][3] + layers[1][4] == lw[1][3]
    assert layers[1][6] + layers[2][6] == lw[1][6] and layers[1][6] > 0 or lw[1][6] == 0
    big = 512 << 20
    plans = [[K.KEEP] * 7,
             [K.KEEP, K.KEEP, K.RC_KEEP, K.KEEP, K.RC_KEEP, K.KEEP, K.RC_KEEP],        # feed-forward halves recomputed
             [K.KEEP, K.RC_KEEP, K.RC_CHAIN, K.SWAP, K.RC_SWAP, K.RC_KEEP, K.KEEP],
             [K.SWAP, K.RC_SWAP, K.RC_CHAIN, K.RC_CHAIN, K.RC_CHAIN, K.SWAP, K.SWAP]]
    for pl in plans:
        ctx.karma_set_plan(big, pl)
        assert ctx.karma_step(ids, labels) == loss, pl
        for name, v in all_grads_split(ctx, 3).items():
            assert np.array_equal(v, ref[name]), (pl, name)
    # planner parity on the seven records, under a budget that forces choices
    layers = [(1000 + 10 * i, 2000 + 10 * i, 1000 + 10 * i) + l[3:] for i, l in enumerate(layers)]
    link = (2 * 10**9, 2 * 10**9, 1000)
    loss_c = (3000,) + tuple(loss_c[1:])
    ctx.karma_set_costs(layers, loss_c, link)
    budget = fixed + int(0.55 * sum(l[3] + l[4] for l in layers)) + max(max(l[5] for l in layers), loss_c[1])
    acts, summ = ctx.karma_plan(budget)
    ao, so = P.plan([P.Layer(*l) for l in layers], P.Link(*link), budget, fixed, P.Loss(*loss_c))
    assert acts == ao and summ["makespan_ns"] == so["makespan_ns"] and summ["peak_bytes"] == so["peak_bytes"]
    assert acts != [K.KEEP] * 7
    assert ctx.karma_step(ids, labels) == loss
    for name, v in all_grads_split(ctx, 3).items():
        assert np.array_equal(v, ref[name]), name
    # one Adam step in both: the same master weights
    l0 = whole.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
    l1 = ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
    assert l0 == l1
    for blk, t in ((0, 2), (1, 8), (2, 11), (2, 0)):
        assert np.array_equal(whole.karma_get_param(blk + 1, t), ctx.karma_get_param(*split_slot(blk, t))), (blk, t)
    whole.close()
    ctx.close()


def test_profiled_step_gives_op_starts_in_stream_order(g):
    """KARMA_STEP_PROFILE: every op's begin and duration; ops of one stream follow each other without overlap,
    and the compute stream's busy time plus its idle gaps span the step."""
    params, ids, labels = small_problem()
    ctx = make_ctx(arena=512 << 20, **SMALL)
    load_params(ctx, params)
    ctx.karma_set_plan(512 << 20, [K.SWAP, K.RC_SWAP, K.RC_CHAIN, K.KEEP])
    ctx.karma_step(ids, labels, K.STEP_PROFILE)
    ops = ctx.karma_get_op_times()
    starts = ctx.karma_get_op_starts()
    assert len(starts) == len(ops) and starts[0] == 0.0
    streams = {"F": 0, "R": 0, "B": 0, "L": 0, "I": 1, "W": 1, "O": 2, "G": 2}
    last_end = {}
    for (kind, layer, _, _, ms), st in zip(ops, starts):
        sid = streams[kind]
        assert ms >= 0.0 and st >= 0.0
        if sid in last_end:
            assert st >= last_end[sid] - 0.02, (kind, layer, st, last_end[sid])   # event resolution
        last_end[sid] = st + ms
    compute = [(st, ms) for (kind, _, _, _, ms), st in zip(ops, starts) if streams[kind] == 0]
    busy = sum(ms for _, ms in compute)
    span = compute[-1][0] + compute[-1][1] - compute[0][0]
    assert busy <= span + 0.05 and abs(busy - ctx.karma_get_stats()["compute_busy_ms"]) <= 1e-3 * busy + 1e-3
    ctx.close()


@pytest.mark.parametrize("device_first", [0, 1], ids=["all_on_host", "first_record_on_device"])
def test_gpt_host_adam(g, device_first):
    """device_first: the embedding record's master weights and moments live in HBM and are updated there."""
    params, ids, labels = small_problem()
    ctx = make_ctx(arena=512 << 20, lr=1e-2, device_update_first=device_first, **SMALL)
    load_params(ctx, params)
    ctx.karma_set_plan(512 << 20, [K.KEEP, K.RC_KEEP, K.SWAP, K.KEEP])
    loss0 = ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
    grads = all_grads(ctx, 3)      # the device gradients of that step
    def check(layer, tensor, before, gname):
        w, m, v = nn.adam_update(np.asarray(before, np.float32).astype(np.float64).reshape(-1), 0.0, 0.0,
                                 grads[gname].astype(np.float64), 1, 1e-2)
        assert g.rel_l2(ctx.karma_get_param(layer, tensor), w) <= 1e-6, gname
    check(0, 0, params["wte"], "wte")
    check(0, 1, params["wpe"], "wpe")
    check(2, 2, params["blocks"][1]["wqkv"], "b1.wqkv")
    check(3, 11, params["blocks"][2]["b2"], "b2.b2")
    check(4, 0, params["lnf_g"], "lnf_g")
    loss1 = ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
    assert loss1 < loss0          # the update went in the descent direction and reached the device
    # a second update, on the first one's moments: the embedding tensors against the oracle's two steps
    g1 = all_grads(ctx, 3)
    for tensor, name in ((0, "wte"), (1, "wpe")):
        w0 = np.asarray(params[name], np.float32).astype(np.float64).reshape(-1)
        w1, m1, v1 = nn.adam_update(w0, 0.0, 0.0, grads[name].astype(np.float64), 1, 1e-2)
        w2, _, _ = nn.adam_update(w1, m1, v1, g1[name].astype(np.float64), 2, 1e-2)
        assert g.rel_l2(ctx.karma_get_param(0, tensor), w2) <= 1e-6, name
    layers, loss_c, fixed = ctx.karma_get_costs()
    if device_first:
        assert layers[0][9] == 0 and layers[0][10] == 0         # no gradients out, no weights back for record 0
        assert fixed >= 12 * (params["wte"].size + params["wpe"].size)
    else:
        assert layers[0][9] > 0 and layers[0][10] > 0
    ctx.close()


def test_gpt_rejects_bad_ids_and_shapes(g):
    ctx = make_ctx(arena=256 << 20, **SMALL)
    ctx.karma_set_plan(256 << 20, [0, 0, 0, 0])
    ids = np.zeros((2, 128), np.int32)
    bad = ids.copy(); bad[1, 5] = SMALL["vocab"]
    with pytest.raises(K.KarmaError) as e:
        ctx.karma_step(bad, ids)
    assert e.value.status == K.E_INVAL
    ctx.close()
    with pytest.raises(K.KarmaError):
        make_ctx(1, 96, 2, 64, 64, 128, 1, 64 << 20)        # head dim 48 unsupported
    with pytest.raises(K.KarmaError):
        make_ctx(1, 128, 2, 64, 64, 100, 1, 64 << 20)       # seq not a multiple of 128
