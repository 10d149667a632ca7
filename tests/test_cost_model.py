"""Analytic cost model (Sec. III-C operation counts projected on device rates): the oracle's counts
against closed forms and published totals, the library against the oracle bit for bit, and a batch
sweep through the planner on analytic costs alone.  CPU only."""
import pytest

import paper_2008_11421_amd as K
from oracle import cost_model as CM
from oracle import planner as P

RATES = (500 * 10**12, 2 * 10**12)     # matrix multiply-adds per second, other operations per second
GPT = dict(n_layers=24, hidden=1024, heads=16, ffn=4096, vocab=32000, seq=1024, batch=32)
CNN = dict(width=64, stage_blocks=(3, 24, 36, 3), image=224, batch=64, classes=1000)


def gpt_desc(batch=32, **over):
    g = dict(GPT, batch=batch, **over)
    return dict(kind=K.MODEL_GPT, n_layers=g["n_layers"], width=g["hidden"], batch=g["batch"], seq=g["seq"],
                n_heads=g["heads"], ffn=g["ffn"], vocab=g["vocab"], stream_weights=0, split_blocks=g.get("split_blocks", 0))


def cnn_desc(batch=64):
    return dict(kind=K.MODEL_CNN, n_layers=0, width=CNN["width"], batch=batch, seq=CNN["image"], n_heads=0, ffn=0,
                vocab=CNN["classes"], stream_weights=0, stage_blocks=CNN["stage_blocks"])


WRN = dict(width=160, group_blocks=(4, 4, 4), image=32, batch=128, classes=16)


def wrn_desc(batch=128):
    return dict(kind=K.MODEL_WRN, n_layers=0, width=WRN["width"], batch=batch, seq=WRN["image"], n_heads=0, ffn=0,
                vocab=WRN["classes"], stream_weights=0, stage_blocks=WRN["group_blocks"] + (0,))


UNET = dict(width=64, depth=4, image=512, batch=4, classes=8)


def unet_desc(batch=4):
    return dict(kind=K.MODEL_UNET, n_layers=UNET["depth"], width=UNET["width"], batch=batch, seq=UNET["image"], n_heads=0,
                ffn=0, vocab=UNET["classes"], stream_weights=0, stage_blocks=(0, 0, 0, 0))


# ------------------------------------------------------------------ oracle pins
def test_oracle_unet_counts_written_out():
    """Padded 3x3 convolutions keep the image size, so every level's convolution count has a closed form."""
    blocks, loss = CM.unet_blocks(**dict(UNET, batch=1))
    assert len(blocks) == 9
    px = 512 * 512
    assert blocks[0] == (px * 64 * 9 * (1 + 64), 20 * px * 64)
    # level 1: pooling of 64 channels down to 256x256, then 64 -> 128 -> 128
    assert blocks[1] == (px // 4 * 128 * 9 * (64 + 128), px // 4 * 64 * 4 + 20 * (px // 4) * 128)
    # lowest level
    assert blocks[4][0] == px // 256 * 1024 * 9 * (512 + 1024)
    # expansive level 3: up-convolution 1024 -> 512 on 64x64, then 1024 -> 512 -> 512
    assert blocks[5] == (px // 64 * 512 * (1024 + 9 * 1024 + 9 * 512), 20 * (px // 64) * 512)
    assert blocks[8][0] == px * 64 * (128 + 9 * 128 + 9 * 64)
    assert loss == (px * 64 * 8, 2 * px * 8)
    # channels double where pixels quarter, so every level below the first costs the same: contracting levels
    # 9 * 1.5 * 64^2 per level-0 pixel, expansive levels (2 + 18 + 9) * 64^2
    total = sum(b[0] for b in blocks) + loss[0]
    assert total == px * (64 * 9 * 65 + 4 * 9 * 3 * 64 * 64 // 2 + 4 * 29 * 64 * 64 + 64 * 8)


def test_oracle_wrn_28_10_total_and_blocks():
    """WRN-28-10 on a 32x32 image is known as a 5.2 G multiply-add network; its blocks written out."""
    blocks, loss = CM.wrn_blocks(**dict(WRN, batch=1))
    assert len(blocks) == 13
    total = sum(b[0] for b in blocks) + loss[0]
    assert 5.1e9 < total < 5.4e9
    assert blocks[0] == (32 * 32 * 16 * 27, 0)
    # first block: 16 -> 160 on 32x32, two 3x3 convolutions and the 1x1 shortcut
    assert blocks[1][0] == 32 * 32 * (160 * 9 * 16 + 160 * 9 * 160 + 160 * 16)
    assert blocks[1][1] == 32 * 32 * (10 * 16 + 10 * 160 + 160)
    assert blocks[2][0] == 32 * 32 * 2 * 160 * 9 * 160
    # first block of the second group: strided 3x3 from 32x32 to 16x16
    assert blocks[5][0] == 16 * 16 * (320 * 9 * 160 + 320 * 9 * 320 + 320 * 160)
    assert blocks[5][1] == 10 * 32 * 32 * 160 + 11 * 16 * 16 * 320
    assert loss == (640 * 16, 11 * 8 * 8 * 640 + 2 * 16)


def test_oracle_fully_connected_and_mlp_counts():
    blocks, loss = CM.mlp_blocks(width=256, n_layers=8, batch=32)
    assert len(blocks) == 8
    # |X| * |Y| per sample for the layer, |Y| comparisons for the ReLU
    assert blocks[0] == (32 * 256 * 256, 32 * 256)
    assert loss == (0, 32 * 256)


def test_oracle_gpt_block_matches_the_parameter_count_rule():
    """With ffn = 4 h a block's weight matrices hold 12 h^2 parameters, and every token meets every
    weight once: 12 h^2 multiply-adds per token, plus the attention products 2 S d per token and head."""
    blocks, loss = CM.gpt_blocks(**GPT)
    T, h, S = GPT["batch"] * GPT["seq"], GPT["hidden"], GPT["seq"]
    assert len(blocks) == GPT["n_layers"] + 1
    assert blocks[0][0] == 0
    assert blocks[1][0] == T * 12 * h * h + T * 2 * S * h
    assert all(b == blocks[1] for b in blocks[2:])
    assert loss[0] == T * h * GPT["vocab"]
    # whole forward pass in FLOP (2 per multiply-add): the 0.962 TFLOP per layer of the shape arithmetic
    assert abs(2 * blocks[1][0] / 0.962e12 - 1) < 0.01


def test_oracle_resnet200_total_is_the_published_size():
    """ResNet-200 at 224x224 is known as a ~15 G multiply-add network; the stem's convolution alone is
    112*112*64*147 and every stage's first block carries the projection."""
    blocks, loss = CM.cnn_blocks(**dict(CNN, batch=1))
    assert len(blocks) == 1 + sum(CNN["stage_blocks"])
    total = sum(b[0] for b in blocks) + loss[0]
    assert 14.5e9 < total < 15.5e9
    assert blocks[0][0] == 112 * 112 * 64 * 49 * 3
    # an identity block of stage 1: 1x1 (256->64), 3x3 (64->64), 1x1 (64->256) on 56x56
    assert blocks[2][0] == 56 * 56 * (64 * 256 + 64 * 9 * 64 + 256 * 64)
    # the first block reads the stem's 64 channels and carries the 64 -> 256 projection
    assert blocks[1][0] == 56 * 56 * (64 * 64 + 64 * 9 * 64 + 256 * 64 + 256 * 64)
    # first block of stage 2: 1x1 on 56x56 (256 -> 128), strided 3x3, 1x1 and projection on 28x28
    assert blocks[4][0] == 56 * 56 * 128 * 256 + 28 * 28 * (128 * 9 * 128 + 512 * 128 + 512 * 256)
    # batch norm = 9 per element, ReLU / add = 1 per element
    assert blocks[2][1] == 56 * 56 * (10 * 64 + 10 * 64 + 9 * 256 + 2 * 256)
    assert loss == (2048 * 1000, 7 * 7 * 2048 + 2 * 1000)


def test_oracle_counts_scale_with_batch_and_times_round_up():
    b1, l1 = CM.gpt_blocks(**dict(GPT, batch=1))
    b4, l4 = CM.gpt_blocks(**dict(GPT, batch=4))
    assert all(4 * x[0] == y[0] and 4 * x[1] == y[1] for x, y in zip(b1, b4))
    assert CM.time_ns((1, 0), (3, 1)) == 333333334      # ceil(1e9 / 3)
    assert CM.time_ns((0, 7), (1, 2 * 10**9)) == 4      # ceil(7e9 / 2e9)
    t, tl = CM.times(b1, l1, RATES)
    assert all(tb == 2 * tf and trc == tf for tf, tb, trc in t)
    assert tl == 3 * CM.time_ns(l1, RATES)


# ------------------------------------------------------------------ library against oracle
def check_times(desc, blocks, loss):
    layers, (t_loss, _), fixed = K.karma_model_costs(desc, *RATES)
    want, want_loss = CM.times(blocks, loss, RATES)
    assert [l[:3] for l in layers] == want
    assert t_loss == want_loss
    assert fixed > 0 and all(l[3] + l[4] > 0 for l in layers)
    return layers, fixed


def test_library_times_bit_exact():
    check_times(dict(kind=K.MODEL_MLP, n_layers=8, width=256, batch=32, seq=0, n_heads=0, ffn=0, vocab=0, stream_weights=0),
                *CM.mlp_blocks(256, 8, 32))
    for batch in (1, 8, 32):
        check_times(gpt_desc(batch), *CM.gpt_blocks(**dict(GPT, batch=batch)))
    check_times(gpt_desc(8, n_layers=72, hidden=3072, heads=24, ffn=12288, vocab=51200),
                *CM.gpt_blocks(n_layers=72, hidden=3072, heads=24, ffn=12288, vocab=51200, seq=1024, batch=8))
    for batch in (2, 64):
        check_times(cnn_desc(batch), *CM.cnn_blocks(**dict(CNN, batch=batch)))
    for batch in (4, 128):
        check_times(wrn_desc(batch), *CM.wrn_blocks(**dict(WRN, batch=batch)))
    for batch in (1, 16):
        check_times(unet_desc(batch), *CM.unet_blocks(**dict(UNET, batch=batch)))


def test_unet_connections_and_plan_on_analytic_costs():
    """The library names the model's connections, and its planner on the analytic costs agrees with the oracle
    planner given the same connections; with connections present no record whose input is read again is chained."""
    desc = unet_desc(16)
    skips = K.karma_model_skips(desc)
    assert skips == [(0, 8), (1, 7), (2, 6), (3, 5)]
    assert K.karma_model_skips(wrn_desc()) == []
    layers, (t_loss, ws_loss), fixed = K.karma_model_costs(desc, *RATES)
    link = (50 * 10**9, 50 * 10**9, 10000)
    need = fixed + sum(l[3] + l[4] for l in layers)
    seen = set()
    for share in (1.0, 0.6, 0.4):
        budget = fixed + int((need - fixed) * share) + 2 * max(l[5] for l in layers)
        ao, so = P.plan([P.Layer(*l) for l in layers], P.Link(*link), budget, fixed, P.Loss(t_loss, ws_loss), skips=skips)
        al, sl = K.karma_plan_graph(layers, link, (t_loss, ws_loss), budget, fixed, skips)
        assert list(al) == list(ao) and sl["makespan_ns"] == so["makespan_ns"] and sl["peak_bytes"] == so["peak_bytes"]
        assert all(al[s + 1] != P.RC_CHAIN for s, _ in skips)
        seen.add(tuple(al))
    assert len(seen) >= 2


def test_split_transformer_blocks_counts_and_bytes():
    """Two records per block: their counts add up to the whole block's, the library's times equal the oracle's,
    and the halves' bytes make up the block's (r1 moves from the saved set to the attention half's output)."""
    whole, loss = CM.gpt_blocks(**GPT)
    halves, loss2 = CM.gpt_blocks(split=True, **GPT)
    assert loss == loss2 and len(halves) == 2 * GPT["n_layers"] + 1 and halves[0] == whole[0]
    for k in range(GPT["n_layers"]):
        a, f = halves[2 * k + 1], halves[2 * k + 2]
        assert (a[0] + f[0], a[1] + f[1]) == whole[k + 1]
    T, h, ffn = GPT["batch"] * GPT["seq"], GPT["hidden"], GPT["ffn"]
    assert halves[2][0] == T * 2 * h * ffn                      # FC1 and FC2
    lay_s, fixed_s = check_times(gpt_desc(split_blocks=1), halves, loss)
    lay_w, fixed_w = check_times(gpt_desc(), whole, loss)
    assert fixed_s == fixed_w
    for k in range(GPT["n_layers"]):
        a, f, w = lay_s[2 * k + 1], lay_s[2 * k + 2], lay_w[k + 1]
        assert a[3] + f[3] + a[4] == w[3] and a[4] == f[4] == w[4]
        assert a[6] + f[6] == w[6] and a[7] + f[7] == w[7]


def test_library_bytes_match_the_shape_arithmetic():
    """Per-block saved set of the benchmark GPT: 1.00 GiB, boundary tensor 64 MiB (shape arithmetic:
    tokens x hidden x 2 bytes); they scale linearly with the batch."""
    layers, _ = check_times(gpt_desc(32), *CM.gpt_blocks(**GPT))
    sav, out = layers[1][3], layers[1][4]
    assert out == 32 * 1024 * 1024 * 2
    assert abs(sav / 2**30 - 1.0) < 0.08
    layers8, _ = check_times(gpt_desc(8), *CM.gpt_blocks(**dict(GPT, batch=8)))
    assert layers8[1][4] * 4 == out and abs(layers8[1][3] * 4 / sav - 1) < 0.01


def test_errors():
    with pytest.raises(K.KarmaError):
        K.karma_model_costs(gpt_desc(32), 0, 1)
    with pytest.raises(K.KarmaError):
        K.karma_model_costs(dict(kind=9, n_layers=1, width=8, batch=1, seq=8, n_heads=1, ffn=8, vocab=8, stream_weights=0), 1, 1)


# ------------------------------------------------------------------ batch sweep on analytic costs
def test_batch_sweep_first_point_fits_rest_do_not():
    """The projection the analytic model is for: one budget, growing batch.  The smallest batch fits
    in-core (all KEEP, no stall); larger ones need swapping or recompute, the predicted rate per sample
    never improves once out of core, and library and oracle planner agree on every point."""
    budget = 16 * 2**30
    link = (57 * 10**9, 57 * 10**9, 6000)
    rates = []
    for batch in (8, 16, 32, 64):
        layers, loss, fixed = K.karma_model_costs(gpt_desc(batch), *RATES)
        try:
            acts, summ = K.karma_plan_pure(layers, link, loss, budget, fixed)
        except K.KarmaError as e:
            assert e.status == K.E_BUDGET
            with pytest.raises(P.Infeasible):
                P.plan([P.Layer(*l) for l in layers], P.Link(*link), budget, fixed, P.Loss(*loss))
            rates.append(None)
            continue
        ao, so = P.plan([P.Layer(*l) for l in layers], P.Link(*link), budget, fixed, P.Loss(*loss))
        assert acts == ao and summ["makespan_ns"] == so["makespan_ns"]
        in_core_ns = sum(l[0] + l[1] for l in layers) + loss[0]
        if batch == 8:
            assert acts == [K.KEEP] * len(acts) and summ["makespan_ns"] == in_core_ns
        else:
            assert summ["makespan_ns"] >= in_core_ns
        rates.append((batch * 10**9 / summ["makespan_ns"], acts, in_core_ns / summ["makespan_ns"]))
    assert rates[0] is not None and rates[0][1] == [K.KEEP] * 25
    assert any(r is not None and r[1] != [K.KEEP] * 25 for r in rates[1:])
    # the share of the in-core rate that the plan keeps is 1 while the batch fits and only falls as
    # the batch grows past the budget (more to swap or recompute per byte of memory)
    share = [r[2] for r in rates if r is not None]
    assert share[0] == 1.0 and all(b <= a for a, b in zip(share, share[1:])) and share[-1] < 1.0
