"""Depth-truncated models at the true widths of the transformer workloads, whole step
against the plain oracle: two blocks, full sequence length and vocabulary, the batch cut to
one or two sequences so that the fp64 oracle finishes in seconds.  These are the shapes the
small-model tests cannot reach: 3072 / 12288 and the ragged 4256 / 17024 products, heads of
128 and 152 at 1024 positions, the 51200-wide chunked head."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import paper_2008_11421_amd as K
from oracle import nn
import synth_inputs as si
import test_gpu_gpt as TG

TOL = 2e-2          # the workload's bar for bf16 gradients, per tensor, relative L2


@pytest.fixture(scope="module")
def g():
    import gpu_util
    import torch
    assert torch.cuda.is_available()
    return gpu_util


@pytest.mark.parametrize("hidden,heads,ffn,vocab,batch,seed", [
    (1024, 16, 4096, 32000, 2, 2008114202),       # 24-layer workload's widths, batch 2 of 32
    (3072, 24, 12288, 51200, 1, 2008114204),      # 8.3B-parameter workload's widths, batch 1 of 8
    (4256, 28, 17024, 51200, 1, 2008114205),      # 17B-parameter workload's widths, batch 1 of 4
], ids=["h1024_batch2of32", "h3072_batch1of8", "h4256_batch1of4"])
def test_two_blocks_at_true_width_match_the_oracle(g, hidden, heads, ffn, vocab, batch, seed):
    dims = dict(n_layers=2, hidden=hidden, heads=heads, ffn=ffn, vocab=vocab, seq=1024, batch=batch)
    params, ids, labels = si.gpt_problem(seed=seed, n_layers=2, hidden=hidden, ffn=ffn, vocab=vocab, seq=1024,
                                         batch=batch, std=0.02, bias_std=0.02)
    ids, labels = ids.astype(np.int32), labels.astype(np.int32)
    arena = 8 << 30
    ctx = TG.make_ctx(arena=arena, **dims)
    TG.load_params(ctx, params)
    ctx.karma_set_plan(arena, [K.KEEP] * 3)
    loss = ctx.karma_step(ids, labels)
    got = TG.all_grads(ctx, 2)
    # a swapped and recomputed step of the same model: bit-identical
    ctx.karma_set_plan(arena, [K.KEEP, K.SWAP, K.RC_KEEP])
    assert ctx.karma_step(ids, labels) == loss
    for t in (2, 8, 10):
        assert np.array_equal(ctx.karma_get_grad(2, t), got["b1.%s" % TG.BLOCK_T[t]])
    ctx.close()

    lo, go, _, _ = nn.gpt_step(TG.rounded(params), ids, labels, heads)
    assert abs(loss - lo) <= 2e-3 * abs(lo), (loss, lo)
    want = TG.oracle_grads(go)
    bad = {}
    for name, v in got.items():
        e = g.rel_l2(v, want[name])
        if not e <= TOL:
            bad[name] = e
    assert not bad, bad
