"""Block granularity chosen by the planner (Sec. III-E/F, first tier: grouping layers into blocks):
oracle properties, and the library against the oracle bit for bit.  CPU only."""
import pytest

import paper_2008_11421_amd as K
from oracle import planner as P
from test_oracle_planner import cases
from test_oracle_weight_stream import with_weights
from test_planner_parity import summaries_equal


def test_merge_and_expand_rules():
    a = P.Layer(tf=3, tb=5, trc=3, sav=100, out=40, ws=7)
    b = P.Layer(tf=2, tb=4, trc=2, sav=60, out=30, ws=9, wb=8, gb=4)
    c = P.Layer(tf=1, tb=1, trc=1, sav=10, out=20, ws=1)
    m = P.merge_group([a, b, c])
    # inner boundaries (outputs of a and b) become internals of the block; its output is c's
    assert m == P.Layer(tf=6, tb=10, trc=6, sav=100 + 60 + 10 + 40 + 30, out=20, ws=9, wb=8, gb=4)
    acts, wres = P.expand_group_actions([P.KEEP, P.RC_SWAP, P.RC_CHAIN, P.SWAP], [0, 1, 0, 1], [2, 3, 1, 2])
    assert acts == [P.KEEP, P.KEEP, P.RC_SWAP, P.RC_CHAIN, P.RC_CHAIN, P.RC_CHAIN, P.SWAP, P.SWAP]
    assert wres == [0, 0, 1, 1, 1, 0, 1, 1] and P.valid_actions(acts)


def test_grouped_plan_is_valid_and_never_worse_than_plain():
    n = 0
    for L, kinds in ((5, ("homogeneous", "front_heavy", "back_heavy", "imbalanced")), (9, ("back_heavy", "imbalanced"))):
        for layers, link, budget, loss in cases(L, seeds=(0,), kinds=kinds, fracs=(0.35, 0.7), bwmuls=(0.3, 4.0)):
            try:
                acts, res, g = P.plan_grouped(layers, link, budget, 0, loss)
            except P.Infeasible:
                with pytest.raises(P.Infeasible):
                    P.plan(layers, link, budget, 0, loss)
                continue
            assert P.valid_actions(acts) and g in P.GROUP_SIZES
            # the summary is the per-layer simulator's for exactly these actions
            again = P.simulate(layers, link, budget, 0, loss, acts, wres=res["wres"])
            assert again["makespan_ns"] == res["makespan_ns"] and again["peak_bytes"] <= budget
            try:
                _, plain = P.plan(layers, link, budget, 0, loss)
                assert P.cost_tuple(res) <= P.cost_tuple(plain)
            except P.Infeasible:
                pass
            # max_group = 1 is the plain planner
            a1, r1, g1 = P.plan_grouped(layers, link, budget, 0, loss, max_group=1)
            assert g1 == 1 and a1 == P.plan(layers, link, budget, 0, loss)[0]
            n += 1
    assert n >= 8


def test_many_small_layers_behind_a_slow_link_prefer_blocks():
    """32 small equal layers, a link whose per-copy latency is as long as a layer: layer-by-layer
    plans pay the latency per layer, blocks amortise it; the grouped planner must do at least as well
    and its choice must be a valid plan within the budget."""
    layers = [P.Layer(tf=1000, tb=2000, trc=1000, sav=4096, out=1024, ws=0) for _ in range(32)]
    link = P.Link(bw_h2d=10**10, bw_d2h=10**10, lat_ns=1000)
    budget = 20 * (4096 + 1024)
    acts, res, g = P.plan_grouped(layers, link, budget, 0, P.Loss(500, 0))
    _, plain = P.plan(layers, link, budget, 0, P.Loss(500, 0))
    assert res["makespan_ns"] <= plain["makespan_ns"] and res["peak_bytes"] <= budget


def test_library_bit_exact():
    n = 0
    for L, seeds, kinds in ((6, (0,), ("homogeneous", "front_heavy", "back_heavy", "imbalanced")), (11, (2,), ("front_heavy", "imbalanced"))):
        for base, link, budget, loss in cases(L, seeds=seeds, kinds=kinds, fracs=(0.35, 0.7), bwmuls=(1.0,)):
            for layers in (base, with_weights(base, 5, scale=1.5)):
                bud = budget + (2 * max(P.al(l.wb) + P.al(l.gb) for l in layers) if layers is not base else 0)
                try:
                    ao, so, go = P.plan_grouped(layers, link, bud, 0, loss)
                except P.Infeasible:
                    with pytest.raises(K.KarmaError) as e:
                        K.karma_plan_grouped_pure(layers, link, loss, bud, 0)
                    assert e.value.status == K.E_BUDGET
                    continue
                al, sl, gl = K.karma_plan_grouped_pure(layers, link, loss, bud, 0)
                assert al == ao and gl == go and sl["wres"] == so["wres"]
                summaries_equal(sl, so)
                for mg in (3,):
                    ao2, so2, go2 = P.plan_grouped(layers, link, bud, 0, loss, max_group=mg)
                    al2, sl2, gl2 = K.karma_plan_grouped_pure(layers, link, loss, bud, 0, max_group=mg)
                    assert al2 == ao2 and gl2 == go2
                n += 1
    assert n >= 4
    with pytest.raises(K.KarmaError) as e:
        K.karma_plan_grouped_pure(base, link, loss, budget, 0, max_group=0)
    assert e.value.status == K.E_INVAL
