"""Acceptance (a): the library planner and simulator agree with the oracle bit for bit.
CPU only: the planner entry points need no GPU."""
import pytest

import paper_2008_11421_amd as K
from oracle import planner as P
import synth_inputs as si
from test_oracle_planner import cases, golden_schedule, mk, six_block_model

KIND = {"F": "F", "B": "B", "R": "R", "L": "L", "OUT": "O", "IN": "I", "WIN": "W", "GOUT": "G", "HOLD": "H"}


def ops_equal(lib_ops, ora_ops):
    assert len(lib_ops) == len(ora_ops)
    for a, b in zip(lib_ops, ora_ops):
        assert chr(a.kind) == KIND[b.kind] and a.layer == b.layer
        assert (a.start_ns, a.end_ns) == (b.start, b.end)
        offs = [(-1 if o is None else o) for o in b.offs] + [-1] * (3 - len(b.offs))
        assert list(a.off) == offs


def summaries_equal(s_lib, s_ora):
    for k in ("makespan_ns", "stall_ns", "busy_ns", "recompute_ns", "peak_bytes", "bytes_d2h", "bytes_h2d", "host_busy_ns",
              "host_end_ns"):
        assert s_lib[k] == s_ora[k], k


def all_vectors(L, stride, seed):
    """A deterministic sample of valid action vectors."""
    r = [int(v) for v in si.splitmix64(seed, 400 * L)]
    for k in range(0, len(r) - L, L * stride):
        v = [r[k + i] % 5 for i in range(L)]
        if P.valid_actions(v):
            yield v


def test_simulator_bit_exact_on_random_vectors():
    n = 0
    for layers, link, budget, loss in cases(7, seeds=(3,), fracs=(0.4, 0.9), bwmuls=(0.5, 3.0)):
        for v in all_vectors(7, 1, 17):
            try:
                so = P.simulate(layers, link, budget, 0, loss, v, want_ops=True)
            except P.Infeasible:
                with pytest.raises(K.KarmaError) as e:
                    K.karma_simulate(layers, link, loss, budget, 0, v)
                assert e.value.status == K.E_BUDGET
                continue
            sl, ops = K.karma_simulate(layers, link, loss, budget, 0, v, want_ops=True)
            summaries_equal(sl, so)
            ops_equal(ops, so["ops"])
            assert K.karma_stage_string(ops) == P.stage_string(so["ops"])
            n += 1
    assert n > 200


def test_plan_bit_exact_on_random_stacks():
    for L, seeds in ((6, (0, 1, 2)), (11, (4,))):
        for layers, link, budget, loss in cases(L, seeds=seeds, fracs=(0.35, 0.7)):
            try:
                ao, so = P.plan(layers, link, budget, 0, loss)
            except P.Infeasible:
                with pytest.raises(K.KarmaError):
                    K.karma_plan_pure(layers, link, loss, budget, 0)
                continue
            al, sl = K.karma_plan_pure(layers, link, loss, budget, 0)
            assert al == ao
            summaries_equal(sl, so)


def test_worked_example_through_library():
    layers, link, loss = six_block_model()
    acts = [K.SWAP, K.RC_KEEP, K.SWAP, K.RC_KEEP, K.KEEP, K.KEEP]
    s, ops = K.karma_simulate(layers, link, loss, 10**6, 0, acts, want_ops=True)
    assert K.karma_stage_string(ops) == golden_schedule()
    assert s["stall_ns"] == 0 and s["makespan_ns"] == 14000


def test_fixed_region_and_errors():
    layers = mk(1, 4, "homogeneous")
    link, loss = (10**9, 10**9, 0), (0, 0)
    with pytest.raises(K.KarmaError) as e:
        K.karma_plan_pure(layers, link, loss, 4096, 0)
    assert e.value.status == K.E_BUDGET
    with pytest.raises(K.KarmaError) as e:
        K.karma_simulate(layers, link, loss, 10**6, 0, [4, 0, 0, 0])
    assert e.value.status == K.E_INVAL
    with pytest.raises(K.KarmaError) as e:
        K.karma_simulate(layers, (0, 1, 0), loss, 10**6, 0, [0, 0, 0, 0])
    assert e.value.status == K.E_INVAL
    s1 = K.karma_simulate(layers, link, loss, 10**6 + 5000, 5000, [0] * 4)
    s0 = P.simulate([P.Layer(*l) for l in layers], P.Link(*link), 10**6 + 5000, 5000, P.Loss(*loss), [0] * 4)
    summaries_equal(s1, s0)


def test_streamed_weights_bit_exact():
    """Simulator and planner with streamed weights (Sec. III-G) against the oracle: random
    action vectors times random weight choices, then whole plans."""
    from test_oracle_weight_stream import with_weights
    n = 0
    for base, link, budget, loss in cases(7, seeds=(8,), fracs=(0.45, 0.9), bwmuls=(0.5, 3.0)):
        layers = with_weights(base, 21, scale=2.0)
        budget += 2 * max(P.al(l.wb) + P.al(l.gb) for l in layers)
        bits = [int(v) for v in si.splitmix64(5, 64)]
        for vi, v in enumerate(all_vectors(7, 3, 29)):
            wres = [(bits[(vi + k) % 64] >> k) & 1 if layers[k].wb else 0 for k in range(7)]
            try:
                so = P.simulate(layers, link, budget, 0, loss, v, want_ops=True, wres=wres)
            except P.Infeasible:
                with pytest.raises(K.KarmaError) as e:
                    K.karma_simulate(layers, link, loss, budget, 0, v, weights_kept=wres)
                assert e.value.status == K.E_BUDGET
                continue
            sl, ops = K.karma_simulate(layers, link, loss, budget, 0, v, want_ops=True, weights_kept=wres)
            summaries_equal(sl, so)
            ops_equal(ops, so["ops"])
            assert K.karma_stage_string(ops) == P.stage_string(so["ops"])
            n += 1
        try:
            ao, so = P.plan(layers, link, budget, 0, loss)
        except P.Infeasible:
            with pytest.raises(K.KarmaError):
                K.karma_plan_pure(layers, link, loss, budget, 0)
            continue
        al, sl = K.karma_plan_pure(layers, link, loss, budget, 0)
        assert al == ao and sl["wres"] == so["wres"]
        summaries_equal(sl, so)
    assert n > 100


def with_host(layers, seed, streamed=False):
    """Host-optimiser fields on every record: update times from a tenth of to three times the record's
    backward time, gradient / weight bytes of resident records around the size of their output."""
    r = [int(v) for v in si.splitmix64(seed, 4 * len(layers))]
    out = []
    for k, l in enumerate(layers):
        th = l.tb * (1 + r[4 * k] % 30) // 10
        if streamed and l.wb:
            out.append(l._replace(th=th))
        else:
            out.append(l._replace(th=th, hg=64 * (1 + r[4 * k + 1] % 64), hw=32 * (1 + r[4 * k + 2] % 64)))
    return out


def test_host_queue_bit_exact():
    """Simulator and planner with the host-optimiser queue and the loaded link rates (Sec. III-G, stages 3 and 5)
    against the oracle: random vectors, then whole plans, with resident and with streamed weights."""
    from test_oracle_weight_stream import with_weights
    n = 0
    for streamed in (False, True):
        for base, link, budget, loss in cases(7, seeds=(6,), fracs=(0.45, 0.9), bwmuls=(0.5, 3.0)):
            layers = with_weights(base, 23, scale=2.0) if streamed else base
            layers = with_host(layers, 31, streamed)
            if streamed:
                budget += 2 * max(P.al(l.wb) + P.al(l.gb) for l in layers)
            link = link._replace(bw_h2d_loaded=link.bw_h2d * 3 // 4, bw_d2h_loaded=link.bw_d2h * 2 // 3)
            loss = loss._replace(th=77, hg=640, hw=320)
            for vi, v in enumerate(all_vectors(7, 3, 41)):
                wres = [(vi >> k) & 1 if layers[k].wb else 0 for k in range(7)]
                try:
                    so = P.simulate(layers, link, budget, 0, loss, v, want_ops=True, wres=wres)
                except P.Infeasible:
                    with pytest.raises(K.KarmaError) as e:
                        K.karma_simulate(layers, link, loss, budget, 0, v, weights_kept=wres)
                    assert e.value.status == K.E_BUDGET
                    continue
                sl, ops = K.karma_simulate(layers, link, loss, budget, 0, v, want_ops=True, weights_kept=wres)
                summaries_equal(sl, so)
                ops_equal(ops, so["ops"])
                assert so["host_busy_ns"] == sum(l.th for l in layers) + loss.th
                n += 1
            try:
                ao, so = P.plan(layers, link, budget, 0, loss)
            except P.Infeasible:
                with pytest.raises(K.KarmaError):
                    K.karma_plan_pure(layers, link, loss, budget, 0)
                continue
            al, sl = K.karma_plan_pure(layers, link, loss, budget, 0)
            assert al == ao and sl["wres"] == so["wres"]
            summaries_equal(sl, so)
            ag, sg, gg = K.karma_plan_grouped_pure(layers, link, loss, budget, 0)
            aog, sog, gog = P.plan_grouped(layers, link, budget, 0, loss)
            assert (ag, gg) == (aog, gog)
            summaries_equal(sg, sog)
    assert n > 150


# ---- connections between non-consecutive layers ---------------------------------------
def graph_cases(seed, n, L_range=(4, 8)):
    import random
    from test_oracle_skips import random_case
    rng = random.Random(seed)
    for _ in range(n):
        L = rng.randrange(*L_range)
        layers, skips, link = random_case(rng, L)
        if rng.random() < 0.4:          # some stacks with host updates and loaded link rates
            layers = [l._replace(th=rng.randrange(0, 90), hg=rng.randrange(0, 3) * 128, hw=rng.randrange(0, 3) * 128) for l in layers]
            link = link._replace(bw_h2d_loaded=link.bw_h2d // 2, bw_d2h_loaded=link.bw_d2h * 2 // 3)
        full = P.simulate(layers, link, 1 << 30, 0, P.Loss(5, 256), [0] * L, skips=skips)["peak_bytes"]
        yield layers, skips, link, P.Loss(5, 256), full, rng


def test_graph_simulator_bit_exact():
    n = unfit = 0
    for layers, skips, link, loss, full, rng in graph_cases(21, 40):
        L = len(layers)
        for frac in (0.5, 0.8, 2.0):
            budget = int(full * frac)
            for _ in range(30):
                v = [rng.randrange(5) for _ in range(L)]
                if not P.valid_actions(v, skips):
                    if P.valid_actions(v):
                        with pytest.raises(K.KarmaError) as e:
                            K.karma_simulate_graph(layers, link, loss, budget, 0, skips, v)
                        assert e.value.status == K.E_INVAL
                    continue
                try:
                    so = P.simulate(layers, link, budget, 0, loss, v, want_ops=True, skips=skips)
                except P.Infeasible:
                    with pytest.raises(K.KarmaError) as e:
                        K.karma_simulate_graph(layers, link, loss, budget, 0, skips, v)
                    assert e.value.status == K.E_BUDGET
                    unfit += 1
                    continue
                sl, ops = K.karma_simulate_graph(layers, link, loss, budget, 0, skips, v, want_ops=True)
                summaries_equal(sl, so)
                ops_equal(ops, so["ops"])
                n += 1
    assert n > 300 and unfit > 50


def test_graph_plan_bit_exact():
    n = none = 0
    for layers, skips, link, loss, full, rng in graph_cases(22, 9, L_range=(5, 9)):
        for frac in (0.45, 0.7):
            budget = int(full * frac)
            try:
                ao, so = P.plan(layers, link, budget, 0, loss, skips)
            except P.Infeasible:
                with pytest.raises(K.KarmaError) as e:
                    K.karma_plan_graph(layers, link, loss, budget, 0, skips)
                assert e.value.status == K.E_BUDGET
                none += 1
                continue
            al, sl = K.karma_plan_graph(layers, link, loss, budget, 0, skips)
            assert al == ao, (skips, budget)
            summaries_equal(sl, so)
            n += 1
    assert n >= 8 and none >= 1


def test_graph_grouped_plan_bit_exact_and_bad_connections():
    for layers, skips, link, loss, full, rng in graph_cases(23, 4, L_range=(8, 11)):
        link = link._replace(lat_ns=60)
        budget = int(full * 0.65)
        try:
            ao, so, go = P.plan_grouped(layers, link, budget, 0, loss, skips=skips)
        except P.Infeasible:
            with pytest.raises(K.KarmaError):
                K.karma_plan_grouped_graph(layers, link, loss, budget, 0, skips)
            continue
        al, sl, gl = K.karma_plan_grouped_graph(layers, link, loss, budget, 0, skips)
        assert (al, gl) == (ao, go)
        summaries_equal(sl, so)
        assert sl["wres"] == so["wres"]
    layers = mk(1, 5, "homogeneous")
    for bad in ([(0, 1)], [(3, 5)], [(4, 2)]):
        with pytest.raises(K.KarmaError) as e:
            K.karma_plan_graph(layers, (10**9, 10**9, 0), (0, 0), 1 << 30, 0, bad)
        assert e.value.status == K.E_INVAL


def test_smallest_budgets_bit_exact_without_connections():
    """Budgets around the smallest that fits, where no start pattern may fit and the search's
    feasibility phase runs: both implementations find the same assignment or none."""
    found = none = 0
    for L, seeds in ((5, (0, 1)), (7, (5,))):
        for layers, link, budget, loss in cases(L, seeds=seeds, fracs=(0.0,), bwmuls=(1.0,)):
            for q in (0.6, 0.95, 1.0, 1.05):
                b = int(budget * q)
                try:
                    ao, so = P.plan(layers, link, b, 0, loss)
                except P.Infeasible:
                    with pytest.raises(K.KarmaError):
                        K.karma_plan_pure(layers, link, loss, b, 0)
                    none += 1
                    continue
                al, sl = K.karma_plan_pure(layers, link, loss, b, 0)
                assert al == ao
                summaries_equal(sl, so)
                found += 1
    assert found and none


def test_premature_swap_in_through_library():
    """Four equal layers (forward 10, backward 20, 256-byte outputs, 1 byte/ns, loss 5), the input of
    layer 1 swapped and read again by layer 3: OUT 20-276, copy back 276-532, F3 532-542, makespan 627
    (worked out by hand in the oracle's pins)."""
    layers = [(10, 20, 5, 0, 256, 0)] * 4
    s, ops = K.karma_simulate_graph(layers, (10**9, 10**9, 0), (5, 0), 1 << 20, 0, [(0, 3)], [K.KEEP, K.SWAP, K.KEEP, K.KEEP],
                                    want_ops=True)
    assert [(o.start_ns, o.end_ns) for o in ops if chr(o.kind) == "I"] == [(276, 532)]
    assert [(o.start_ns, o.end_ns) for o in ops if chr(o.kind) == "F"][3] == (532, 542)
    assert s["makespan_ns"] == 627 and s["bytes_h2d"] == s["bytes_d2h"] == 256 and s["peak_bytes"] == 1536
    with pytest.raises(K.KarmaError) as e:      # the input of layer 2 is read again: it cannot be chained
        K.karma_simulate_graph(layers, (10**9, 10**9, 0), (5, 0), 1 << 20, 0, [(1, 3)], [K.KEEP, K.RC_KEEP, K.RC_CHAIN, K.KEEP])
    assert e.value.status == K.E_INVAL
