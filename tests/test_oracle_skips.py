"""Pins of the planner oracle's treatment of connections between non-consecutive layers
(Sec. III-F.3: a swapped tensor that a later layer reads again needs a premature swap-in;
recomputing from a kept checkpoint avoids it).  Expected timelines are worked out by hand
in the comments; the rest are invariants and brute force."""
import itertools
import random

import pytest

from oracle import planner as P

K, S, RK, RS, RC = P.KEEP, P.SWAP, P.RC_KEEP, P.RC_SWAP, P.RC_CHAIN

# four equal layers: forward 10, backward 20, recompute 5, no internals, 256-byte outputs,
# no workspace; 1 byte/ns each way, no latency; loss 5
FOUR = [P.Layer(10, 20, 5, 0, 256, 0)] * 4
LINK = P.Link(10**9, 10**9, 0)
LOSS = P.Loss(5, 0)
BIG = 1 << 20
X1_TO_3 = ((0, 3),)         # the output of layer 0 (= x_1, the input of layer 1) is read again by layer 3


def sim(acts, skips=(), budget=BIG, layers=FOUR, ops=False):
    return P.simulate(layers, LINK, budget, 0, LOSS, acts, want_ops=ops, skips=skips)


def spans(res, kind):
    return [(o.layer, o.start, o.end) for o in res["ops"] if o.kind == kind]


def test_kept_source_costs_memory_not_time():
    # F 0-40, L 40-45, B3 45-65, B2 -85, B1 -105, B0 -125, with or without the connection
    a = sim([K] * 4)
    b = sim([K] * 4, X1_TO_3)
    assert a["makespan_ns"] == b["makespan_ns"] == 125
    assert b["bytes_d2h"] == b["bytes_h2d"] == 0
    # without: x1..x4 + dx4 at the loss = 5 buffers; at B3 x1..x3 + dx4 + dx3 = 5 -> 1280.
    # with: B3 also leaves the gradient w.r.t. x1, which lives until B1 adds it in -> 1536
    assert a["peak_bytes"] == 1280 and b["peak_bytes"] == 1536
    assert sim([K] * 4, X1_TO_3, budget=1536)["makespan_ns"] == 125
    with pytest.raises(P.Infeasible):
        sim([K] * 4, X1_TO_3, budget=1535)      # 5 whole units of 256 only
    assert sim([K] * 4, (), budget=1280)["makespan_ns"] == 125


def test_swapped_source_needs_a_premature_swap_in():
    # x1 leaves after F1: OUT 20-276.  Its reader is layer 3, so the copy back is queued when F2
    # starts (t = 20) but the data must have reached the host first: IN 276-532.  F2 20-30,
    # F3 waits for x1: 532-542, L -547, B3 -567, B2 -587; x1 is already there and layer 1 has no
    # internals, so B1 fetches nothing: B1 -607, B0 -627.
    r = sim([K, S, K, K], X1_TO_3, ops=True)
    assert spans(r, "OUT") == [(1, 20, 276)]
    assert spans(r, "IN") == [(1, 276, 532)]
    assert spans(r, "F") == [(0, 0, 10), (1, 10, 20), (2, 20, 30), (3, 532, 542)]
    assert spans(r, "B") == [(3, 547, 567), (2, 567, 587), (1, 587, 607), (0, 607, 627)]
    assert r["makespan_ns"] == 627 and r["stall_ns"] == 502
    assert r["bytes_d2h"] == r["bytes_h2d"] == 256          # it comes back once, not twice
    # the same plan without the connection: x1 is fetched for B1 only (IN 276-532, issued at the
    # loss), which B3 and B2 (to 85) hide in part: B1 532-552, B0 -572
    q = sim([K, S, K, K], (), ops=True)
    assert spans(q, "IN") == [(1, 276, 532)] and q["makespan_ns"] == 572


def test_recomputed_source_stays_as_a_checkpoint():
    # a kept checkpoint is still there when layer 3 reads it: no copy, one recompute of 5
    r = sim([K, RK, K, K], X1_TO_3, ops=True)
    assert r["makespan_ns"] == 130 and r["bytes_d2h"] == 0 and spans(r, "R") == [(1, 85, 90)]
    # a swapped checkpoint behaves like the swapped tensor above, plus the recompute:
    # B2 ends at 587, R1 587-592, B1 -612, B0 -632
    r = sim([K, RS, K, K], X1_TO_3, ops=True)
    assert spans(r, "IN") == [(1, 276, 532)] and spans(r, "R") == [(1, 587, 592)]
    assert r["makespan_ns"] == 632


def test_swapped_source_with_internals_fetches_only_them_for_backward():
    # layer 1 with 512 bytes of internals: OUT moves 256 + 512 = 768 bytes, 20-788.  The
    # premature copy brings x1 alone: 788-1044, F3 1044-1054, L -1059.  The internals are
    # queued at the loss (t = 1054, after the forward pass): IN 1054-1566.  B3 1059-1079,
    # B2 -1099, B1 waits: 1566-1586, B0 -1606.
    layers = [P.Layer(10, 20, 5, 0, 256, 0), P.Layer(10, 20, 5, 512, 256, 0)] + [P.Layer(10, 20, 5, 0, 256, 0)] * 2
    r = sim([K, S, K, K], X1_TO_3, layers=layers, ops=True)
    assert spans(r, "OUT") == [(1, 20, 788)]
    assert spans(r, "IN") == [(1, 788, 1044), (1, 1054, 1566)]
    assert spans(r, "B")[2:] == [(1, 1566, 1586), (0, 1586, 1606)]
    assert r["bytes_d2h"] == r["bytes_h2d"] == 768 and r["makespan_ns"] == 1606


def test_two_readers_share_one_gradient_buffer():
    # x1 read again by layers 2 and 3: one extra buffer from B3 to B1, peak as with one reader
    r = sim([K] * 4, ((0, 2), (0, 3)))
    assert r["peak_bytes"] == 1536 and r["makespan_ns"] == 125
    # swapped: the first reader is layer 2, right behind layer 1 -> the copy back is issued when F2
    # starts, OUT 20-276, IN 276-532, F2 532-542, F3 -552, L -557, four backwards -> 637
    r = sim([K, S, K, K], ((0, 2), (0, 3)), ops=True)
    assert spans(r, "IN") == [(1, 276, 532)] and spans(r, "F")[2] == (2, 532, 542) and r["makespan_ns"] == 637


def test_a_tensor_read_again_cannot_be_dropped():
    assert not P.valid_actions([K, RK, RC, K], ((1, 3),))       # x2 would be dropped after F2
    assert P.valid_actions([K, RK, RC, K], ((0, 3),))
    with pytest.raises(ValueError):
        sim([K, RK, RC, K], ((1, 3),))
    for bad in (((0, 1),), ((2, 4),), ((3, 2),)):               # neighbours, out of range, backwards
        with pytest.raises(ValueError):
            sim([K] * 4, bad)


def random_case(rng, L):
    layers = [P.Layer(rng.randrange(5, 60), rng.randrange(10, 120), rng.randrange(2, 40),
                      rng.randrange(0, 4) * 128, rng.randrange(1, 5) * 256, rng.randrange(0, 2) * 256) for _ in range(L)]
    pairs = [(s, d) for s in range(L - 2) for d in range(s + 2, L)]
    skips = tuple(sorted(rng.sample(pairs, rng.randrange(1, min(3, len(pairs)) + 1))))
    link = P.Link(rng.choice([10**9, 4 * 10**9, 2 * 10**8]), rng.choice([10**9, 4 * 10**9]), rng.choice([0, 7]))
    return layers, skips, link


def test_every_swapped_byte_returns_exactly_once_and_the_ledger_closes():
    rng = random.Random(5)
    seen = 0
    for _ in range(60):
        L = rng.randrange(3, 7)
        layers, skips, link = random_case(rng, L)
        for acts in itertools.product((K, S, RK, RS, RC), repeat=L):
            if not P.valid_actions(acts, skips) or rng.random() > 0.08:
                continue
            try:
                r = P.simulate(layers, link, 1 << 20, 0, LOSS, list(acts), skips=skips)     # asserts an empty arena at the end
            except P.Infeasible:
                continue
            seen += 1
            assert r["bytes_d2h"] == r["bytes_h2d"]
            plain = P.simulate(layers, link, 1 << 20, 0, LOSS, list(acts))
            assert r["bytes_d2h"] == plain["bytes_d2h"] and r["busy_ns"] == plain["busy_ns"]
            assert r["peak_bytes"] >= plain["peak_bytes"] or any(acts[s + 1] in (S, RS) for s, _ in skips)
            if all(acts[s + 1] in (K, RK) for s, _ in skips):
                assert r["makespan_ns"] == plain["makespan_ns"]
    assert seen > 300


def test_plan_equals_brute_force_with_connections():
    rng = random.Random(13)
    hits = total = 0
    for _ in range(20):
        L = rng.randrange(4, 7)
        layers, skips, link = random_case(rng, L)
        full = P.simulate(layers, link, 1 << 30, 0, LOSS, [K] * L, skips=skips)["peak_bytes"]
        for frac in (0.55, 0.75):
            budget = int(full * frac)
            bf = P.brute_force(layers, link, budget, 0, LOSS, skips=skips)
            if bf is None:
                with pytest.raises(P.Infeasible):
                    P.plan(layers, link, budget, 0, LOSS, skips)
                continue
            acts, res = P.plan(layers, link, budget, 0, LOSS, skips)
            total += 1
            hits += (P.cost_tuple(res), acts) == bf
            assert res["makespan_ns"] <= bf[0][0] * 1.02
            assert P.valid_actions(acts, skips)
    assert total >= 8 and hits == total, (hits, total)


def test_contracting_path_is_recomputed_not_swapped():
    """An encoder-decoder stack of eight layers whose first three outputs are read again by the last
    three (Sec. III-F.3, connections from the contracting to the expansive path): at a budget that
    cannot keep everything, the optimum without the connections swaps early layers; with them every
    tensor that is read again is kept or recomputed from a kept checkpoint, never swapped, because
    its copy back would have to finish before the forward pass does."""
    layers = [P.Layer(40, 80, 20, 256, 1024, 0)] * 8
    skips = ((0, 7), (1, 6), (2, 5))
    link = P.Link(8 * 10**9, 8 * 10**9, 0)
    full = P.simulate(layers, link, 1 << 30, 0, LOSS, [K] * 8, skips=skips)["peak_bytes"]
    budget = int(full * 0.8)
    plain, _ = P.plan(layers, link, budget, 0, LOSS)
    acts, res = P.plan(layers, link, budget, 0, LOSS, skips)
    assert any(a in (S, RS) for a in plain[1:4])
    assert all(acts[s + 1] == RK for s, _ in skips)
    assert not [o for o in P.simulate(layers, link, budget, 0, LOSS, acts, want_ops=True, skips=skips)["ops"]
                if o.kind == "IN" and o.end <= 8 * 40]


def test_grouping_maps_connections_between_blocks():
    assert P.group_skips(((1, 5), (0, 3), (3, 5), (1, 3)), [2, 2, 2]) == ((0, 2),)
    assert P.group_skips(((2, 7),), [3, 3, 2]) == ((0, 2),)
    rng = random.Random(3)
    for _ in range(4):
        L = 8
        layers, skips, link = random_case(rng, L)
        link = P.Link(link.bw_h2d, link.bw_d2h, 40)
        full = P.simulate(layers, link, 1 << 30, 0, LOSS, [K] * L, skips=skips)["peak_bytes"]
        budget = int(full * 0.6)
        try:
            a1, r1 = P.plan(layers, link, budget, 0, LOSS, skips)
        except P.Infeasible:
            continue
        a2, r2, g = P.plan_grouped(layers, link, budget, 0, LOSS, skips=skips)
        assert P.valid_actions(a2, skips)
        assert P.cost_tuple(r2) <= P.cost_tuple(r1)
        assert P.cost_tuple(P.simulate(layers, link, budget, 0, LOSS, a2, wres=r2["wres"], skips=skips)) == P.cost_tuple(r2)
