"""Pins for the host-optimiser queue of the planner oracle (Sec. III-G, pipeline stages 3 and
5: gradients leave after a block's backward, the weights are updated on the CPU): timelines
computed by hand, and the invariants the queue must keep.  Link of 1 byte/ns, no latency,
unless said otherwise."""
import pytest

from oracle import planner as P

BIG = 10**6
LINK = P.Link(10**9, 10**9, 0)


def two_resident_layers():
    # tf 10, tb 20; layer 0: update 5 ns, 10 B of gradients out, 4 B of weights back;
    # layer 1: update 50 ns, 30 B out, 8 B back
    return [P.Layer(10, 20, 10, 0, 0, 0, 0, 0, th=5, hg=10, hw=4), P.Layer(10, 20, 10, 0, 0, 0, 0, 0, th=50, hg=30, hw=8)]


def test_resident_weights_timeline_by_hand():
    """F0 0-10, F1 10-20, loss 20-25, B1 25-45, B0 45-65.
    D2H: g1 45-75, g0 max(75, 65) = 75-85.  Host: u1 75-125, u0 max(125, 85) = 125-130.
    H2D (behind the program, which has no copies): w1 125-133, w0 max(133, 130) = 133-137."""
    r = P.simulate(two_resident_layers(), LINK, BIG, 0, P.Loss(5, 0), [P.KEEP, P.KEEP])
    assert r["makespan_ns"] == 137 and r["host_end_ns"] == 130 and r["host_busy_ns"] == 55
    assert r["busy_ns"] == 65 and r["stall_ns"] == 0
    assert r["bytes_d2h"] == 0 and r["bytes_h2d"] == 0       # nothing the plan chose to move


def test_loaded_link_rates_apply_after_the_forward_pass():
    """Loaded rates of 0.5 B/ns both ways: g1 45-105, g0 105-125; u1 105-155, u0 155-160;
    w1 155-171, w0 max(171, 160) = 171-179."""
    link = P.Link(10**9, 10**9, 0, 5 * 10**8, 5 * 10**8)
    r = P.simulate(two_resident_layers(), link, BIG, 0, P.Loss(5, 0), [P.KEEP, P.KEEP])
    assert r["makespan_ns"] == 179 and r["host_end_ns"] == 160
    # a swap-out happens in the forward phase (idle rate), its swap-in in the backward phase (loaded rate):
    # layer 1 swapped, input 40 B (layer 0's output) and 60 B of internals
    layers = [P.Layer(10, 20, 10, 0, 40, 0, th=1), P.Layer(10, 20, 10, 60, 0, 0)]
    r = P.simulate(layers, link, BIG, 0, P.Loss(5, 0), [P.KEEP, P.SWAP], want_ops=True)
    out = [o for o in r["ops"] if o.kind == "OUT"][0]
    inn = [o for o in r["ops"] if o.kind == "IN"][0]
    assert out.end - out.start == 100 and inn.end - inn.start == 200
    # without host updates the link is never loaded
    layers = [P.Layer(10, 20, 10, 0, 40, 0), P.Layer(10, 20, 10, 60, 0, 0)]
    r = P.simulate(layers, link, BIG, 0, P.Loss(5, 0), [P.KEEP, P.SWAP], want_ops=True)
    inn = [o for o in r["ops"] if o.kind == "IN"][0]
    assert inn.end - inn.start == 100


def test_streamed_weights_update_after_their_gradients_land():
    """One layer with streamed weights (100 B in, 40 B of gradients out), update 30 ns; loss record with
    a 7 ns update of its own (no bytes).  W 0-100, F 100-110, loss 110-115 (its update 115-122),
    B 115-135, G 135-175, update max(122, 175) = 175-205; the new weights stay on the host."""
    layers = [P.Layer(10, 20, 10, 0, 0, 0, 100, 40, th=30)]
    r = P.simulate(layers, LINK, BIG, 0, P.Loss(5, 0, th=7), [P.KEEP], wres=[1])
    assert r["makespan_ns"] == 205 and r["host_busy_ns"] == 37 and r["bytes_h2d"] == 100 and r["bytes_d2h"] == 40


def test_weights_go_back_behind_the_programs_own_copies():
    """The program's swap-in is enqueued ahead of time, so a weight copy that becomes ready earlier still
    runs after it.  Layer 0 swapped (internals 300 B): out 10-310, in max(loss start 20, 310) = 310-610,
    B0 waits for it.  Layer 1's gradients (5 B) queue behind that swap-out: 310-315; its update 315-320 is done long before its
    8 B of weights go back at 610-618."""
    layers = [P.Layer(10, 20, 10, 300, 0, 0), P.Layer(10, 20, 10, 0, 0, 0, 0, 0, th=5, hg=5, hw=8)]
    r = P.simulate(layers, LINK, BIG, 0, P.Loss(5, 0), [P.SWAP, P.KEEP], want_ops=True)
    inn = [o for o in r["ops"] if o.kind == "IN"][0]
    assert (inn.start, inn.end) == (310, 610)
    b0 = [o for o in r["ops"] if o.kind == "B" and o.layer == 0][0]
    assert (b0.start, b0.end) == (610, 630)
    assert r["host_end_ns"] == 320 and r["makespan_ns"] == 630 and r["bytes_h2d"] == 300


def test_no_host_fields_no_change():
    """Records without host updates give the timeline they always gave."""
    layers = [P.Layer(10, 20, 10, 64, 32, 0), P.Layer(12, 25, 11, 64, 32, 0), P.Layer(9, 18, 9, 64, 32, 0)]
    r = P.simulate(layers, P.Link(10**9, 10**9, 3, 10**8, 10**8), BIG, 0, P.Loss(5, 0), [P.SWAP, P.RC_KEEP, P.KEEP])
    assert r["host_busy_ns"] == 0 and r["host_end_ns"] == 0
    r2 = P.simulate(layers, P.Link(10**9, 10**9, 3), BIG, 0, P.Loss(5, 0), [P.SWAP, P.RC_KEEP, P.KEEP])
    assert {k: v for k, v in r.items()} == {k: v for k, v in r2.items()}


def test_invariants():
    base = [P.Layer(100, 200, 90, 4096, 1024, 0, 0, 0, th, 512, 256) for th in (40, 300, 20, 500)]
    link = P.Link(10**9, 10**9, 5, 7 * 10**8, 6 * 10**8)
    loss = P.Loss(50, 0, 10, 64, 64)
    prev = None
    for scale in (0, 1, 4, 16):
        layers = [l._replace(th=l.th * scale) for l in base]
        r = P.simulate(layers, link, BIG, 0, loss, [P.KEEP] * 4)
        # the step cannot end before the host has done all its work after the first gradients land
        assert r["makespan_ns"] >= r["host_end_ns"] >= r["host_busy_ns"]
        assert r["host_busy_ns"] == sum(l.th for l in layers) + loss.th
        if prev is not None:
            assert r["makespan_ns"] >= prev          # a slower host never shortens the step
        prev = r["makespan_ns"]
    # merged blocks carry their members' host work
    m = P.merge_group(base[:3])
    assert (m.th, m.hg, m.hw) == (360, 1536, 768)


def test_a_host_bound_step_makes_swap_and_recompute_equally_good():
    """When the host optimiser outlasts everything else, the makespan is the host's and the planner falls
    back on its secondary keys (bytes moved, recompute time)."""
    layers = [P.Layer(100, 200, 90, 4096, 1024, 0, 0, 0, 10**5, 0, 0) for _ in range(5)]
    link = P.Link(10**9, 10**9, 0)
    full = sum(P.al(l.sav) + P.al(l.out) for l in layers)
    acts, s = P.plan(layers, link, full // 2 + 2048, 0, P.Loss(10, 0))
    assert s["makespan_ns"] == s["host_end_ns"] > s["busy_ns"]
    assert s["bytes_d2h"] == 0      # recompute moves nothing: preferred at equal makespan
