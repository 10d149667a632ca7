"""Planner oracle for the out-of-core training step (TEST INFRASTRUCTURE ONLY).

This file is the slow, plain reference for the planner half of the hot path.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import it; the product
library never does, and the two share no code.

What it follows (KARMA, SC20):
  * Sec. III-E "capacity-based strategy": keep the tail of the model resident, swap a
    block out right after its forward, prefetch in FIFO order of need for as long as
    memory allows.
  * Sec. III-F and the second optimisation problem (Eq. 10, constraint 10.1): a block
    is recomputed instead of swapped when recomputing up to the next checkpoint is
    cheaper than the swap-in it replaces; the goal of recompute is makespan, not memory.
  * Constraint 9.4: device memory in use never exceeds the capacity, at any instant.
  * Eq. 1: occupancy = busy / (busy + idle) of the compute queue.
  * Algorithm 1 and the worked six-block schedule of Sec. III-F.3: the plan is printed
    as stages `F`, `B`, `S^in`, `S^out` joined by "->" with "||" for overlap.

The paper hands its two integer programs to a proprietary stochastic solver; a result
of that solver cannot be reproduced.  The deterministic procedure below stands in for
it.  All arithmetic is on Python integers (nanoseconds and bytes).

Model of one step (a "block" of the paper is one layer record here):
  three in-order queues (compute, device-to-host, host-to-device) and one arena of
  `budget - fixed` bytes managed by a two-ended first-fit allocator.  Long-lived
  buffers (layer inputs x_i, saved internals s_i) are carved from the lowest fitting
  free range, short-lived ones (workspace, activation gradients dx_i) from the highest.

Host optimiser (Sec. III-G, stages 3 and 5: a block's gradients are swapped out after its
backward and the weights are updated on the CPU): a fourth in-order queue.  The gradients
of layer i leave on the device-to-host queue when B_i ends (gb bytes for streamed weights,
hg bytes for resident ones); the update of layer i starts when they have landed and the
host is free, and takes th_i; updates run in the order the backward ops complete.  New weights of
a resident layer (hw bytes) go back on the host-to-device queue behind every copy of the
step's own program (the program is enqueued ahead of time, the weight copies as updates
finish).  The makespan ends with the last update and the last weight copy: one step in
isolation.  (An executor may hide that tail under the next step's forward pass; the model
does not count on it.)  Copies issued after the forward pass are priced at the link's loaded
rates.

Connections between non-consecutive layers (Sec. III-F.3: residual networks, fully
convolutional networks with connections from the contracting to the expansive path): a
skip (src, dst), dst >= src + 2, says that the output of layer src, which is the input x_s
of layer s = src + 1, is read again by layer dst, in its forward and in its backward pass.
x_s follows the action of layer s.  Kept, or kept as a recompute checkpoint, it is simply
still there.  Swapped out after F_s, it has to come back before F_dst: a premature
swap-in on the host-to-device queue during the forward pass (issued one layer ahead of
dst when it can be placed then), after which it stays until B_s (only the internals of s
are left to fetch for the backward pass).  A chained layer's input is dropped, so the
input of a layer that something else reads again cannot be RC_CHAIN.  In the backward pass
B_dst leaves a gradient with respect to x_s, which is held (high end) until B_s adds it
to its own.

Weight streaming (Sec. III-G: a swapped block carries its weights; stage 3 of the
pipeline swaps a block's gradients out after its backward while earlier blocks are
swapped in): a layer with wb > 0 keeps its weights on the host.  They are copied in
before F_i, one layer ahead of the compute queue.  With wres[i] = 1 they then stay until
B_i ends (the capacity-based choice for the tail of the model); with wres[i] = 0 they are
freed after F_i and copied in again before R_i / B_i, queued with the activation swap-ins
in order of need.  The gradients get a buffer when B_i starts and leave on the
device-to-host queue when it ends.
"""
from collections import deque, namedtuple

KEEP, SWAP, RC_KEEP, RC_SWAP, RC_CHAIN = 0, 1, 2, 3, 4
N_ACTIONS = 5
ALIGN = 256

# per-layer costs.  tf/tb: forward, backward time (ns).  trc: time to recompute the layer's internals
# alone, for a layer whose output need not be rebuilt because it still exists as the next layer's
# kept or swapped-in input (the last layer of a recomputed run); a layer inside a run must rebuild
# its output too and costs tf (Sec. III-F: a recomputed block re-runs its forward pass).  sav: bytes of
# internals backward needs besides the layer input.  out: bytes of the layer output
# (= the next layer's input).  ws: transient workspace bytes of any op of this layer.
# wb/gb: bytes of the layer's weights / weight gradients when they are streamed over the
# host link instead of living in the fixed region (0 = resident).
# th: time (ns) the host optimiser needs for the layer's parameters (Sec. III-G, stage 5: the
# weights are updated on the CPU); hg / hw: for a layer whose weights are resident, the bytes of
# gradients that leave for the host after its backward and of new weights that come back after
# the update (a streamed layer's gradients are gb, its new weights stay on the host).
Layer = namedtuple("Layer", "tf tb trc sav out ws wb gb th hg hw", defaults=(0, 0, 0, 0, 0))
# host link: bytes/s per direction and a fixed per-copy latency (ns).  The *_loaded rates hold
# while gradients stream to the host and the host optimiser runs (every copy issued after the
# forward pass of a step with host updates); 0 = same as the idle rate.
Link = namedtuple("Link", "bw_h2d bw_d2h lat_ns bw_h2d_loaded bw_d2h_loaded", defaults=(0, 0))
# loss op that sits between forward and backward: time and workspace; th / hg / hw as for a
# layer (the parameters that belong to the loss record, e.g. a final normalisation)
Loss = namedtuple("Loss", "t ws th hg hw", defaults=(0, 0, 0))
Op = namedtuple("Op", "kind layer start end offs")   # kind in F B R L OUT IN WIN GOUT HOLD


class Infeasible(Exception):
    """The arena could not grant an allocation.  `progress` = compute ops (F, L, R, B) completed before that."""

    def __init__(self, progress=0):
        super().__init__(progress)
        self.progress = progress


def al(b):
    return (b + ALIGN - 1) // ALIGN * ALIGN


def copy_ns(b, bw, lat):
    """Time of one copy: latency plus bytes over bandwidth, rounded up (Eq. 4 reading:
    one measured throughput per direction)."""
    if b == 0:
        return 0
    return lat + (b * 10**9 + bw - 1) // bw


class Arena:
    """Two-ended first-fit allocator over [0, cap) with coalescing free list."""

    def __init__(self, cap):
        self.cap = cap
        self.free = [[0, cap]] if cap > 0 else []   # sorted [offset, size]
        self.used = 0
        self.peak_used = 0
        self.peak_extent_lo = 0     # highest end of a low-end allocation
        self.low_water_hi = cap     # lowest start of a high-end allocation

    def total_free(self):
        return self.cap - self.used

    def alloc(self, size, low):
        """Returns offset, or None when no free range fits.  size is already aligned
        and > 0."""
        fl = self.free
        rng = range(len(fl)) if low else range(len(fl) - 1, -1, -1)
        for k in rng:
            off, sz = fl[k]
            if sz >= size:
                if low:
                    res = off
                    if sz == size:
                        del fl[k]
                    else:
                        fl[k][0] = off + size
                        fl[k][1] = sz - size
                    self.peak_extent_lo = max(self.peak_extent_lo, res + size)
                else:
                    res = off + sz - size
                    if sz == size:
                        del fl[k]
                    else:
                        fl[k][1] = sz - size
                    self.low_water_hi = min(self.low_water_hi, res)
                self.used += size
                if self.used > self.peak_used:
                    self.peak_used = self.used
                return res
        return None

    def release(self, off, size):
        fl = self.free
        k = 0
        while k < len(fl) and fl[k][0] < off:
            k += 1
        fl.insert(k, [off, size])
        if k + 1 < len(fl) and fl[k][0] + fl[k][1] == fl[k + 1][0]:
            fl[k][1] += fl[k + 1][1]
            del fl[k + 1]
        if k > 0 and fl[k - 1][0] + fl[k - 1][1] == fl[k][0]:
            fl[k - 1][1] += fl[k][1]
            del fl[k]
        self.used -= size


def valid_actions(actions, skips=()):
    prev = KEEP
    for i, a in enumerate(actions):
        if not 0 <= a < N_ACTIONS:
            return False
        if a == RC_CHAIN and (i == 0 or prev not in (RC_KEEP, RC_SWAP, RC_CHAIN)):
            return False
        prev = a
    for src, dst in skips:
        if src + 1 < len(actions) and actions[src + 1] == RC_CHAIN:
            return False        # the tensor another layer reads again would be dropped
    return True


def valid_skips(skips, L):
    return all(0 <= src and src + 2 <= dst < L for src, dst in skips)


def backward_units(actions):
    """Backward proceeds over units in descending layer order.  A unit is either one
    KEEP/SWAP layer, or a recompute segment: a head (RC_KEEP / RC_SWAP, the checkpoint)
    plus the RC_CHAIN layers that follow it (the set of blocks up to the next
    checkpoint, Eq. 10)."""
    units = []
    i = len(actions) - 1
    while i >= 0:
        h = i
        while actions[h] == RC_CHAIN:
            h -= 1
        units.append((h, i))
        i = h - 1
    return units


def simulate(layers, link, budget, fixed, loss, actions, want_ops=False, wres=None, skips=()):
    """Timeline of one training step under a given per-layer action vector (and, for
    layers with streamed weights, the per-layer choice `wres`; `skips`: connections
    (src, dst) between non-consecutive layers).

    Returns a dict with makespan_ns, stall_ns, busy_ns, peak_bytes, bytes_d2h,
    bytes_h2d (what the plan moves: swapped activations, streamed weights and their
    gradients; the gradients and weights of resident layers, the same under every plan,
    are not counted), recompute_ns, host_busy_ns, host_end_ns (and `ops` when asked).  Raises Infeasible when the arena
    cannot grant an allocation (constraint 9.4)."""
    L = len(layers)
    if len(actions) != L or not valid_skips(skips, L) or not valid_actions(actions, skips):
        raise ValueError("invalid action vector")
    cap = (budget - fixed) // ALIGN * ALIGN     # whole alignment units: offsets from either end stay aligned
    if cap <= 0:
        raise Infeasible()
    ar = Arena(cap)
    done = [0]                # compute ops completed
    # xb[i] = aligned bytes of x_i, the input of layer i; x_0 is the step input and
    # lives in the fixed region, x_L feeds the loss.
    xraw = [0] + [layers[i].out for i in range(L)]
    xb = [al(b) for b in xraw]
    sb = [al(l.sav) for l in layers]
    wsb = [al(l.ws) for l in layers]
    wB = [al(l.wb) for l in layers]       # streamed weights (0 = resident in `fixed`)
    gB = [al(l.gb) if l.wb else 0 for l in layers]
    if wres is None:
        wres = [0] * L
    if len(wres) != L:
        raise ValueError("invalid wres vector")
    X = [None] * (L + 1)      # offsets
    S = [None] * L
    DX = [None] * (L + 1)
    W = [None] * L
    G = [None] * L
    warr = [0] * L            # arrival time of the weights for the current phase
    pending = deque()         # (time, [(off, size), ...]) frees at D2H completion
    out_end = [0] * L         # end of layer i's swap-out: its swap-in cannot start earlier
    ops = []
    tc = td = th = 0
    busy = 0
    d2h = h2d = rc_ns = 0
    hosted = loss.th > 0 or any(l.th > 0 for l in layers)   # a step with host updates
    rate = {"h2d": link.bw_h2d, "d2h": link.bw_d2h}          # current price of a copy
    landed = []               # (time the gradients are on the host, th, hw) in landing order
    # connections between non-consecutive layers: readers[s] = the layers that read x_s again
    readers = {}
    for src, dst in skips:
        readers.setdefault(src + 1, set()).add(dst)
    early_at, early_need, early_arr = {}, {}, {}   # premature swap-ins: where issued, where needed, arrival
    extra = [0] * L           # bytes of skip gradients first allocated by B_j
    for s_, ds in sorted(readers.items()):
        first, last = min(ds), max(ds)
        extra[last] += xb[s_]
        if actions[s_] in (SWAP, RC_SWAP) and xraw[s_]:
            early_at.setdefault(first - 1 if first - 1 > s_ else first, []).append(s_)
            early_need.setdefault(first, []).append(s_)
    DSK = {}                  # offset of the gradient w.r.t. x_s left by its readers, until B_s

    def apply_pending(t):
        while pending and pending[0][0] <= t:
            for off, size in pending.popleft()[1]:
                ar.release(off, size)

    def grant(size, low, t):
        """Allocate, waiting on outstanding swap-outs if need be (a memory stall)."""
        if size == 0:
            return None, t
        while True:
            off = ar.alloc(size, low)
            if off is not None:
                return off, t
            if not pending:
                raise Infeasible(done[0])
            tm, bufs = pending.popleft()
            for o, s in bufs:
                ar.release(o, s)
            if tm > t:
                t = tm

    def rel(off, size):
        if off is not None:
            ar.release(off, size)

    def weight_in(i, t):
        """Copy of layer i's weights into W[i] (already allocated), on the H2D queue."""
        nonlocal th, h2d
        st = max(th, t)
        th = st + copy_ns(layers[i].wb, rate["h2d"], link.lat_ns)
        h2d += layers[i].wb
        warr[i] = th
        if want_ops:
            ops.append(Op("WIN", i, st, th, (W[i],)))

    def early_in(s_, t, must):
        """Premature swap-in of x_s for a forward reader; `must`: the reader is next, wait for memory."""
        nonlocal th, h2d
        if s_ in early_arr:
            return t
        if must:
            X[s_], t = grant(xb[s_], True, t)
        else:
            X[s_] = ar.alloc(xb[s_], True)
            if X[s_] is None:
                return t
        st = max(th, t, out_end[s_])
        th = st + copy_ns(xraw[s_], rate["h2d"], link.lat_ns)
        h2d += xraw[s_]
        early_arr[s_] = th
        if want_ops:
            ops.append(Op("IN", s_, st, th, (X[s_], None)))
        return t

    # ---------------- forward ----------------
    for i in range(L):
        t = tc
        apply_pending(t)
        for s_ in early_at.get(i, ()):
            t = early_in(s_, t, i in readers[s_])
        for s_ in early_need.get(i, ()):
            t = early_in(s_, t, True)
            t = max(t, early_arr[s_])
        if wB[i] and W[i] is None:      # not prefetched: fetched now, the layer waits
            W[i], t = grant(wB[i], bool(wres[i]), t)
            weight_in(i, t)
        X[i + 1], t = grant(xb[i + 1], True, t)
        S[i], t = grant(sb[i], True, t)
        w, t = grant(wsb[i], False, t)
        if wB[i]:
            t = max(t, warr[i])
        # the next layer's weights start their trip when this layer starts computing
        if i + 1 < L and wB[i + 1]:
            W[i + 1] = ar.alloc(wB[i + 1], bool(wres[i + 1]))
            if W[i + 1] is not None:
                weight_in(i + 1, t)
        end = t + layers[i].tf
        busy += layers[i].tf
        done[0] += 1
        if want_ops:
            ops.append(Op("F", i, t, end, (X[i + 1], S[i], w)))
        tc = end
        rel(w, wsb[i])
        if wB[i] and not wres[i]:
            rel(W[i], wB[i])
            W[i] = None
        a = actions[i]
        if a == SWAP or a == RC_SWAP:
            nbytes = xraw[i] + (layers[i].sav if a == SWAP else 0)
            bufs = []
            if X[i] is not None:
                bufs.append((X[i], xb[i]))
            if a == SWAP and S[i] is not None:
                bufs.append((S[i], sb[i]))
            if nbytes:
                st = max(td, end)
                td = st + copy_ns(nbytes, rate["d2h"], link.lat_ns)
                d2h += nbytes
                pending.append((td, bufs))
                out_end[i] = td
                if want_ops:
                    ops.append(Op("OUT", i, st, td, ()))
            if a == RC_SWAP:
                rel(S[i], sb[i])
        elif a == RC_KEEP:
            rel(S[i], sb[i])
        elif a == RC_CHAIN:
            rel(S[i], sb[i])
            rel(X[i], xb[i])

    # ---------------- prefetch queue and reserves ----------------
    # Items of the H2D queue during backward, in order of need: ("A", i) = the swapped
    # tensors of layer i, ("W", i) = the weights of a layer that did not keep them.
    units = backward_units(actions)
    items = deque()
    def in_bytes(i):
        """What the backward swap-in of layer i still has to bring (x_i is there already after a premature swap-in)."""
        x_part = 0 if i in early_arr else xraw[i]
        return x_part + (layers[i].sav if actions[i] == SWAP else 0)

    for h, e in units:
        if actions[h] in (SWAP, RC_SWAP) and in_bytes(h):
            items.append(("A", h))
        for j in range(h, e + 1):
            if wB[j] and not wres[j]:
                items.append(("W", j))
    arrive = {}

    def unit_need(h, e):
        if actions[h] in (KEEP, SWAP):
            return xb[h] + wsb[h] + gB[h] + extra[h]
        s = sum(sb[j] for j in range(h, e + 1)) + sum(xb[j + 1] for j in range(h, e))
        return s + max(xb[j] + wsb[j] + gB[j] + extra[j] for j in range(h, e + 1))

    needs = [unit_need(h, e) for h, e in units]
    res_after = [0] * len(units)
    for k in range(len(units) - 2, -1, -1):
        res_after[k] = max(res_after[k + 1], needs[k + 1])
    res_all = max(needs) if needs else 0
    loss_need = xb[L] + al(loss.ws)

    def item_need(it):
        kind, i = it
        if kind == "W":
            return wB[i]
        return (0 if i in early_arr else xb[i]) + (sb[i] if actions[i] == SWAP else 0)

    def place(it):
        """Try to allocate the buffers of a queued copy (low end); roll back on
        failure."""
        kind, i = it
        if kind == "W":
            off = ar.alloc(wB[i], True)
            if off is None:
                return False
            W[i] = off
            return True
        xo = so = None
        fetch_x = i not in early_arr
        if fetch_x and xb[i]:
            xo = ar.alloc(xb[i], True)
            if xo is None:
                return False
        if actions[i] == SWAP and sb[i]:
            so = ar.alloc(sb[i], True)
            if so is None:
                if xo is not None:
                    ar.release(xo, xb[i])
                return False
        if fetch_x:
            X[i] = xo
        if actions[i] == SWAP:
            S[i] = so
        return True

    def issue_in(it, t):
        nonlocal th, h2d
        kind, i = it
        if kind == "W":
            weight_in(i, t)
            arrive[it] = th
            return
        nbytes = in_bytes(i)
        st = max(th, t, out_end[i])
        th = st + copy_ns(nbytes, rate["h2d"], link.lat_ns)
        h2d += nbytes
        arrive[it] = th
        if want_ops:
            ops.append(Op("IN", i, st, th, (None if i in early_arr else X[i], S[i] if actions[i] == SWAP else None)))

    def admit(t, reserve):
        """Copy in ahead of need, in order of need, while the arena keeps `reserve`
        bytes for the compute ops still to come (Sec. III-E: keep swapping in as long
        as there is space)."""
        apply_pending(t)
        while items:
            it = items[0]
            if ar.total_free() < item_need(it) + reserve or not place(it):
                break
            items.popleft()
            issue_in(it, t)

    def force(it, t):
        """This item is needed now: admit everything up to and including it."""
        while it not in arrive:
            jt = items.popleft()
            kind, j = jt
            if kind == "W":
                W[j], t = grant(wB[j], True, t)
            else:
                if j not in early_arr:
                    X[j], t = grant(xb[j], True, t)
                if actions[j] == SWAP:
                    S[j], t = grant(sb[j], True, t)
            issue_in(jt, t)
        return t

    def wait_for(it, t):
        if it in arrive or it in items:
            t = force(it, t)
            t = max(t, arrive[it])
        return t

    def grads_leave(rec, end, streamed_landing):
        """Gradients of a record go to the host after the op that completed them (at `end`);
        its update is queued for when they have landed."""
        nonlocal td
        if streamed_landing is not None:
            if rec.th:
                landed.append((streamed_landing, rec.th, 0))
            return
        when = end
        if rec.hg:
            st = max(td, end)
            td = st + copy_ns(rec.hg, rate["d2h"], link.lat_ns)
            when = td
        if rec.th or rec.hw:
            landed.append((when, rec.th, rec.hw))

    # ---------------- loss ----------------
    if hosted:
        # the forward pass is over: from here on gradients stream to the host and the optimiser
        # works on them, and every copy issued is priced at the loaded rates
        rate["h2d"] = link.bw_h2d_loaded or link.bw_h2d
        rate["d2h"] = link.bw_d2h_loaded or link.bw_d2h
    admit(tc, max(res_all, loss_need))
    t = tc
    apply_pending(t)
    DX[L], t = grant(xb[L], False, t)
    w, t = grant(al(loss.ws), False, t)
    end = t + loss.t
    busy += loss.t
    done[0] += 1
    if want_ops:
        ops.append(Op("L", L, t, end, (DX[L], w)))
    tc = end
    rel(w, al(loss.ws))
    rel(X[L], xb[L])
    grads_leave(loss, end, None)
    admit(tc, res_all)

    # ---------------- backward ----------------
    def backward_op(j, t, reserve):
        nonlocal tc, td, busy, d2h
        apply_pending(t)
        DX[j], t = grant(xb[j], False, t)
        w, t = grant(wsb[j], False, t)
        G[j], t = grant(gB[j], False, t)
        for s_ in sorted(readers):          # gradients this layer leaves for the inputs it read again
            if j in readers[s_] and s_ not in DSK:
                DSK[s_], t = grant(xb[s_], False, t)
                if want_ops:                # where the executor finds that buffer
                    ops.append(Op("HOLD", s_, t, t, (DSK[s_],)))
        end = t + layers[j].tb
        busy += layers[j].tb
        done[0] += 1
        if want_ops:
            ops.append(Op("B", j, t, end, (DX[j], w, G[j])))
        tc = end
        rel(w, wsb[j])
        rel(DX[j + 1], xb[j + 1])
        rel(S[j], sb[j])
        rel(X[j], xb[j])
        if j in DSK:                        # added to dx_j by this backward
            rel(DSK.pop(j), xb[j])
        if wB[j]:
            rel(W[j], wB[j])
            W[j] = None
        if gB[j]:
            # the gradients leave right after the layer's backward (pipeline stage 3)
            st = max(td, end)
            td = st + copy_ns(layers[j].gb, rate["d2h"], link.lat_ns)
            d2h += layers[j].gb
            pending.append((td, [(G[j], gB[j])]))
            if want_ops:
                ops.append(Op("GOUT", j, st, td, ()))
            grads_leave(layers[j], end, td)
        else:
            grads_leave(layers[j], end, None)
        admit(tc, reserve)

    for k, (h, e) in enumerate(units):
        a = actions[h]
        t = tc
        if a in (SWAP, RC_SWAP):
            t = wait_for(("A", h), t)
        if a in (KEEP, SWAP):
            t = wait_for(("W", h), t)
            backward_op(h, t, res_after[k])
            continue
        inner = max(xb[j] + wsb[j] + gB[j] + extra[j] for j in range(h, e + 1))
        for j in range(h, e + 1):
            t = wait_for(("W", j), t)
            apply_pending(t)
            S[j], t = grant(sb[j], True, t)
            if j < e:
                X[j + 1], t = grant(xb[j + 1], True, t)
            w, t = grant(wsb[j], False, t)
            redo = layers[j].tf if j < e else layers[j].trc
            end = t + redo
            busy += redo
            done[0] += 1
            rc_ns += redo
            if want_ops:
                ops.append(Op("R", j, t, end, (S[j], X[j + 1] if j < e else None, w)))
            tc = end
            rel(w, wsb[j])
            t = end
        for j in range(e, h - 1, -1):
            backward_op(j, tc, res_after[k] if j == h else max(res_after[k], inner))

    apply_pending(max(tc, td, th))
    assert ar.used == 0, "ledger leak"
    # ---------------- host optimiser queue ----------------
    t_host = host_busy = 0
    for when, t_upd, back in landed:
        t_host = max(t_host, when) + t_upd
        host_busy += t_upd
        if back:    # new weights of a resident layer: behind the program's own copies
            th = max(th, t_host) + copy_ns(back, rate["h2d"], link.lat_ns)
    makespan = max(tc, td, th, t_host)
    res = dict(makespan_ns=makespan, stall_ns=tc - busy, busy_ns=busy,
               peak_bytes=fixed + ar.peak_used, bytes_d2h=d2h, bytes_h2d=h2d,
               recompute_ns=rc_ns, host_busy_ns=host_busy, host_end_ns=t_host)
    if want_ops:
        res["ops"] = ops
    return res


def occupancy(summary):
    """Eq. 1 on the compute queue of the whole step."""
    return summary["busy_ns"] / (summary["busy_ns"] + summary["stall_ns"])


def cost_tuple(summary):
    return (summary["makespan_ns"], summary["bytes_d2h"] + summary["bytes_h2d"],
            summary["recompute_ns"])


def try_cost(layers, link, budget, fixed, loss, actions, wres=None, skips=()):
    if not valid_actions(actions, skips):
        return None
    try:
        return cost_tuple(simulate(layers, link, budget, fixed, loss, actions, wres=wres, skips=skips))
    except Infeasible:
        return None


def plan(layers, link, budget, fixed, loss, skips=()):
    """Deterministic stand-in for the paper's two-tier optimisation (`skips`: connections
    between non-consecutive layers, priced by the simulator and respected by every candidate).

    1. Capacity rule (Sec. III-E): everything fits -> all KEEP (streamed weights stay
       from F_i to B_i).  Otherwise the resident tail is as long as memory allows, the
       prefix before it is swapped.
    2. Recompute marking (Eq. 10.1, read with the prose above it): going down the
       prefix, a swapped layer becomes a recompute layer when its recompute time is
       strictly less than the swap-in it replaces.
    3. Makespan refinement (`refine`): local search on (makespan, bytes moved,
       recompute time), from two starts (swapped prefix after step 2; recomputed
       prefix); the better local optimum wins.
    4. Streamed weights (steps 1-3 run with every streamed layer fetching its weights
       twice): going down from the last layer, a layer keeps its weights between F_i and
       B_i as long as that fits and does not lengthen the step (the capacity-based rule
       applied to weights: the tail of the model stays); the first layer that cannot
       ends the scan.
    Returns (actions, summary) with summary["wres"] the per-layer weight choice; raises
    Infeasible when no assignment tried fits."""
    L = len(layers)
    streamed = [1 if l.wb else 0 for l in layers]
    cur = [KEEP] * L
    c = try_cost(layers, link, budget, fixed, loss, cur, streamed, skips)
    if c is not None:
        res = simulate(layers, link, budget, fixed, loss, cur, wres=streamed, skips=skips)
        res["wres"] = streamed
        return cur, res

    # step 1: longest resident tail; the prefix before it swapped, or (second start)
    # recomputed from kept checkpoints; patterns that hold less memory as fall-backs.
    reread = {src + 1 for src, _ in skips}     # inputs that a later layer reads again: never dropped

    def longest_tail(fill, at_reread=None):
        """Longest resident tail whose prefix takes `fill`; the prefix's read-again inputs (and, for
        chains, layer 0) take `at_reread` when given."""
        for k in range(1, L + 1):
            cand = [fill] * k + [KEEP] * (L - k)
            if at_reread is not None:
                for i in range(k):
                    if i in reread or (i == 0 and fill == RC_CHAIN):
                        cand[i] = at_reread
            if try_cost(layers, link, budget, fixed, loss, cand, None, skips) is not None:
                return cand
        return None

    starts = [s for s in (longest_tail(SWAP), longest_tail(RC_KEEP)) if s is not None]
    if not starts or skips:
        # chains from as few checkpoints as the connections allow; with connections also a swapped
        # prefix whose read-again tensors stay, as checkpoints or whole
        more = [longest_tail(RC_CHAIN, RC_KEEP) or longest_tail(RC_CHAIN, RC_SWAP)]
        if skips:
            more += [longest_tail(SWAP, RC_KEEP), longest_tail(SWAP, KEEP)]
        for s in more:
            if s is not None and s not in starts:
                starts.append(s)
    if not starts:
        # none of the patterns fits: the search starts from one that does not (its feasibility phase)
        starts = [[RC_SWAP if i == 0 or i in reread else RC_CHAIN for i in range(L)]]

    # step 2: Eq. 10.1 scan over the swapped prefix of the first start, descending
    xraw = [0] + [l.out for l in layers]
    hosted = loss.th > 0 or any(l.th > 0 for l in layers)
    bw_in = (link.bw_h2d_loaded or link.bw_h2d) if hosted else link.bw_h2d   # swap-ins run in the backward phase
    cur = starts[0]
    unmarked = list(cur)
    for i in range(L - 1, -1, -1):
        if cur[i] != SWAP:
            continue
        t_in = copy_ns(xraw[i] + layers[i].sav, bw_in, link.lat_ns)
        if layers[i].trc < t_in:
            for a in (RC_KEEP, RC_SWAP):
                cand = list(cur)
                cand[i] = a
                if try_cost(layers, link, budget, fixed, loss, cand, None, skips) is not None:
                    cur = cand
                    break
    starts[0] = cur
    if cur != unmarked:
        starts.append(unmarked)     # the capacity-based schedule itself (Fig. 2(b)) is a start too

    # step 3: refinement of each start; the best local optimum wins
    best = None
    for start in starts:
        key = refine(layers, link, budget, fixed, loss, start, skips)
        if best is None or key < best:
            best = key
    (unfit, cost), cur = best
    if unfit:
        raise Infeasible()

    # step 4: the tail keeps its streamed weights
    wres = [0] * L
    for i in range(L - 1, -1, -1):
        if not streamed[i]:
            continue
        cand = list(wres)
        cand[i] = 1
        cc = try_cost(layers, link, budget, fixed, loss, cur, cand, skips)
        if cc is None or not cc < cost:
            break
        wres, cost = cand, cc
    res = simulate(layers, link, budget, fixed, loss, cur, wres=wres, skips=skips)
    res["wres"] = wres
    return cur, res


GROUP_SIZES = (1, 2, 3, 4, 6, 8)


def merge_group(members):
    """Cost record of consecutive layers planned as one block (Sec. III-E/F: the first tier of the
    optimisation groups layers into blocks; a block is swapped, kept or recomputed as a whole).  Times
    add up (recomputing the block re-runs every member's forward pass but the last one's output); the block's internals are its members' internals plus the boundaries between them; its
    output is the last member's; workspace is the largest; streamed weights and gradients add up."""
    return Layer(tf=sum(m.tf for m in members), tb=sum(m.tb for m in members),
                 trc=sum(m.tf for m in members[:-1]) + members[-1].trc,
                 sav=sum(m.sav for m in members) + sum(m.out for m in members[:-1]), out=members[-1].out,
                 ws=max(m.ws for m in members), wb=sum(m.wb for m in members), gb=sum(m.gb for m in members),
                 th=sum(m.th for m in members), hg=sum(m.hg for m in members), hw=sum(m.hw for m in members))


def expand_group_actions(group_actions, group_wres, sizes):
    """Per-layer actions of a block-level plan: a kept or swapped block keeps or swaps every member; a
    recomputed block keeps (or swaps) its first member's input as the checkpoint and recomputes the rest
    in a chain from it; a chained block is chained throughout."""
    acts, wres = [], []
    for a, w, n in zip(group_actions, group_wres, sizes):
        if a in (KEEP, SWAP, RC_CHAIN):
            acts += [a] * n
        else:
            acts += [a] + [RC_CHAIN] * (n - 1)
        wres += [w] * n
    return acts, wres


def group_skips(skips, sizes):
    """Connections of the merged stack: a connection survives at block level when its source is the
    last member of its block (the tensor is then that block's output) and its reader sits at least two
    blocks further on; the others lie inside a block or between neighbours and are priced only by the
    per-layer simulator."""
    first, a = [], 0
    for n in sizes:
        first.append(a)
        a += n
    def block_of(i):
        k = 0
        while k + 1 < len(first) and first[k + 1] <= i:
            k += 1
        return k
    out = set()
    for src, dst in skips:
        gs, gd = block_of(src), block_of(dst)
        if src == first[gs] + sizes[gs] - 1 and gd >= gs + 2:
            out.add((gs, gd))
    return tuple(sorted(out))


def plan_grouped(layers, link, budget, fixed, loss, max_group=8, skips=()):
    """The planner with the block granularity chosen as well: for each group size g in GROUP_SIZES up to
    max_group, consecutive layers are merged g at a time (the last block may be shorter), the merged stack
    is planned, the block-level plan is expanded to per-layer actions and priced by the per-layer
    simulator (which is what the executor follows; it sees every copy's latency and every allocation).
    The cheapest expansion wins, the smaller group size on ties; g = 1 is the plain planner, so the result
    is never worse than plan().  `skips` are per-layer connections between non-consecutive layers; every
    expansion is priced with all of them.  Returns (actions, summary, g)."""
    L = len(layers)
    best = None
    for g in GROUP_SIZES:
        if g > max_group or (g > 1 and g > L):
            continue
        sizes = [min(g, L - a) for a in range(0, L, g)]
        if g == 1:
            try:
                acts, res = plan(layers, link, budget, fixed, loss, skips)
            except Infeasible:
                continue
            wres = res["wres"]
        else:
            merged, a = [], 0
            for n in sizes:
                merged.append(merge_group(layers[a:a + n]))
                a += n
            try:
                gacts, gres = plan(merged, link, budget, fixed, loss, group_skips(skips, sizes))
            except Infeasible:
                continue
            acts, wres = expand_group_actions(gacts, gres["wres"], sizes)
            if not valid_actions(acts, skips):
                continue
        c = try_cost(layers, link, budget, fixed, loss, acts, wres, skips)
        if c is None:
            continue
        if best is None or c < best[0]:
            best = (c, acts, wres, g)
    if best is None:
        raise Infeasible()
    _, acts, wres, g = best
    res = simulate(layers, link, budget, fixed, loss, acts, wres=wres, skips=skips)
    res["wres"] = wres
    return acts, res, g


PAIR_WINDOW = 4


def refine(layers, link, budget, fixed, loss, start, skips=()):
    """Local search (variable neighbourhood descent).  A candidate replaces the incumbent
    when its (cost tuple, action vector) is lexicographically smaller.  Neighbourhoods:
    (a) one layer takes another action; (b) two layers exchange their actions; (c) two
    layers at most PAIR_WINDOW apart take any pair of actions; (d) three consecutive
    layers take any triple of actions.  A larger neighbourhood is searched only when a
    full pass over every smaller one has changed nothing; any improvement sends the
    search back to (a).  It ends when a pass over (d) changes nothing.

    Feasibility phase: an assignment that does not fit is measured by how many compute ops
    its timeline completes before an allocation fails.  While the incumbent does not fit, a
    candidate replaces it when it fits or gets strictly further; every assignment that fits
    is better than every one that does not.  Returns (((0, cost tuple) or (1, -ops
    completed)), actions)."""
    L = len(layers)

    def measure(acts):
        if not valid_actions(acts, skips):
            return None
        try:
            return (0, cost_tuple(simulate(layers, link, budget, fixed, loss, acts, skips=skips)))
        except Infeasible as e:
            return (1, -e.progress)

    key = (measure(start), list(start))

    def consider(cand):
        nonlocal key
        cc = measure(cand)
        if cc is None:
            return False
        if (cc, cand) < key if not key[0][0] else cc < key[0]:
            key = (cc, cand)
            return True
        return False

    def singles():
        changed = False
        for i in range(L):
            for a in range(N_ACTIONS):
                if a != key[1][i]:
                    cand = list(key[1])
                    cand[i] = a
                    changed |= consider(cand)
        return changed

    def exchanges():
        changed = False
        for i in range(L):
            for j in range(i + 1, L):
                if key[1][i] != key[1][j]:
                    cand = list(key[1])
                    cand[i], cand[j] = cand[j], cand[i]
                    changed |= consider(cand)
        return changed

    def pairs():
        changed = False
        for i in range(L - 1):
            for j in range(i + 1, min(L, i + 1 + PAIR_WINDOW)):
                for a in range(N_ACTIONS):
                    for b in range(N_ACTIONS):
                        if (a, b) != (key[1][i], key[1][j]):
                            cand = list(key[1])
                            cand[i], cand[j] = a, b
                            changed |= consider(cand)
        return changed

    def triples():
        changed = False
        for i in range(L - 2):
            for a in range(N_ACTIONS):
                for b in range(N_ACTIONS):
                    for c in range(N_ACTIONS):
                        if (a, b, c) != tuple(key[1][i:i + 3]):
                            cand = list(key[1])
                            cand[i:i + 3] = [a, b, c]
                            changed |= consider(cand)
        return changed

    def quads():
        changed = False
        for i in range(L - 3):
            for q in range(N_ACTIONS ** 4):
                abcd = [q // 125, q // 25 % 5, q // 5 % 5, q % 5]
                if abcd != key[1][i:i + 4]:
                    cand = list(key[1])
                    cand[i:i + 4] = abcd
                    changed |= consider(cand)
        return changed

    def kicks():
        """One layer is forced to another action and held there while single-layer changes of the
        others descend from that point; the end of the descent is the candidate."""
        nonlocal key
        for i in range(L):
            for a in range(N_ACTIONS):
                if a == key[1][i]:
                    continue
                cand = list(key[1])
                cand[i] = a
                m = measure(cand)
                if m is None:
                    continue
                local = (m, cand)
                moved = True
                while moved:
                    moved = False
                    for j in range(L):
                        if j == i:
                            continue
                        for b in range(N_ACTIONS):
                            if b != local[1][j]:
                                c2 = list(local[1])
                                c2[j] = b
                                m2 = measure(c2)
                                if m2 is not None and (m2, c2) < local:
                                    local = (m2, c2)
                                    moved = True
                if local < key:
                    key = local
                    return True
        return False

    hoods = (singles, exchanges, pairs, triples) + ((quads, kicks) if skips else ())
    k = 0
    while k < len(hoods):
        k = 0 if hoods[k]() else k + 1
    return key


def brute_force(layers, link, budget, fixed, loss, alphabet=(KEEP, SWAP, RC_KEEP, RC_SWAP, RC_CHAIN), wres=None,
                prefix=(), skips=()):
    """Exhaustive search over every valid assignment: smallest cost tuple, ties to the
    lexicographically smallest action vector.  Exponential; for small stacks only.
    `prefix` fixes the actions of the first layers (a caller may split the enumeration
    over processes by prefix and take the smallest result)."""
    L = len(layers)
    best = None
    cur = list(prefix) + [alphabet[0]] * (L - len(prefix))
    if not valid_actions(list(prefix)):
        return None

    def rec(i):
        nonlocal best
        if i == L:
            c = try_cost(layers, link, budget, fixed, loss, cur, wres, skips)
            if c is not None and (best is None or (c, cur) < best):
                best = (c, list(cur))
            return
        for a in alphabet:
            if a == RC_CHAIN and (i == 0 or cur[i - 1] not in (RC_KEEP, RC_SWAP, RC_CHAIN)):
                continue
            cur[i] = a
            rec(i + 1)

    rec(len(prefix))
    return best


def stage_string(ops):
    """Algorithm 1's output in the paper's notation.  One stage per forward, backward
    or recompute op (a recompute is printed as F, as in the worked example); a copy is
    listed on the stage that is running when the copy starts.  Recompute stages are
    inserted as fresh stages by Algorithm 1 and carry no copies: a copy that starts
    during one is listed on the next forward/backward stage.  Layers print 1-based."""
    stages = [o for o in ops if o.kind in "FBR"]
    copies = [o for o in ops if o.kind in ("IN", "OUT", "WIN", "GOUT")]
    att = [[] for _ in stages]
    for c in copies:
        idx = None
        for k, s in enumerate(stages):
            if s.kind != "R" and s.end > c.start:
                idx = k
                break
        if idx is None:
            idx = len(stages) - 1
        att[idx].append(c)
    parts = []
    for s, cs in zip(stages, att):
        txt = ("B" if s.kind == "B" else "F") + str(s.layer + 1)
        for c in cs:
            txt += "||%s%d^%s" % ({"WIN": "W", "GOUT": "G"}.get(c.kind, "S"), c.layer + 1,
                                  "in" if c.kind in ("IN", "WIN") else "out")
        parts.append(txt)
    return " -> ".join(parts)


# ---- comparison policies run through the same simulator (Fig. 2 a/b) ----
def policy_eager_swap(L):
    """vDNN-style: every layer is swapped out after its forward, the last one too."""
    return [SWAP] * L


def policy_checkpoint_every(L, stride):
    """Plain gradient checkpointing: a kept checkpoint every `stride` layers, the rest
    dropped and recomputed."""
    return [RC_KEEP if i % stride == 0 else RC_CHAIN for i in range(L)]
