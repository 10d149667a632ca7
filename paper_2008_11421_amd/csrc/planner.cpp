// Planner of the out-of-core training step: timeline simulator, assignment search and
// stage printing.  Pure host code (no HIP calls), integer arithmetic only.
//
// KARMA, Sec. III-E (capacity-based swapping: resident tail, swap-out right after the
// forward of a block, prefetch in order of need while memory allows), Sec. III-F and
// Eq. 10 / 10.1 (recompute instead of swap where that shortens the makespan),
// constraint 9.4 (memory in use never above capacity), Eq. 1 (occupancy), Algorithm 1
// (stage list).  The paper solves its two integer programs with a stochastic solver; a
// deterministic local search over the simulator takes its place here.
#include "planner.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <deque>
#include <string>

namespace karma {

static inline int64_t align_up(int64_t b) { return (b + 255) / 256 * 256; }

int64_t copy_ns(uint64_t bytes, uint64_t bw, int64_t lat) {
  if (bytes == 0) return 0;
  unsigned __int128 num = (unsigned __int128)bytes * 1000000000ull + (bw - 1);
  return lat + (int64_t)(num / bw);
}

// ---- two-ended first-fit allocator ------------------------------------------------
void Arena::reset(int64_t capacity) {
  cap = capacity;
  holes.clear();
  if (cap > 0) holes.push_back({0, cap});
  used = 0;
  peak = 0;
}

int64_t Arena::take(int64_t size, bool low) {
  if (low) {
    for (size_t k = 0; k < holes.size(); ++k) {
      if (holes[k].size >= size) {
        int64_t at = holes[k].off;
        if (holes[k].size == size) holes.erase(holes.begin() + k);
        else { holes[k].off += size; holes[k].size -= size; }
        used += size;
        peak = std::max(peak, used);
        return at;
      }
    }
  } else {
    for (size_t k = holes.size(); k-- > 0;) {
      if (holes[k].size >= size) {
        int64_t at = holes[k].off + holes[k].size - size;
        if (holes[k].size == size) holes.erase(holes.begin() + k);
        else holes[k].size -= size;
        used += size;
        peak = std::max(peak, used);
        return at;
      }
    }
  }
  return -1;
}

void Arena::give(int64_t off, int64_t size) {
  size_t k = 0;
  while (k < holes.size() && holes[k].off < off) ++k;
  holes.insert(holes.begin() + k, Hole{off, size});
  if (k + 1 < holes.size() && holes[k].off + holes[k].size == holes[k + 1].off) {
    holes[k].size += holes[k + 1].size;
    holes.erase(holes.begin() + k + 1);
  }
  if (k > 0 && holes[k - 1].off + holes[k - 1].size == holes[k].off) {
    holes[k - 1].size += holes[k].size;
    holes.erase(holes.begin() + k);
  }
  used -= size;
}

bool actions_valid(const uint8_t* a, uint32_t n, const karma_skip* skips, uint32_t n_skips) {
  uint8_t prev = KARMA_KEEP;
  for (uint32_t i = 0; i < n; ++i) {
    if (a[i] > KARMA_RC_CHAIN) return false;
    if (a[i] == KARMA_RC_CHAIN && (i == 0 || prev < KARMA_RC_KEEP)) return false;
    prev = a[i];
  }
  for (uint32_t k = 0; k < n_skips; ++k)
    if (skips[k].src + 1 < n && a[skips[k].src + 1] == KARMA_RC_CHAIN) return false;
  return true;
}

bool skips_valid(const karma_skip* skips, uint32_t n_skips, uint32_t n) {
  for (uint32_t k = 0; k < n_skips; ++k)
    if ((uint64_t)skips[k].src + 2 > skips[k].dst || skips[k].dst >= n) return false;
  return true;
}

// ---- timeline simulator -----------------------------------------------------------
namespace {

struct Timeline {
  const Problem& P;
  const uint8_t* act;
  const uint8_t* keepw;                           // per layer: streamed weights stay from F_i to B_i (null = none do)
  std::vector<karma_op>* ops;
  uint32_t L;
  Arena arena;
  std::vector<int64_t> x_raw, x_sz, s_sz, w_sz;   // bytes of x_i (raw / aligned), internals, workspace
  std::vector<int64_t> p_sz, g_sz;               // streamed weights and their gradients (0 = resident)
  std::vector<int64_t> x_at, s_at, dx_at;        // current offsets, -1 = not allocated
  std::vector<int64_t> p_at, g_at, p_here;       // weight / gradient buffers; arrival of the weights
  struct Pending { int64_t when; int64_t off[2], size[2]; int n; };
  std::deque<Pending> outgoing;                   // frees that happen when a device-to-host copy ends
  // copies still to prefetch during backward, in order of need: the swapped tensors of a
  // layer, or the weights of a layer that did not keep them
  struct Want { bool weights; uint32_t layer; };
  std::deque<Want> wanted;
  std::vector<int64_t> arrival, w_arrival;        // end of that copy, -1 = not issued
  std::vector<int64_t> left;                      // end of the swap-out of layer i
  int64_t t_comp = 0, t_out = 0, t_in = 0, busy = 0, redo = 0;
  uint64_t moved_out = 0, moved_in = 0;
  bool failed = false;
  // host optimiser queue (Sec. III-G, stages 3 and 5): updates in the order of the backward ops
  struct Update { int64_t landed, t_ns; uint64_t back_bytes; };
  std::vector<Update> updates;
  bool hosted = false;                            // a step with host updates
  uint64_t bw_in = 0, bw_out = 0;                 // current price of a copy (idle rates, then loaded ones)
  int64_t done = 0;                               // compute ops completed (how far a timeline that does not fit got)
  // Connections between non-consecutive layers (Sec. III-F.3).  x_s is "read again" when a layer
  // other than s reads it.  reads[j]: the inputs layer j reads again, ascending.  A swapped x_s
  // comes back ahead of its first reader (a premature swap-in) and then stays until B_s;
  // the gradient its readers leave for it waits in hold_at[s] until B_s adds it in.
  std::vector<std::vector<uint32_t>> reads, early_try, early_due;
  std::vector<int64_t> back_early;                // end of the premature swap-in of x_s, -1 = none
  std::vector<int64_t> hold_at, hold_first;       // offset of that gradient; bytes B_j is the first to hold

  Timeline(const Problem& p, const uint8_t* a, const uint8_t* kw, std::vector<karma_op>* o)
      : P(p), act(a), keepw(kw), ops(o), L(p.n) {}
  bool keeps(uint32_t i) const { return keepw && keepw[i]; }

  void emit(uint8_t kind, uint32_t layer, int64_t s, int64_t e, int64_t a0, int64_t a1, int64_t a2) {
    if (ops) ops->push_back(karma_op{kind, layer, s, e, {a0, a1, a2}});
  }
  void settle(int64_t now) {
    while (!outgoing.empty() && outgoing.front().when <= now) {
      const Pending& p = outgoing.front();
      for (int k = 0; k < p.n; ++k) arena.give(p.off[k], p.size[k]);
      outgoing.pop_front();
    }
  }
  // allocate; when the arena is full wait for the next swap-out to finish
  int64_t obtain(int64_t size, bool low, int64_t& now) {
    if (size == 0 || failed) return -1;
    for (;;) {
      int64_t at = arena.take(size, low);
      if (at >= 0) return at;
      if (outgoing.empty()) { failed = true; return -1; }
      const Pending& p = outgoing.front();
      for (int k = 0; k < p.n; ++k) arena.give(p.off[k], p.size[k]);
      now = std::max(now, p.when);
      outgoing.pop_front();
    }
  }
  void drop(int64_t& at, int64_t size) {
    if (at >= 0) { arena.give(at, size); at = -1; }
  }
  bool swapped_whole(uint32_t i) const { return act[i] == KARMA_SWAP; }
  int64_t move_bytes(uint32_t i) const { return x_raw[i] + (swapped_whole(i) ? (int64_t)P.layers[i].sav_bytes : 0); }
  bool here_already(uint32_t i) const { return back_early[i] >= 0; }
  // what the backward swap-in of layer i still has to bring
  int64_t fetch_bytes(uint32_t i) const {
    return (here_already(i) ? 0 : x_raw[i]) + (swapped_whole(i) ? (int64_t)P.layers[i].sav_bytes : 0);
  }
  // premature swap-in of x_s for a forward reader; `must`: the reader is next, wait for memory
  void fetch_early(uint32_t s, int64_t& now, bool must) {
    if (here_already(s) || failed) return;
    if (must) {
      x_at[s] = obtain(x_sz[s], true, now);
      if (failed) return;
    } else {
      x_at[s] = arena.take(x_sz[s], true);
      if (x_at[s] < 0) return;
    }
    int64_t st = std::max(std::max(t_in, now), left[s]);
    t_in = st + copy_ns((uint64_t)x_raw[s], bw_in, P.link.lat_ns);
    moved_in += (uint64_t)x_raw[s];
    back_early[s] = t_in;
    emit('I', s, st, t_in, x_at[s], -1, -1);
  }

  // copy of layer i's weights into p_at[i] (already allocated)
  void fetch_weights(uint32_t i, int64_t now) {
    int64_t s = std::max(t_in, now);
    t_in = s + copy_ns(P.layers[i].w_bytes, bw_in, P.link.lat_ns);
    moved_in += P.layers[i].w_bytes;
    p_here[i] = t_in;
    emit('W', i, s, t_in, p_at[i], -1, -1);
  }
  void start_prefetch(const Want& it, int64_t now) {
    const uint32_t i = it.layer;
    if (it.weights) {
      fetch_weights(i, now);
      w_arrival[i] = t_in;
      return;
    }
    int64_t nbytes = fetch_bytes(i);
    int64_t s = std::max(std::max(t_in, now), left[i]);   // data must have reached the host first
    t_in = s + copy_ns((uint64_t)nbytes, bw_in, P.link.lat_ns);
    moved_in += (uint64_t)nbytes;
    arrival[i] = t_in;
    emit('I', i, s, t_in, here_already(i) ? -1 : x_at[i], swapped_whole(i) ? s_at[i] : -1, -1);
  }
  void prefetch_ahead(int64_t now, int64_t reserve) {
    settle(now);
    while (!wanted.empty()) {
      const Want it = wanted.front();
      const uint32_t i = it.layer;
      int64_t need = it.weights ? p_sz[i] : (here_already(i) ? 0 : x_sz[i]) + (swapped_whole(i) ? s_sz[i] : 0);
      if (arena.cap - arena.used < need + reserve) break;
      if (it.weights) {
        int64_t pa = arena.take(p_sz[i], true);
        if (pa < 0) break;
        p_at[i] = pa;
      } else {
        int64_t xa = -1, sa = -1;
        const bool fetch_x = !here_already(i);
        if (fetch_x && x_sz[i]) { xa = arena.take(x_sz[i], true); if (xa < 0) break; }
        if (swapped_whole(i) && s_sz[i]) {
          sa = arena.take(s_sz[i], true);
          if (sa < 0) { if (xa >= 0) arena.give(xa, x_sz[i]); break; }
        }
        if (fetch_x) x_at[i] = xa;
        if (swapped_whole(i)) s_at[i] = sa;
      }
      wanted.pop_front();
      start_prefetch(it, now);
    }
  }
  // the copy `it` is needed now: admit everything up to and including it, then wait for it
  int64_t need_now(const Want& it, int64_t now) {
    std::vector<int64_t>& arr = it.weights ? w_arrival : arrival;
    bool queued = false;
    for (const Want& q : wanted) queued |= (q.weights == it.weights && q.layer == it.layer);
    if (arr[it.layer] < 0 && !queued) return now;
    while (arr[it.layer] < 0 && !failed) {
      const Want j = wanted.front();
      wanted.pop_front();
      if (j.weights) {
        p_at[j.layer] = obtain(p_sz[j.layer], true, now);
      } else {
        if (!here_already(j.layer)) x_at[j.layer] = obtain(x_sz[j.layer], true, now);
        if (swapped_whole(j.layer)) s_at[j.layer] = obtain(s_sz[j.layer], true, now);
      }
      if (!failed) start_prefetch(j, now);
    }
    if (failed) return now;
    return std::max(now, arr[it.layer]);
  }
  // gradients of a record with resident weights go to the host after the op that completed them; its
  // update is queued for when they have landed
  void grads_leave(int64_t t_ns, uint64_t out_bytes, uint64_t back_bytes, int64_t end) {
    int64_t when = end;
    if (out_bytes) {
      int64_t s = std::max(t_out, end);
      t_out = s + copy_ns(out_bytes, bw_out, P.link.lat_ns);   // (the same under every plan: not counted as moved)
      when = t_out;
    }
    if (t_ns || back_bytes) updates.push_back(Update{when, t_ns, back_bytes});
  }
  void backward(uint32_t j, int64_t now, int64_t reserve) {
    settle(now);
    dx_at[j] = obtain(x_sz[j], false, now);
    int64_t w = obtain(w_sz[j], false, now);
    g_at[j] = obtain(g_sz[j], false, now);
    for (uint32_t s : reads[j])           // gradients this layer leaves for the inputs it read again
      if (hold_at[s] < 0) {
        hold_at[s] = obtain(x_sz[s], false, now);
        if (!failed) emit('H', s, now, now, hold_at[s], -1, -1);   // where the executor finds that buffer
      }
    if (failed) return;
    int64_t end = now + P.layers[j].tb_ns;
    busy += P.layers[j].tb_ns;
    ++done;
    emit('B', j, now, end, dx_at[j], w, g_at[j]);
    t_comp = end;
    drop(w, w_sz[j]);
    drop(dx_at[j + 1], x_sz[j + 1]);
    drop(s_at[j], s_sz[j]);
    drop(x_at[j], x_sz[j]);
    drop(hold_at[j], x_sz[j]);            // added to dx_j by this backward
    if (p_sz[j]) drop(p_at[j], p_sz[j]);
    if (g_sz[j]) {
      // the gradients leave right after the layer's backward (pipeline stage 3)
      int64_t s = std::max(t_out, end);
      t_out = s + copy_ns(P.layers[j].g_bytes, bw_out, P.link.lat_ns);
      moved_out += P.layers[j].g_bytes;
      outgoing.push_back(Pending{t_out, {g_at[j], 0}, {g_sz[j], 0}, 1});
      g_at[j] = -1;
      emit('G', j, s, t_out, -1, -1, -1);
      if (P.layers[j].th_ns) updates.push_back(Update{t_out, P.layers[j].th_ns, 0});
    } else {
      grads_leave(P.layers[j].th_ns, P.layers[j].hg_bytes, P.layers[j].hw_bytes, end);
    }
    prefetch_ahead(t_comp, reserve);
  }

  bool run(karma_plan_summary* out) {
    // whole alignment units: buffers carved from the high end then start on 256-byte boundaries too, so that
    // which kernel a shape takes (some need 16-byte aligned operands) never depends on the budget
    int64_t cap = ((int64_t)P.budget - (int64_t)P.fixed) / 256 * 256;
    if (cap <= 0) return false;
    arena.reset(cap);
    hosted = P.loss.th_ns > 0;
    for (uint32_t i = 0; i < L; ++i) hosted |= P.layers[i].th_ns > 0;
    bw_in = P.link.bw_h2d;
    bw_out = P.link.bw_d2h;
    x_raw.assign(L + 1, 0); x_sz.assign(L + 1, 0); s_sz.assign(L, 0); w_sz.assign(L, 0);
    p_sz.assign(L, 0); g_sz.assign(L, 0);
    for (uint32_t i = 0; i < L; ++i) {
      x_raw[i + 1] = (int64_t)P.layers[i].out_bytes;
      x_sz[i + 1] = align_up(x_raw[i + 1]);
      s_sz[i] = align_up((int64_t)P.layers[i].sav_bytes);
      w_sz[i] = align_up((int64_t)P.layers[i].ws_bytes);
      p_sz[i] = align_up((int64_t)P.layers[i].w_bytes);
      g_sz[i] = P.layers[i].w_bytes ? align_up((int64_t)P.layers[i].g_bytes) : 0;
    }
    x_at.assign(L + 1, -1); s_at.assign(L, -1); dx_at.assign(L + 2, -1);
    p_at.assign(L, -1); g_at.assign(L, -1); p_here.assign(L, 0);
    x_sz.push_back(0);  // x_sz[L+1] so that backward(L-1...) can index j+1 == L safely
    arrival.assign(L, -1);
    w_arrival.assign(L, -1);
    left.assign(L, 0);
    reads.assign(L, {}); early_try.assign(L, {}); early_due.assign(L, {});
    back_early.assign(L, -1); hold_at.assign(L + 1, -1); hold_first.assign(L, 0);
    if (P.n_skips) {
      std::vector<int64_t> first(L, -1), last(L, -1);
      for (uint32_t k = 0; k < P.n_skips; ++k) {
        const uint32_t s = P.skips[k].src + 1, d = P.skips[k].dst;
        reads[d].push_back(s);
        first[s] = first[s] < 0 ? (int64_t)d : std::min(first[s], (int64_t)d);
        last[s] = std::max(last[s], (int64_t)d);
      }
      for (uint32_t j = 0; j < L; ++j) {
        std::sort(reads[j].begin(), reads[j].end());
        reads[j].erase(std::unique(reads[j].begin(), reads[j].end()), reads[j].end());
      }
      for (uint32_t s = 0; s < L; ++s) {
        if (first[s] < 0) continue;
        hold_first[last[s]] += x_sz[s];
        if ((act[s] == KARMA_SWAP || act[s] == KARMA_RC_SWAP) && x_raw[s]) {
          // queued one layer ahead of the first reader when there is a layer between, else at the reader
          early_try[first[s] - 1 > (int64_t)s ? first[s] - 1 : first[s]].push_back(s);
          early_due[first[s]].push_back(s);
        }
      }
    }

    // forward
    for (uint32_t i = 0; i < L && !failed; ++i) {
      int64_t now = t_comp;
      settle(now);
      for (uint32_t s : early_try[i]) fetch_early(s, now, std::binary_search(reads[i].begin(), reads[i].end(), s));
      for (uint32_t s : early_due[i]) {
        fetch_early(s, now, true);
        if (failed) break;
        now = std::max(now, back_early[s]);
      }
      if (failed) break;
      if (p_sz[i] && p_at[i] < 0) {   // not prefetched: fetched now, the layer waits
        p_at[i] = obtain(p_sz[i], keeps(i), now);
        if (failed) break;
        fetch_weights(i, now);
      }
      x_at[i + 1] = obtain(x_sz[i + 1], true, now);
      s_at[i] = obtain(s_sz[i], true, now);
      int64_t w = obtain(w_sz[i], false, now);
      if (failed) break;
      if (p_sz[i]) now = std::max(now, p_here[i]);
      // the next layer's weights start their trip when this layer starts computing
      if (i + 1 < L && p_sz[i + 1]) {
        p_at[i + 1] = arena.take(p_sz[i + 1], keeps(i + 1));
        if (p_at[i + 1] >= 0) fetch_weights(i + 1, now);
      }
      int64_t end = now + P.layers[i].tf_ns;
      busy += P.layers[i].tf_ns;
      ++done;
      emit('F', i, now, end, x_at[i + 1], s_at[i], w);
      t_comp = end;
      drop(w, w_sz[i]);
      if (p_sz[i] && !keeps(i)) drop(p_at[i], p_sz[i]);
      switch (act[i]) {
        case KARMA_SWAP:
        case KARMA_RC_SWAP: {
          int64_t nbytes = move_bytes(i);
          Pending p{0, {0, 0}, {0, 0}, 0};
          if (x_at[i] >= 0) { p.off[p.n] = x_at[i]; p.size[p.n] = x_sz[i]; ++p.n; }
          if (act[i] == KARMA_SWAP && s_at[i] >= 0) { p.off[p.n] = s_at[i]; p.size[p.n] = s_sz[i]; ++p.n; }
          if (nbytes) {
            int64_t s = std::max(t_out, end);
            t_out = s + copy_ns((uint64_t)nbytes, bw_out, P.link.lat_ns);
            moved_out += (uint64_t)nbytes;
            p.when = t_out;
            left[i] = t_out;
            outgoing.push_back(p);
            emit('O', i, s, t_out, -1, -1, -1);
            x_at[i] = -1;
            if (act[i] == KARMA_SWAP) s_at[i] = -1;
          }
          if (act[i] == KARMA_RC_SWAP) drop(s_at[i], s_sz[i]);
          break;
        }
        case KARMA_RC_KEEP: drop(s_at[i], s_sz[i]); break;
        case KARMA_RC_CHAIN: drop(s_at[i], s_sz[i]); drop(x_at[i], x_sz[i]); break;
        default: break;
      }
    }
    if (failed) return false;

    // backward units: single KEEP/SWAP layers, or recompute segments head..tail
    struct Unit { uint32_t head, tail; int64_t need, inner; };
    std::vector<Unit> units;
    for (int64_t i = (int64_t)L - 1; i >= 0;) {
      int64_t h = i;
      while (act[h] == KARMA_RC_CHAIN) --h;
      Unit u{(uint32_t)h, (uint32_t)i, 0, 0};
      if (act[h] <= KARMA_SWAP) {
        u.need = x_sz[h] + w_sz[h] + g_sz[h] + hold_first[h];
      } else {
        int64_t held = 0, top = 0;
        for (int64_t j = h; j <= i; ++j) {
          held += s_sz[j];
          if (j < i) held += x_sz[j + 1];
          top = std::max(top, x_sz[j] + w_sz[j] + g_sz[j] + hold_first[j]);
        }
        u.need = held + top;
        u.inner = top;
      }
      units.push_back(u);
      i = h - 1;
    }
    std::vector<int64_t> after(units.size(), 0);
    for (size_t k = units.size(); k-- > 1;) after[k - 1] = std::max(after[k], units[k].need);
    int64_t any = 0;
    for (const Unit& u : units) any = std::max(any, u.need);
    for (const Unit& u : units) {
      const uint32_t h = u.head;
      if ((act[h] == KARMA_SWAP || act[h] == KARMA_RC_SWAP) && fetch_bytes(h) > 0) wanted.push_back(Want{false, h});
      for (uint32_t j = h; j <= u.tail; ++j)
        if (p_sz[j] && !keeps(j)) wanted.push_back(Want{true, j});
    }

    // loss
    int64_t lw_sz = align_up((int64_t)P.loss.ws_bytes);
    if (hosted) {
      // the forward pass is over: from here on gradients stream to the host and the optimiser works
      // on them, and every copy issued is priced at the loaded rates
      if (P.link.bw_h2d_loaded) bw_in = P.link.bw_h2d_loaded;
      if (P.link.bw_d2h_loaded) bw_out = P.link.bw_d2h_loaded;
    }
    prefetch_ahead(t_comp, std::max(any, x_sz[L] + lw_sz));
    {
      int64_t now = t_comp;
      settle(now);
      dx_at[L] = obtain(x_sz[L], false, now);
      int64_t w = obtain(lw_sz, false, now);
      if (failed) return false;
      int64_t end = now + P.loss.t_ns;
      busy += P.loss.t_ns;
      ++done;
      emit('L', L, now, end, dx_at[L], w, -1);
      t_comp = end;
      drop(w, lw_sz);
      drop(x_at[L], x_sz[L]);
      grads_leave(P.loss.th_ns, P.loss.hg_bytes, P.loss.hw_bytes, end);
      prefetch_ahead(t_comp, any);
    }

    for (size_t k = 0; k < units.size() && !failed; ++k) {
      const Unit& u = units[k];
      uint8_t a = act[u.head];
      int64_t now = t_comp;
      if (a == KARMA_SWAP || a == KARMA_RC_SWAP) {
        now = need_now(Want{false, u.head}, now);
        if (failed) break;
      }
      if (a <= KARMA_SWAP) {
        now = need_now(Want{true, u.head}, now);
        if (failed) break;
        backward(u.head, now, after[k]);
        continue;
      }
      for (uint32_t j = u.head; j <= u.tail && !failed; ++j) {
        now = need_now(Want{true, j}, now);
        if (failed) break;
        settle(now);
        s_at[j] = obtain(s_sz[j], true, now);
        if (j < u.tail) x_at[j + 1] = obtain(x_sz[j + 1], true, now);
        int64_t w = obtain(w_sz[j], false, now);
        if (failed) break;
        // inside a run the layer's output is rebuilt too (a forward pass); the run's last layer rebuilds its internals only
        const int64_t again = j < u.tail ? P.layers[j].tf_ns : P.layers[j].trc_ns;
        int64_t end = now + again;
        busy += again;
        redo += again;
        ++done;
        emit('R', j, now, end, s_at[j], j < u.tail ? x_at[j + 1] : -1, w);
        t_comp = end;
        drop(w, w_sz[j]);
        now = end;
      }
      for (int64_t j = u.tail; j >= (int64_t)u.head && !failed; --j)
        backward((uint32_t)j, t_comp, j == (int64_t)u.head ? after[k] : std::max(after[k], u.inner));
    }
    if (failed) return false;
    // host optimiser queue; new weights of resident layers go back behind the program's own copies
    int64_t t_host = 0, host_busy = 0;
    for (const Update& u : updates) {
      t_host = std::max(t_host, u.landed) + u.t_ns;
      host_busy += u.t_ns;
      if (u.back_bytes) {
        t_in = std::max(t_in, t_host) + copy_ns(u.back_bytes, bw_in, P.link.lat_ns);
      }
    }
    int64_t endall = std::max(std::max(t_comp, t_host), std::max(t_out, t_in));
    if (out) {
      out->makespan_ns = endall;
      out->stall_ns = t_comp - busy;
      out->busy_ns = busy;
      out->recompute_ns = redo;
      out->peak_bytes = P.fixed + (uint64_t)arena.peak;
      out->bytes_d2h = moved_out;
      out->bytes_h2d = moved_in;
      out->host_busy_ns = host_busy;
      out->host_end_ns = t_host;
    }
    return true;
  }
};

// What the search minimises.  An assignment that fits: (makespan, bytes moved, recompute time).  One
// that does not fit is worse than every one that does, and is measured by how many compute ops its
// timeline completes before an allocation fails (makespan holds minus that count).
struct Cost {
  int unfit; int64_t makespan; uint64_t moved; int64_t redo;
  bool operator<(const Cost& o) const {
    if (unfit != o.unfit) return unfit < o.unfit;
    if (makespan != o.makespan) return makespan < o.makespan;
    if (moved != o.moved) return moved < o.moved;
    return redo < o.redo;
  }
  bool operator==(const Cost& o) const {
    return unfit == o.unfit && makespan == o.makespan && moved == o.moved && redo == o.redo;
  }
};

// false: not a valid assignment
bool evaluate(const Problem& P, const std::vector<uint8_t>& a, Cost& c, const uint8_t* keepw = nullptr) {
  karma_plan_summary s;
  if (!actions_valid(a.data(), P.n, P.skips, P.n_skips)) return false;
  Timeline tl(P, a.data(), keepw, nullptr);
  if (tl.run(&s)) c = Cost{0, s.makespan_ns, s.bytes_d2h + s.bytes_h2d, s.recompute_ns};
  else c = Cost{1, -tl.done, 0, 0};
  return true;
}
bool fits(const Problem& P, const std::vector<uint8_t>& a, Cost& c, const uint8_t* keepw = nullptr) {
  return evaluate(P, a, c, keepw) && !c.unfit;
}

struct Incumbent {
  Cost cost; std::vector<uint8_t> act;
  bool after(const Cost& c, const std::vector<uint8_t>& a) const {   // (c, a) < (cost, act)
    if (c < cost) return true;
    if (!(c == cost)) return false;
    return a < act;   // lexicographic
  }
  // the search's acceptance rule: while the incumbent does not fit only strict progress counts
  bool beaten_by(const Cost& c, const std::vector<uint8_t>& a) const { return cost.unfit ? c < cost : after(c, a); }
};

// Local search (variable neighbourhood descent) on (cost, action vector).  Neighbourhoods: one
// layer takes another action; two layers exchange their actions; two layers at most PAIR_WINDOW
// apart take any pair of actions; three consecutive layers take any triple of actions.  A larger
// neighbourhood is searched only when a full pass over every smaller one changed nothing; any
// improvement sends the search back to the smallest.  With connections between non-consecutive
// layers two more follow: four consecutive layers take any four actions; and "kicks": one layer is
// forced to another action and held there while single-layer changes of the others descend from that
// point, the end of the descent being the candidate.
static const uint32_t PAIR_WINDOW = 4;

void improve(const Problem& P, Incumbent& inc) {
  const uint32_t L = P.n;
  std::vector<uint8_t> cand;
  auto attempt = [&]() {
    Cost c;
    if (evaluate(P, cand, c) && inc.beaten_by(c, cand)) { inc.cost = c; inc.act = cand; return true; }
    return false;
  };
  auto pass = [&](int hood) {
    bool moved = false;
    if (hood == 0) {
      for (uint32_t i = 0; i < L; ++i)
        for (uint8_t a = 0; a <= KARMA_RC_CHAIN; ++a)
          if (a != inc.act[i]) { cand = inc.act; cand[i] = a; moved |= attempt(); }
    } else if (hood == 1) {
      for (uint32_t i = 0; i < L; ++i)
        for (uint32_t j = i + 1; j < L; ++j)
          if (inc.act[i] != inc.act[j]) { cand = inc.act; std::swap(cand[i], cand[j]); moved |= attempt(); }
    } else if (hood == 2) {
      for (uint32_t i = 0; i + 1 < L; ++i)
        for (uint32_t j = i + 1; j < L && j <= i + PAIR_WINDOW; ++j)
          for (uint8_t a = 0; a <= KARMA_RC_CHAIN; ++a)
            for (uint8_t b = 0; b <= KARMA_RC_CHAIN; ++b)
              if (a != inc.act[i] || b != inc.act[j]) { cand = inc.act; cand[i] = a; cand[j] = b; moved |= attempt(); }
    } else if (hood == 3) {
      for (uint32_t i = 0; i + 2 < L; ++i)
        for (uint8_t a = 0; a <= KARMA_RC_CHAIN; ++a)
          for (uint8_t b = 0; b <= KARMA_RC_CHAIN; ++b)
            for (uint8_t d = 0; d <= KARMA_RC_CHAIN; ++d)
              if (a != inc.act[i] || b != inc.act[i + 1] || d != inc.act[i + 2]) {
                cand = inc.act; cand[i] = a; cand[i + 1] = b; cand[i + 2] = d;
                moved |= attempt();
              }
    } else if (hood == 4) {
      for (uint32_t i = 0; i + 3 < L; ++i)
        for (uint32_t q = 0; q < 625; ++q) {
          const uint8_t w[4] = {(uint8_t)(q / 125), (uint8_t)(q / 25 % 5), (uint8_t)(q / 5 % 5), (uint8_t)(q % 5)};
          if (w[0] != inc.act[i] || w[1] != inc.act[i + 1] || w[2] != inc.act[i + 2] || w[3] != inc.act[i + 3]) {
            cand = inc.act;
            for (int k = 0; k < 4; ++k) cand[i + k] = w[k];
            moved |= attempt();
          }
        }
    } else {
      for (uint32_t i = 0; i < L; ++i)
        for (uint8_t a = 0; a <= KARMA_RC_CHAIN; ++a) {
          if (a == inc.act[i]) continue;
          Incumbent local;
          local.act = inc.act;
          local.act[i] = a;
          if (!evaluate(P, local.act, local.cost)) continue;
          for (bool went = true; went;) {
            went = false;
            for (uint32_t j = 0; j < L; ++j) {
              if (j == i) continue;
              for (uint8_t b = 0; b <= KARMA_RC_CHAIN; ++b) {
                if (b == local.act[j]) continue;
                cand = local.act;
                cand[j] = b;
                Cost c;
                if (evaluate(P, cand, c) && local.after(c, cand)) { local.cost = c; local.act = cand; went = true; }
              }
            }
          }
          if (inc.after(local.cost, local.act)) { inc = local; return true; }
        }
    }
    return moved;
  };
  const int hoods = P.n_skips ? 6 : 4;
  for (int hood = 0; hood < hoods;) hood = pass(hood) ? 0 : hood + 1;
}

}  // namespace

bool simulate(const Problem& P, const uint8_t* actions, const uint8_t* keepw, karma_plan_summary* out,
              std::vector<karma_op>* ops) {
  Timeline tl(P, actions, keepw, ops);
  return tl.run(out);
}

bool plan(const Problem& P, std::vector<uint8_t>& actions, std::vector<uint8_t>& keepw, karma_plan_summary* out) {
  const uint32_t L = P.n;
  Cost c;
  actions.assign(L, KARMA_KEEP);
  keepw.assign(L, 0);
  for (uint32_t i = 0; i < L; ++i) keepw[i] = P.layers[i].w_bytes ? 1 : 0;
  if (fits(P, actions, c, keepw.data())) return simulate(P, actions.data(), keepw.data(), out, nullptr);   // everything fits
  const std::vector<uint8_t> streamed = keepw;
  keepw.assign(L, 0);

  // capacity rule: the longest resident tail for a given treatment of the prefix.  The prefix's read-again
  // inputs (and, for chains, layer 0) take `special` when it is an action.
  std::vector<uint8_t> reread(L, 0);
  for (uint32_t k = 0; k < P.n_skips; ++k) reread[P.skips[k].src + 1] = 1;
  const int NONE = -1;
  auto longest_tail = [&](uint8_t fill, int special, std::vector<uint8_t>& res) {
    for (uint32_t k = 1; k <= L; ++k) {
      res.assign(L, KARMA_KEEP);
      for (uint32_t i = 0; i < k; ++i)
        res[i] = special != NONE && (reread[i] || (i == 0 && fill == KARMA_RC_CHAIN)) ? (uint8_t)special : fill;
      if (fits(P, res, c)) return true;
    }
    return false;
  };
  std::vector<std::vector<uint8_t>> starts;
  std::vector<uint8_t> s;
  if (longest_tail(KARMA_SWAP, NONE, s)) starts.push_back(s);
  if (longest_tail(KARMA_RC_KEEP, NONE, s)) starts.push_back(s);
  if (starts.empty() || P.n_skips) {
    // chains from as few checkpoints as the connections allow; with connections also a swapped prefix
    // whose read-again tensors stay, as checkpoints or whole
    auto add = [&](bool found) {
      if (found && std::find(starts.begin(), starts.end(), s) == starts.end()) starts.push_back(s);
    };
    add(longest_tail(KARMA_RC_CHAIN, KARMA_RC_KEEP, s) || longest_tail(KARMA_RC_CHAIN, KARMA_RC_SWAP, s));
    if (P.n_skips) {
      add(longest_tail(KARMA_SWAP, KARMA_RC_KEEP, s));
      add(longest_tail(KARMA_SWAP, KARMA_KEEP, s));
    }
  }
  if (starts.empty()) {
    // none of the patterns fits: the search starts from one that does not (its feasibility phase)
    s.assign(L, KARMA_RC_CHAIN);
    for (uint32_t i = 0; i < L; ++i)
      if (i == 0 || reread[i]) s[i] = KARMA_RC_SWAP;
    starts.push_back(s);
  }
  // Eq. 10.1: recompute where it is cheaper than the swap-in it replaces
  {
    const std::vector<uint8_t> unmarked = starts[0];
    bool hosted = P.loss.th_ns > 0;
    for (uint32_t i = 0; i < L; ++i) hosted |= P.layers[i].th_ns > 0;
    // swap-ins run in the backward phase
    const uint64_t bw_swap_in = hosted && P.link.bw_h2d_loaded ? P.link.bw_h2d_loaded : P.link.bw_h2d;
    std::vector<uint8_t> cur = starts[0];
    for (int64_t i = (int64_t)L - 1; i >= 0; --i) {
      if (cur[i] != KARMA_SWAP) continue;
      uint64_t xin = i ? P.layers[i - 1].out_bytes : 0;
      int64_t t_in = copy_ns(xin + P.layers[i].sav_bytes, bw_swap_in, P.link.lat_ns);
      if (P.layers[i].trc_ns < t_in) {
        for (uint8_t a : {(uint8_t)KARMA_RC_KEEP, (uint8_t)KARMA_RC_SWAP}) {
          std::vector<uint8_t> cand = cur;
          cand[i] = a;
          if (fits(P, cand, c)) { cur = cand; break; }
        }
      }
    }
    starts[0] = cur;
    if (cur != unmarked) starts.push_back(unmarked);   // the capacity-based schedule itself (Fig. 2(b)) is a start too
  }
  bool have = false;
  Incumbent best;
  for (auto& st : starts) {
    Incumbent inc;
    inc.act = st;
    if (!evaluate(P, st, inc.cost)) continue;
    improve(P, inc);
    if (!have || best.after(inc.cost, inc.act)) { best = inc; have = true; }
  }
  if (!have || best.cost.unfit) return false;
  actions = best.act;
  // the tail of the model keeps its streamed weights between forward and backward for as
  // long as that fits and does not lengthen the step; the first layer that cannot ends the scan
  Cost cost = best.cost;
  for (int64_t i = (int64_t)L - 1; i >= 0; --i) {
    if (!streamed[i]) continue;
    keepw[i] = 1;
    if (fits(P, actions, c, keepw.data()) && c < cost) {
      cost = c;
    } else {
      keepw[i] = 0;
      break;
    }
  }
  return simulate(P, actions.data(), keepw.data(), out, nullptr);
}

// Algorithm 1's notation.  A copy is printed on the stage that is running when the copy
// starts; recompute stages are inserted as fresh stages and carry no copies.
std::string stage_string(const karma_op* ops, uint32_t n) {
  std::vector<uint32_t> stages;
  for (uint32_t k = 0; k < n; ++k)
    if (ops[k].kind == 'F' || ops[k].kind == 'B' || ops[k].kind == 'R') stages.push_back(k);
  std::vector<std::string> text(stages.size());
  for (size_t s = 0; s < stages.size(); ++s) {
    const karma_op& o = ops[stages[s]];
    text[s] = std::string(o.kind == 'B' ? "B" : "F") + std::to_string(o.layer + 1);
  }
  for (uint32_t k = 0; k < n; ++k) {
    const uint8_t kd = ops[k].kind;
    if (kd != 'I' && kd != 'O' && kd != 'W' && kd != 'G') continue;
    if (stages.empty()) break;
    size_t at = stages.size() - 1;
    for (size_t s = 0; s < stages.size(); ++s) {
      const karma_op& o = ops[stages[s]];
      if (o.kind != 'R' && o.end_ns > ops[k].start_ns) { at = s; break; }
    }
    text[at] += std::string("||") + (kd == 'W' ? "W" : kd == 'G' ? "G" : "S") + std::to_string(ops[k].layer + 1) +
                ((kd == 'I' || kd == 'W') ? "^in" : "^out");
  }
  std::string res;
  for (size_t s = 0; s < text.size(); ++s) { if (s) res += " -> "; res += text[s]; }
  return res;
}

// The planner with the block granularity chosen as well (Sec. III-E/F: the first tier of the
// optimisation groups layers into blocks, which are then kept, swapped or recomputed as a whole).
// For each candidate group size consecutive layers are merged (times, streamed weights and
// gradients add up; the block's internals are its members' internals plus the boundaries between
// them; its output is the last member's; workspace is the largest), the merged stack is planned, the
// block-level plan is expanded to per-layer actions (a recomputed block keeps or swaps its first
// member's input as the checkpoint and chains the rest) and priced by the per-layer simulator, which
// is what the executor follows.  The cheapest expansion wins, the smaller group on ties; size 1 is
// the plain planner, so the result is never worse than plan().
bool plan_grouped(const Problem& P, uint32_t max_group, std::vector<uint8_t>& actions, std::vector<uint8_t>& keepw,
                  karma_plan_summary* out, uint32_t* group_out) {
  static const uint32_t sizes_tried[] = {1, 2, 3, 4, 6, 8};
  const uint32_t L = P.n;
  bool have = false;
  Cost best{};
  std::vector<uint8_t> best_a, best_w;
  uint32_t best_g = 1;
  for (uint32_t g : sizes_tried) {
    if (g > max_group || (g > 1 && g > L)) continue;
    std::vector<uint8_t> a, w;
    if (g == 1) {
      karma_plan_summary s;
      if (!plan(P, a, w, &s)) continue;
    } else {
      std::vector<karma_layer_cost> merged;
      std::vector<uint32_t> count;
      for (uint32_t first = 0; first < L; first += g) {
        const uint32_t n = std::min(g, L - first);
        karma_layer_cost m{};
        for (uint32_t k = 0; k < n; ++k) {
          const karma_layer_cost& l = P.layers[first + k];
          m.tf_ns += l.tf_ns; m.tb_ns += l.tb_ns; m.trc_ns += k + 1 < n ? l.tf_ns : l.trc_ns;
          m.sav_bytes += l.sav_bytes + (k + 1 < n ? l.out_bytes : 0);
          m.ws_bytes = std::max(m.ws_bytes, l.ws_bytes);
          m.w_bytes += l.w_bytes; m.g_bytes += l.g_bytes;
          m.th_ns += l.th_ns; m.hg_bytes += l.hg_bytes; m.hw_bytes += l.hw_bytes;
        }
        m.out_bytes = P.layers[first + n - 1].out_bytes;
        merged.push_back(m);
        count.push_back(n);
      }
      // a connection survives at block level when its source is the last member of its block (the tensor
      // is then that block's output) and its reader sits at least two blocks on; the others lie inside a
      // block or between neighbours and are priced only by the per-layer simulator
      std::vector<karma_skip> gs;
      for (uint32_t k = 0; k < P.n_skips; ++k) {
        const uint32_t bs = P.skips[k].src / g, bd = P.skips[k].dst / g;
        if (P.skips[k].src == bs * g + count[bs] - 1 && bd >= bs + 2) gs.push_back(karma_skip{bs, bd});
      }
      std::sort(gs.begin(), gs.end(), [](const karma_skip& a, const karma_skip& b) {
        return a.src != b.src ? a.src < b.src : a.dst < b.dst;
      });
      gs.erase(std::unique(gs.begin(), gs.end(), [](const karma_skip& a, const karma_skip& b) {
        return a.src == b.src && a.dst == b.dst;
      }), gs.end());
      Problem G{merged.data(), (uint32_t)merged.size(), P.link, P.loss, P.budget, P.fixed, gs.data(), (uint32_t)gs.size()};
      std::vector<uint8_t> ga, gw;
      karma_plan_summary s;
      if (!plan(G, ga, gw, &s)) continue;
      for (size_t b = 0; b < count.size(); ++b)
        for (uint32_t k = 0; k < count[b]; ++k) {
          const bool whole = ga[b] == KARMA_KEEP || ga[b] == KARMA_SWAP || ga[b] == KARMA_RC_CHAIN;
          a.push_back(whole || k == 0 ? ga[b] : (uint8_t)KARMA_RC_CHAIN);
          w.push_back(gw[b]);
        }
    }
    Cost c;
    if (!fits(P, a, c, w.data())) continue;
    if (!have || c < best) {
      have = true;
      best = c; best_a = a; best_w = w; best_g = g;
    }
  }
  if (!have) return false;
  actions = best_a;
  keepw = best_w;
  if (group_out) *group_out = best_g;
  return simulate(P, actions.data(), keepw.data(), out, nullptr);
}

}  // namespace karma
