// Stream/event executor of the out-of-core training step (KARMA Fig. 2(c), Algorithm 1,
// Sec. III-G stage 3 and 5).  The plan is compiled once into a static program: every op
// knows its arena offsets and the ops it must wait for, so a step is a replay that
// allocates nothing.  Swap-out and prefetch are pinned hipMemcpyAsync calls on their own
// streams; cross-stream ordering is by events.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstring>

#include "context.h"
#include "kernels.h"
#include "layers.h"

using namespace karma;

struct karma_ctx : public Ctx {};

namespace {

inline uint64_t up256(uint64_t b) { return (b + 255) / 256 * 256; }

double now_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

int fail(Ctx* c, int code, const std::string& msg) {
  c->err = msg;
  return code;
}

void free_plan_resources(Ctx* c) {
  for (auto e : c->ev) if (e) (void)hipEventDestroy(e);
  for (auto e : c->ev_begin) if (e) (void)hipEventDestroy(e);
  c->ev.clear();
  c->ev_begin.clear();
  if (c->swap_pool) (void)hipHostFree(c->swap_pool);
  c->swap_pool = nullptr;
  c->swap_pool_bytes = 0;
  c->planned = false;
}

// ---- compile the simulated timeline into the executable program ------------------
struct Released { int64_t off, size; uint32_t op; };

struct Builder {
  Ctx& c;
  std::vector<Released> gone;   // ranges of the arena that were freed, with the op that freed them
  std::vector<int64_t> x_at, s_at, dx_at, x_sz, s_sz, w_sz;
  std::vector<int64_t> p_at, g_at, p_sz, g_sz;   // streamed weights and their gradients
  explicit Builder(Ctx& ctx) : c(ctx) {}

  // the new tenant of [off, off+size) must wait for whoever released any part of it
  void claim(ProgOp& op, int64_t off, int64_t size) {
    if (off < 0 || size == 0) return;
    std::vector<Released> keep;
    for (const Released& r : gone) {
      int64_t lo = std::max(r.off, off), hi = std::min(r.off + r.size, off + size);
      if (lo >= hi) { keep.push_back(r); continue; }
      op.waits.push_back(r.op);
      if (r.off < lo) keep.push_back({r.off, lo - r.off, r.op});
      if (hi < r.off + r.size) keep.push_back({hi, r.off + r.size - hi, r.op});
    }
    gone.swap(keep);
  }
  void release(int64_t& off, int64_t size, uint32_t op) {
    if (off >= 0 && size) gone.push_back({off, size, op});
    off = -1;
  }

  int run() {
    const uint32_t L = c.L;
    x_sz.assign(L + 2, 0); s_sz.assign(L, 0); w_sz.assign(L, 0);
    p_sz.assign(L, 0); g_sz.assign(L, 0);
    for (uint32_t i = 0; i < L; ++i) {
      x_sz[i + 1] = (int64_t)up256(c.cost[i].out_bytes);
      s_sz[i] = (int64_t)up256(c.cost[i].sav_bytes);
      w_sz[i] = (int64_t)up256(c.cost[i].ws_bytes);
      p_sz[i] = (int64_t)up256(c.cost[i].w_bytes);
      g_sz[i] = c.cost[i].w_bytes ? (int64_t)up256(c.cost[i].g_bytes) : 0;
    }
    p_at.assign(L, -1); g_at.assign(L, -1);
    std::vector<int64_t> win_op(L, -1), b_op(L, -1);
    const int64_t lw_sz = (int64_t)up256(c.loss_cost.ws_bytes);
    x_at.assign(L + 2, -1); s_at.assign(L, -1); dx_at.assign(L + 2, -1);
    std::vector<int64_t> f_op(L, -1), in_op(L, -1), out_op(L, -1);
    // connections between non-consecutive records: reads[j] = the inputs x_s record j reads again (ascending);
    // hold_at[s] = the buffer in which the readers' gradient for x_s waits for B_s
    std::vector<std::vector<uint32_t>> reads(L);
    for (const karma_skip& e : c.skips) reads[e.dst].push_back(e.src + 1);
    for (auto& r : reads) {
      std::sort(r.begin(), r.end());
      r.erase(std::unique(r.begin(), r.end()), r.end());
      if (r.size() > (size_t)LayerIO::MAX_SKIPS) return KARMA_E_INVAL;
    }
    std::vector<int64_t> hold_at(L + 1, -1), x_in_op(L + 1, -1);   // x_in_op[s]: the copy that brought x_s back
    std::vector<uint8_t> hold_written(L + 1, 0);
    // what a reader's op takes from the records it reads again; false when one of them is not in memory
    auto read_again = [&](ProgOp& p, uint32_t j) {
      for (uint32_t s : reads[j]) {
        if (x_at[s] < 0) return false;
        p.rx.push_back(x_at[s]);
        if (x_in_op[s] >= 0) p.waits.push_back((uint32_t)x_in_op[s]);   // a premature swap-in
      }
      return true;
    };
    uint64_t host_top = 0;
    std::vector<int64_t> host_x(L, -1), host_s(L, -1);
    c.prog.clear();
    c.prog.reserve(c.ops.size());
    for (uint32_t k = 0; k < c.ops.size(); ++k) {
      const karma_op& o = c.ops[k];
      ProgOp p;
      p.kind = (char)o.kind;
      p.layer = o.layer;
      const uint32_t i = o.layer;
      const uint8_t a = i < L ? c.actions[i] : 0;
      switch (o.kind) {
        case 'F':
          p.stream = 0;
          p.x = i == 0 ? -2 : x_at[i];
          p.out = o.off[0]; p.s = o.off[1]; p.ws = o.off[2];
          claim(p, p.out, x_sz[i + 1]); claim(p, p.s, s_sz[i]); claim(p, p.ws, w_sz[i]);
          x_at[i + 1] = p.out; s_at[i] = p.s;
          if (!read_again(p, i)) return KARMA_E_INVAL;
          f_op[i] = k;
          { int64_t w = p.ws; release(w, w_sz[i], k); }
          if (p_sz[i]) {
            p.w = p_at[i];
            p.waits.push_back((uint32_t)win_op[i]);
            if (!c.keepw[i]) release(p_at[i], p_sz[i], k);
          }
          if (a == KARMA_RC_KEEP || a == KARMA_RC_CHAIN) release(s_at[i], s_sz[i], k);
          if (a == KARMA_RC_CHAIN) release(x_at[i], x_sz[i], k);
          if (a == KARMA_RC_SWAP) release(s_at[i], s_sz[i], k);
          break;
        case 'O':
          p.stream = 2;
          p.x = x_at[i];
          p.x_bytes = i ? c.cost[i - 1].out_bytes : 0;
          if (a == KARMA_SWAP) { p.s = s_at[i]; p.s_bytes = c.cost[i].sav_bytes; }
          if (p.x < 0) p.x_bytes = 0;
          if (p.s < 0) p.s_bytes = 0;
          p.waits.push_back((uint32_t)f_op[i]);
          if (p.x_bytes) { host_x[i] = (int64_t)host_top; host_top += up256(p.x_bytes); }
          if (p.s_bytes) { host_s[i] = (int64_t)host_top; host_top += up256(p.s_bytes); }
          p.host_x = host_x[i]; p.host_s = host_s[i];
          out_op[i] = k;
          release(x_at[i], x_sz[i], k);
          if (a == KARMA_SWAP) release(s_at[i], s_sz[i], k);
          break;
        case 'I':
          p.stream = 1;
          p.x = o.off[0]; p.s = o.off[1];
          p.x_bytes = p.x >= 0 ? c.cost[i - 1].out_bytes : 0;
          p.s_bytes = p.s >= 0 ? c.cost[i].sav_bytes : 0;
          p.host_x = host_x[i]; p.host_s = host_s[i];
          claim(p, p.x, x_sz[i]); claim(p, p.s, s_sz[i]);
          if (out_op[i] >= 0) p.waits.push_back((uint32_t)out_op[i]);   // host copy must be complete
          if (p.x >= 0) { x_at[i] = p.x; x_in_op[i] = k; }   // (an input that came back early for a reader stays where it is)
          if (a == KARMA_SWAP && p.s >= 0) s_at[i] = p.s;
          in_op[i] = k;
          break;
        case 'W':
          p.stream = 1;
          p.w = o.off[0];
          claim(p, p.w, p_sz[i]);
          p_at[i] = p.w;
          win_op[i] = k;
          break;
        case 'G':
          p.stream = 2;
          p.g = g_at[i];
          p.waits.push_back((uint32_t)b_op[i]);
          release(g_at[i], g_sz[i], k);
          p.record = true;   // the host update waits for it
          break;
        case 'L':
          p.stream = 0;
          p.x = x_at[L]; p.dx = o.off[0]; p.ws = o.off[1];
          claim(p, p.dx, x_sz[L]); claim(p, p.ws, lw_sz);
          dx_at[L] = p.dx;
          { int64_t w = p.ws; release(w, lw_sz, k); }
          release(x_at[L], x_sz[L], k);
          p.record = true;
          break;
        case 'R':
          p.stream = 0;
          p.x = i == 0 ? -2 : x_at[i];
          p.s = o.off[0]; p.out = o.off[1]; p.ws = o.off[2];
          claim(p, p.s, s_sz[i]); claim(p, p.out, x_sz[i + 1]); claim(p, p.ws, w_sz[i]);
          s_at[i] = p.s;
          if (p.out >= 0) x_at[i + 1] = p.out;
          if (in_op[i] >= 0) p.waits.push_back((uint32_t)in_op[i]);
          if (!read_again(p, i)) return KARMA_E_INVAL;
          { int64_t w = p.ws; release(w, w_sz[i], k); }
          if (p_sz[i]) {
            p.w = p_at[i];
            p.waits.push_back((uint32_t)win_op[i]);
          }
          break;
        case 'H':
          // no work of its own: on the compute stream, so that the backward op behind it inherits the waits
          // for whoever held this memory before
          p.stream = 0;
          if (i > L || hold_at[i] >= 0) return KARMA_E_INVAL;
          claim(p, o.off[0], x_sz[i]);
          hold_at[i] = o.off[0];
          hold_written[i] = 0;
          break;
        case 'B':
          p.stream = 0;
          p.x = i == 0 ? -2 : x_at[i];
          p.s = s_at[i]; p.dy = dx_at[i + 1]; p.dx = o.off[0]; p.ws = o.off[1];
          claim(p, p.dx, x_sz[i]); claim(p, p.ws, w_sz[i]);
          dx_at[i] = p.dx;
          if (in_op[i] >= 0) p.waits.push_back((uint32_t)in_op[i]);
          if (!read_again(p, i)) return KARMA_E_INVAL;
          for (uint32_t sdx : reads[i]) {
            if (hold_at[sdx] < 0) return KARMA_E_INVAL;
            p.rdx.push_back(hold_at[sdx]);
            p.rdx_first.push_back(hold_written[sdx] ? 0 : 1);
            hold_written[sdx] = 1;
          }
          if (hold_at[i] >= 0) {
            if (!hold_written[i] || p.dx < 0) return KARMA_E_INVAL;
            p.hold = hold_at[i];
            p.hold_elems = c.cost[i - 1].out_bytes / 2;
            release(hold_at[i], x_sz[i], k);
          }
          { int64_t w = p.ws; release(w, w_sz[i], k); }
          release(dx_at[i + 1], x_sz[i + 1], k);
          release(s_at[i], s_sz[i], k);
          if (i) release(x_at[i], x_sz[i], k);
          if (p_sz[i]) {
            p.w = p_at[i];
            p.waits.push_back((uint32_t)win_op[i]);
            release(p_at[i], p_sz[i], k);
            p.g = o.off[2];
            claim(p, p.g, g_sz[i]);
            g_at[i] = p.g;
            b_op[i] = k;
          }
          p.record = true;
          break;
        default:
          return KARMA_E_INVAL;
      }
      c.prog.push_back(std::move(p));
    }
    // only cross-stream waits need events
    for (ProgOp& p : c.prog) {
      std::vector<uint32_t> w;
      for (uint32_t d : p.waits)
        if (c.prog[d].stream != p.stream && std::find(w.begin(), w.end(), d) == w.end()) {
          w.push_back(d);
          c.prog[d].record = true;
        }
      p.waits.swap(w);
    }
    c.swap_pool_bytes = host_top;
    return KARMA_OK;
  }
};

int finish_all_updates(Ctx* c);

int install_plan(Ctx* c, uint64_t budget, const std::vector<uint8_t>& actions, const std::vector<uint8_t>& keepw) {
  if (budget > c->arena_bytes) return fail(c, KARMA_E_OOM, "budget exceeds the arena handed to karma_create");
  int fst = finish_all_updates(c);
  if (fst) return fst;
  Problem P{c->cost.data(), c->L, c->link, c->loss_cost, budget, c->fixed_bytes, c->skips.data(), (uint32_t)c->skips.size()};
  std::vector<karma_op> ops;
  karma_plan_summary s;
  if (!actions_valid(actions.data(), c->L, P.skips, P.n_skips)) return fail(c, KARMA_E_INVAL, "invalid action vector");
  if (!simulate(P, actions.data(), keepw.data(), &s, &ops)) return fail(c, KARMA_E_BUDGET, "assignment does not fit the budget");
  free_plan_resources(c);
  c->actions = actions;
  c->keepw = keepw;
  c->ops = ops;
  c->summary = s;
  c->budget = budget;
  Builder b(*c);
  int st = b.run();
  if (st) return fail(c, st, "schedule compilation failed");
  if (c->swap_pool_bytes) {
    if (hipHostMalloc((void**)&c->swap_pool, c->swap_pool_bytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();   // or the next launch check would report this allocation's error as its own
      c->swap_pool = nullptr;
      c->planned = false;        // the previous plan's resources are gone and this one's are not there
      return fail(c, KARMA_E_HOSTMEM, "pinned swap pool allocation failed");
    }
  }
  c->ev.assign(c->prog.size(), nullptr);
  c->ev_begin.assign(c->prog.size(), nullptr);
  for (size_t k = 0; k < c->prog.size(); ++k) {
    KARMA_HIP(c, hipEventCreate(&c->ev[k]));
    KARMA_HIP(c, hipEventCreate(&c->ev_begin[k]));
  }
  c->op_ms.assign(c->prog.size(), 0.f);
  c->op_start_ms.assign(c->prog.size(), 0.f);
  c->planned = true;
  return KARMA_OK;
}

int issue(Ctx* c, const ProgOp& p) {
  hipStream_t s = c->st[p.stream];
  LayerIO io;
  io.x = p.x == -2 ? (const void*)c->fixed_ptr(c->in_off) : (const void*)c->act_ptr(p.x);
  io.out = c->act_ptr(p.out);
  io.sav = c->act_ptr(p.s);
  io.ws = c->act_ptr(p.ws);
  io.dy = c->act_ptr(p.dy);
  io.dx = c->act_ptr(p.dx);
  io.w = c->act_ptr(p.w);
  io.g = c->act_ptr(p.g);
  io.n_skips = (int)p.rx.size();
  for (size_t j = 0; j < p.rx.size(); ++j) io.skip_x[j] = c->act_ptr(p.rx[j]);
  for (size_t j = 0; j < p.rdx.size(); ++j) {
    io.skip_dx[j] = c->act_ptr(p.rdx[j]);
    io.skip_dx_first[j] = p.rdx_first[j] != 0;
  }
  switch (p.kind) {
    case 'F':
    case 'R': return layer_forward(*c, p.layer, io, s);
    case 'B': {
      int st = layer_backward(*c, p.layer, io, s);
      if (st) return st;
      // the gradient its other readers left for this record's input joins the one just computed
      if (p.hold >= 0) return add_inplace_bf16((bf16_t*)io.dx, (const bf16_t*)c->act_ptr(p.hold), p.hold_elems, s);
      return KARMA_OK;
    }
    case 'H': return KARMA_OK;
    case 'L': return loss_op(*c, io, s);
    case 'O':
      if (p.x_bytes) KARMA_HIP(c, hipMemcpyAsync(c->swap_pool + p.host_x, c->act_ptr(p.x), p.x_bytes, hipMemcpyDeviceToHost, s));
      if (p.s_bytes) KARMA_HIP(c, hipMemcpyAsync(c->swap_pool + p.host_s, c->act_ptr(p.s), p.s_bytes, hipMemcpyDeviceToHost, s));
      return KARMA_OK;
    case 'I':
      if (p.x_bytes) KARMA_HIP(c, hipMemcpyAsync(c->act_ptr(p.x), c->swap_pool + p.host_x, p.x_bytes, hipMemcpyHostToDevice, s));
      if (p.s_bytes) KARMA_HIP(c, hipMemcpyAsync(c->act_ptr(p.s), c->swap_pool + p.host_s, p.s_bytes, hipMemcpyHostToDevice, s));
      return KARMA_OK;
    case 'W':
      KARMA_HIP(c, hipMemcpyAsync(c->act_ptr(p.w), c->rec[p.layer].stage_w_all, c->rec[p.layer].w_total, hipMemcpyHostToDevice, s));
      return KARMA_OK;
    case 'G':
      // gradients that share the weights' pinned buffer leave the device only when the host update that
      // turns them into the next weights is part of the step
      if (c->rec[p.layer].shared_staging) {
        const Record& r = c->rec[p.layer];
        if (!c->applying) return KARMA_OK;
        if (r.shared_bytes)
          KARMA_HIP(c, hipMemcpyAsync(r.stage_w_all, c->act_ptr(p.g), r.shared_bytes, hipMemcpyDeviceToHost, s));
        if (r.g_total > r.shared_bytes)
          KARMA_HIP(c, hipMemcpyAsync(r.stage_g_all, c->act_ptr(p.g) + r.shared_bytes, r.g_total - r.shared_bytes,
                                      hipMemcpyDeviceToHost, s));
        return KARMA_OK;
      }
      KARMA_HIP(c, hipMemcpyAsync(c->rec[p.layer].stage_g_all, c->act_ptr(p.g), c->rec[p.layer].g_total, hipMemcpyDeviceToHost, s));
      return KARMA_OK;
  }
  return KARMA_E_INVAL;
}

// gradients of one record: device -> pinned host in chunks, after the op that completed them
int send_grads(Ctx* c, uint32_t r, hipEvent_t after) {
  hipStream_t s = c->st[2];
  KARMA_HIP(c, hipStreamWaitEvent(s, after, 0));
  Record& rc = c->rec[r];
  if (rc.whole_copies) {
    KARMA_HIP(c, hipMemcpyAsync(rc.stage_g_all, c->arena + rc.g_base, rc.g_span, hipMemcpyDeviceToHost, s));
    KARMA_HIP(c, hipEventRecord(rc.grads_ev, s));
    return KARMA_OK;
  }
  for (Param& p : c->rec[r].p) {
    const uint64_t gs = p.grad_bf16 ? 2 : 4;
    for (size_t k = 0; k < p.chunk_ev.size(); ++k) {
      const uint64_t lo = k * PARAM_CHUNK, n = std::min(PARAM_CHUNK, p.n - lo);
      KARMA_HIP(c, hipMemcpyAsync((char*)p.stage_g + lo * gs, c->arena + p.g_off + lo * gs, n * gs, hipMemcpyDeviceToHost, s));
      KARMA_HIP(c, hipEventRecord(p.chunk_ev[k], s));
    }
  }
  return KARMA_OK;
}

// host update of one record's master weights, chunk by chunk as the gradients land; each
// chunk's new device weights go back at once
// step: the optimiser step the gradients belong to; landed: the gradients are known to be on the host
// already (an update left over from a finished step), no event is waited for
int update_record(Ctx* c, uint32_t r, hipEvent_t grads_landed, uint64_t step, bool landed) {
  const karma_config& g = c->cfg;
  const bool streamed = c->rec[r].streamed;
  // streamed records: the whole gradient buffer arrives with one copy of the program, and
  // the new weights stay in pinned memory for the next step's copy-in
  if (streamed && !landed) KARMA_HIP(c, hipEventSynchronize(grads_landed));
  const bool whole = c->rec[r].whole_copies;
  if (whole && !landed) KARMA_HIP(c, hipEventSynchronize(c->rec[r].grads_ev));
  double spent_ms = 0.0;
  for (Param& p : c->rec[r].p) {
    const uint64_t gs = p.grad_bf16 ? 2 : 4, ws = p.dev_bf16 ? 2 : 4;
    for (size_t k = 0; k < p.chunk_ev.size(); ++k) {
      const uint64_t base = k * PARAM_CHUNK, n = std::min(PARAM_CHUNK, p.n - base);
      if (!streamed && !whole && !landed) KARMA_HIP(c, hipEventSynchronize(p.chunk_ev[k]));
      double t0 = now_ms();
      c->pool->parallel_for(n, [&](size_t lo, size_t hi) {
        const char* gp = (const char*)p.stage_g + (base + lo) * gs;
        char* wp = (char*)p.stage_w + (base + lo) * ws;
        if (g.optimizer == KARMA_OPT_ADAM)
          adam_update(p.master.data() + base + lo, p.m.data() + base + lo, p.v.data() + base + lo, gp, p.grad_bf16,
                      hi - lo, g.lr, g.beta1, g.beta2, g.eps, step, wp, p.dev_bf16);
        else if (g.optimizer == KARMA_OPT_SGD_MOMENTUM)
          sgd_momentum_update(p.master.data() + base + lo, p.m.data() + base + lo, gp, p.grad_bf16, hi - lo, g.lr, g.beta1, wp,
                              p.dev_bf16);
        else
          sgd_update(p.master.data() + base + lo, gp, p.grad_bf16, hi - lo, g.lr, wp, p.dev_bf16);
      });
      const double dt = now_ms() - t0;
      c->stats.host_opt_ms += dt;
      spent_ms += dt;
      if (!streamed && !whole)
        KARMA_HIP(c, hipMemcpyAsync(c->arena + p.w_off + base * ws, (char*)p.stage_w + base * ws, n * ws,
                                    hipMemcpyHostToDevice, c->st[1]));
    }
  }
  if (whole)   // every tensor's new weights with one copy (the gaps between them are alignment padding on both sides)
    KARMA_HIP(c, hipMemcpyAsync(c->arena + c->rec[r].w_base, c->rec[r].stage_w_all, c->rec[r].w_span, hipMemcpyHostToDevice,
                                c->st[1]));
  if (r < c->update_ns.size()) c->update_ns[r] = (int64_t)(spent_ms * 1e6);
  return KARMA_OK;
}

// An update that the step which produced its gradients left for later: run it now.  reader: the stream of the
// op about to read the record's weights (nullptr: none); it is made to wait for the weight copies.
int finish_update(Ctx* c, uint32_t r, hipStream_t reader) {
  if (r >= c->pending_update.size() || !c->pending_update[r]) return KARMA_OK;
  const uint64_t step = c->pending_update[r];
  c->pending_update[r] = 0;
  int st = update_record(c, r, nullptr, step, true);
  if (st) return st;
  if (!c->rec[r].streamed && reader && reader != c->st[1]) {
    KARMA_HIP(c, hipEventRecord(c->weights_uploaded, c->st[1]));
    KARMA_HIP(c, hipStreamWaitEvent(reader, c->weights_uploaded, 0));
  }
  return KARMA_OK;
}

// Every update still owed, in record order, and the weight copies they start
int finish_all_updates(Ctx* c) {
  bool any = false;
  for (uint32_t r = 0; r < c->pending_update.size(); ++r)
    if (c->pending_update[r]) {
      any = true;
      int st = finish_update(c, r, nullptr);
      if (st) return st;
    }
  if (any) KARMA_HIP(c, hipStreamSynchronize(c->st[1]));
  return KARMA_OK;
}

// one GEMM launch in this many carries timing events under KARMA_STEP_KERNEL_TIMES
static const unsigned GEMM_TIMER_STRIDE = 8;

int run_step(Ctx* c, const void* in, const void* lab, uint32_t flags, float* loss_out, bool profile) {
  if (!c->planned) return fail(c, KARMA_E_STATE, "karma_step before karma_plan / karma_set_plan");
  const bool apply = flags & KARMA_STEP_APPLY_OPTIMIZER;
  c->applying = apply;
  c->ktime = (flags & KARMA_STEP_KERNEL_TIMES) != 0;
  c->kev_used = 0;
  c->kflops.clear();
  GemmTimer timer{&c->kev, &c->kev_used, &c->kflops, GEMM_TIMER_STRIDE, (unsigned)(c->ktime_steps++ % GEMM_TIMER_STRIDE), 0};
  struct TimerScope {   // per-launch GEMM timing for the duration of this step only
    explicit TimerScope(GemmTimer* t) { g_gemm_timer = t; }
    ~TimerScope() { g_gemm_timer = nullptr; }
  } timer_scope(c->ktime ? &timer : nullptr);
  double t0 = now_ms();
  c->stats = karma_step_stats{};
  int st = KARMA_OK;
  hipStream_t sc = c->st[0];
  if (in) {
    st = model_prepare_step(*c, in, lab);
    if (st) return st;
    KARMA_HIP(c, hipMemcpyAsync(c->fixed_ptr(c->in_off), c->stage_in, c->in_bytes, hipMemcpyHostToDevice, sc));
    KARMA_HIP(c, hipMemcpyAsync(c->fixed_ptr(c->lab_off), c->stage_lab, c->lab_bytes, hipMemcpyHostToDevice, sc));
  } else if (!c->inputs_resident) {
    return fail(c, KARMA_E_STATE, "karma_step without inputs before any step with inputs");
  }
  if (apply) ++c->step_no;
  std::vector<std::pair<uint32_t, hipEvent_t>> done_order;   // record, event after which its gradients are on the host
  for (size_t k = 0; k < c->prog.size(); ++k) {
    const ProgOp& p = c->prog[k];
    hipStream_t s = c->st[p.stream];
    for (uint32_t d : p.waits) KARMA_HIP(c, hipStreamWaitEvent(s, c->ev[d], 0));
    if (p.kind == 'B' && p.layer == 0 && c->misc_bytes) {
      // host-side preparation that only this op needs; the GPU has been busy all along
      st = model_prepare_late(*c);
      if (st) return st;
      KARMA_HIP(c, hipMemcpyAsync(c->fixed_ptr(c->misc_off), c->stage_misc, c->misc_bytes, hipMemcpyHostToDevice, s));
    }
    // weights whose update the previous step left for now: finished right before their first reader (the
    // forward pass asks for them in record order; the loss also reads tensors of other records)
    if (p.kind == 'L') st = finish_all_updates(c);
    else if (p.kind == 'F' || p.kind == 'R' || p.kind == 'B' || p.kind == 'W') st = finish_update(c, p.layer, s);
    else st = KARMA_OK;
    if (st) return st;
    if (profile) KARMA_HIP(c, hipEventRecord(c->ev_begin[k], s));
    st = issue(c, p);
    if (st) return st;
    if (p.record || profile) KARMA_HIP(c, hipEventRecord(c->ev[k], s));
    if (apply && (p.kind == 'L' || p.kind == 'B')) {
      uint32_t r = p.kind == 'L' ? c->L : p.layer;
      // gradients of a record are complete after its backward; a tied tensor that several
      // records add to is owned by the record that finishes last
      if (!c->rec[r].p.empty() && c->rec[r].p[0].dev_opt) {
        // updated where they are, behind the backward op on the compute stream
        const karma_config& g = c->cfg;
        for (Param& q : c->rec[r].p) {
          st = optim_update_dev((int)g.optimizer, (float*)(c->arena + q.dmaster_off), (float*)(c->arena + q.dm_off),
                                (float*)(c->arena + q.dv_off), c->arena + q.g_off, q.grad_bf16, (size_t)q.n, g.lr, g.beta1,
                                g.beta2, g.eps, c->step_no, c->arena + q.w_off, q.dev_bf16, s);
          if (st) return st;
        }
      } else if (!c->rec[r].p.empty() && !c->rec[r].streamed) {
        st = send_grads(c, r, c->ev[k]);
        if (st) return st;
        done_order.push_back({r, nullptr});
      }
    }
    if (apply && p.kind == 'G') done_order.push_back({p.layer, c->ev[k]});
  }
  KARMA_HIP(c, hipMemcpyAsync(c->stage_loss, c->fixed_ptr(c->loss_off), sizeof(float), hipMemcpyDeviceToHost, sc));
  // Updates run here as their gradients land, while the GPU works on the rest of the step.  Once the GPU has
  // finished the step, what is left is put off: the next step (or whoever asks for the weights) finishes each
  // record's update right before its first use, so the forward pass of the next iteration overlaps them.
  // (the H2D stream is asked through an event behind the program's own copies: the updates below add their
  // weight copies to it)
  KARMA_HIP(c, hipEventRecord(c->program_h2d_done, c->st[1]));
  auto gpu_finished = [&]() {
    if (hipStreamQuery(c->st[0]) == hipSuccess && hipStreamQuery(c->st[2]) == hipSuccess &&
        hipEventQuery(c->program_h2d_done) == hipSuccess)
      return true;
    (void)hipGetLastError();   // "not ready" is an answer, not an error for the next launch check to find
    return false;
  };
  size_t di = 0;
  for (; di < done_order.size(); ++di) {
    if (!profile && gpu_finished()) break;
    st = update_record(c, done_order[di].first, done_order[di].second, c->step_no, false);
    if (st) return st;
  }
  for (int k = 0; k < 3; ++k) KARMA_HIP(c, hipStreamSynchronize(c->st[k]));
  c->stats.updates_deferred = done_order.size() - di;
  for (; di < done_order.size(); ++di) c->pending_update[done_order[di].first] = c->step_no;
  if (loss_out) *loss_out = *c->stage_loss;
  c->stats.step_ms = now_ms() - t0;
  c->stats.bytes_d2h = c->summary.bytes_d2h;
  c->stats.bytes_h2d = c->summary.bytes_h2d;
  c->stats.arena_peak_bytes = c->summary.peak_bytes;
  if (c->ktime) {
    c->gemm_launches = c->kflops.size();
    c->gemm_ms = 0;
    c->gemm_flops = 0;
    for (size_t j = 0; j < c->kflops.size(); ++j) {
      float ms = 0.f;
      KARMA_HIP(c, hipEventElapsedTime(&ms, c->kev[2 * j], c->kev[2 * j + 1]));
      c->gemm_ms += ms;
      c->gemm_flops += c->kflops[j];
    }
  }
  if (profile) {
    for (size_t k = 0; k < c->prog.size(); ++k) {
      float ms = 0.f;
      KARMA_HIP(c, hipEventElapsedTime(&ms, c->ev_begin[k], c->ev[k]));
      c->op_ms[k] = ms;
      float since = 0.f;
      if (k) KARMA_HIP(c, hipEventElapsedTime(&since, c->ev_begin[0], c->ev_begin[k]));
      c->op_start_ms[k] = since;
      int sidx = c->prog[k].stream;
      if (sidx == 0) c->stats.compute_busy_ms += ms;
      else if (sidx == 1) c->stats.h2d_ms += ms;
      else c->stats.d2h_ms += ms;
    }
  }
  return KARMA_OK;
}

}  // namespace

// Records, the layout of the fixed region and the byte fields of the cost records, from the
// model description alone (no GPU call): shared by karma_create and the analytic cost model.
int karma::derive_layout(Ctx& c) {
  int st = model_build_records(c);
  if (st) return st;
  c.L = (uint32_t)c.rec.size() - 1;
  for (uint32_t r = 0; r < c.cfg.device_update_first && r < c.L; ++r)
    if (!c.rec[r].streamed)
      for (Param& p : c.rec[r].p) p.dev_opt = true;
  // fixed-region layout: weights, gradients, inputs, labels, loss, misc
  uint64_t off = 0;
  for (Record& r : c.rec) {
    if (r.streamed) {
      // tensors whose gradient has the weight's element type come first: their offsets in the record's
      // weight and gradient buffers coincide (one pinned buffer can then serve both)
      for (int pass = 0; pass < 2; ++pass) {
        for (Param& p : r.p) {
          if ((p.w_bytes() == p.g_bytes()) != (pass == 0)) continue;
          p.w_rel = r.w_total; r.w_total += up256(p.w_bytes());
          p.g_rel = r.g_total; r.g_total += up256(p.g_bytes());
        }
        if (pass == 0) r.shared_bytes = r.w_total;
      }
      continue;
    }
    r.w_base = off;
    for (Param& p : r.p) { p.w_off = off; off += up256(p.w_bytes()); }
    r.w_span = off - r.w_base;
    r.g_base = off;
    for (Param& p : r.p) { p.g_off = off; off += up256(p.g_bytes()); }
    r.g_span = off - r.g_base;
    r.whole_copies = r.p.size() > 1 && r.g_span <= WHOLE_RECORD_BYTES;
    for (Param& p : r.p)
      if (p.dev_opt) {
        p.dmaster_off = off; off += up256(p.n * 4);
        p.dm_off = off; off += up256(p.n * 4);
        p.dv_off = off; off += up256(p.n * 4);
      }
  }
  c.in_off = off; off += up256(c.in_bytes);
  c.lab_off = off; off += up256(c.lab_bytes);
  c.loss_off = off; off += 256;
  c.misc_off = off; off += up256(c.misc_bytes);
  c.fixed_bytes = off;
  c.cost.resize(c.L);
  // gradients that go to the host after a record's backward and new weights that come back, for records whose
  // weights are resident (a streamed record's are its w_total / g_total; its new weights stay on the host)
  auto host_bytes = [](const Record& r, uint64_t& g, uint64_t& w) {
    g = w = 0;
    if (r.streamed) return;
    for (const Param& p : r.p)
      if (!p.dev_opt) { g += p.g_bytes(); w += p.w_bytes(); }
  };
  for (uint32_t i = 0; i < c.L; ++i) {
    uint64_t hg, hw;
    host_bytes(c.rec[i], hg, hw);
    c.cost[i] = karma_layer_cost{0, 0, 0, c.rec[i].sav_bytes, c.rec[i].out_bytes, c.rec[i].ws_bytes,
                                  c.rec[i].streamed ? c.rec[i].w_total : 0, c.rec[i].streamed ? c.rec[i].g_total : 0,
                                  0, hg, hw};
  }
  {
    uint64_t hg, hw;
    host_bytes(c.rec[c.L], hg, hw);
    c.loss_cost = karma_loss_cost{0, c.rec[c.L].ws_bytes, 0, hg, hw};
  }
  return KARMA_OK;
}

// ------------------------------------------------------------------ C ABI
extern "C" int karma_model_layers(const karma_model_desc* d, uint32_t* n_out) {
  if (!d || !n_out) return KARMA_E_INVAL;
  if (d->kind == KARMA_MODEL_MLP) *n_out = d->n_layers;
  else if (d->kind == KARMA_MODEL_GPT) *n_out = (d->split_blocks ? 2 * d->n_layers : d->n_layers) + 1;
  else if (d->kind == KARMA_MODEL_CNN) *n_out = 1 + d->stage_blocks[0] + d->stage_blocks[1] + d->stage_blocks[2] + d->stage_blocks[3];
  else if (d->kind == KARMA_MODEL_WRN) *n_out = 1 + d->stage_blocks[0] + d->stage_blocks[1] + d->stage_blocks[2];
  else if (d->kind == KARMA_MODEL_UNET) *n_out = 2 * d->n_layers + 1;
  else return KARMA_E_INVAL;
  return KARMA_OK;
}

extern "C" int karma_model_skips(const karma_model_desc* d, karma_skip* skips_out, uint32_t* n_inout) {
  if (!d || !n_inout) return KARMA_E_INVAL;
  std::vector<karma_skip> sk;
  if (d->kind == KARMA_MODEL_UNET) {
    int st = unet_skips(*d, sk);
    if (st) return st;
  }
  if (skips_out) {
    if (*n_inout < sk.size()) { *n_inout = (uint32_t)sk.size(); return KARMA_E_OOM; }
    std::memcpy(skips_out, sk.data(), sk.size() * sizeof(karma_skip));
  }
  *n_inout = (uint32_t)sk.size();
  return KARMA_OK;
}

extern "C" int karma_create(const karma_model_desc* desc, const karma_config* cfg, void* arena_dev,
                            uint64_t arena_bytes, void* stream_compute, void* stream_h2d, void* stream_d2h,
                            karma_ctx** out) {
  if (!desc || !cfg || !arena_dev || !out) return KARMA_E_INVAL;
  if (((uintptr_t)arena_dev & 255) != 0) return KARMA_E_INVAL;
  if (cfg->optimizer != KARMA_OPT_SGD && cfg->optimizer != KARMA_OPT_ADAM && cfg->optimizer != KARMA_OPT_SGD_MOMENTUM)
    return KARMA_E_INVAL;
  if (desc->stream_weights > 2) return KARMA_E_INVAL;
  karma_ctx* c = new (std::nothrow) karma_ctx();
  if (!c) return KARMA_E_HOSTMEM;
  c->desc = *desc;
  c->cfg = *cfg;
  c->arena = (char*)arena_dev;
  c->arena_bytes = arena_bytes;
  c->st[0] = (hipStream_t)stream_compute;
  c->st[1] = (hipStream_t)stream_h2d;
  c->st[2] = (hipStream_t)stream_d2h;
  int st = derive_layout(*c);
  if (st) { delete c; return st; }
  if (c->fixed_bytes >= arena_bytes) { delete c; return KARMA_E_OOM; }
  c->link = karma_link{50000000000ull, 50000000000ull, 10000, 0, 0};
  // host state
  bool ok = true;
  auto pin = [&](void** p, uint64_t bytes) {
    if (!ok) return;
    hipError_t e = hipHostMalloc(p, bytes ? bytes : 256, hipHostMallocDefault);
    if (e != hipSuccess) {
      std::fprintf(stderr, "karma_create: hipHostMalloc(%llu) failed: %s\n", (unsigned long long)bytes, hipGetErrorString(e));
      (void)hipGetLastError();
      ok = false;
    }
  };
  for (Record& r : c->rec) {
    if (!r.streamed) {
      pin((void**)&r.stage_g_all, r.g_span);
      pin((void**)&r.stage_w_all, r.w_span);
      if (ok) { std::memset(r.stage_g_all, 0, r.g_span ? r.g_span : 256); std::memset(r.stage_w_all, 0, r.w_span ? r.w_span : 256); }
      if (ok && r.whole_copies && hipEventCreateWithFlags(&r.grads_ev, hipEventDisableTiming) != hipSuccess) ok = false;
    }
    if (r.streamed) {
      pin((void**)&r.stage_w_all, r.w_total);
      if (desc->stream_weights == 2) {
        // gradients of the weight's element type land in the weights' buffer (same offsets); the others
        // (fp32 gradients of bf16 vectors) get a small buffer of their own
        r.shared_staging = true;
        pin((void**)&r.stage_g_all, r.g_total - r.shared_bytes);
        if (ok) { std::memset(r.stage_w_all, 0, r.w_total); std::memset(r.stage_g_all, 0, r.g_total - r.shared_bytes); }
      } else {
        pin((void**)&r.stage_g_all, r.g_total);
        if (ok) { std::memset(r.stage_w_all, 0, r.w_total); std::memset(r.stage_g_all, 0, r.g_total); }
      }
    }
    for (Param& p : r.p) {
      p.master.assign(p.n, 0.f);
      if (p.dev_opt) {
        // master weights and optimiser state in the fixed region start at zero like the host's
        if (ok && (hipMemset(c->arena + p.dmaster_off, 0, p.n * 4) != hipSuccess || hipMemset(c->arena + p.dm_off, 0, p.n * 4) != hipSuccess ||
                   hipMemset(c->arena + p.dv_off, 0, p.n * 4) != hipSuccess)) {
          (void)hipGetLastError();
          ok = false;
        }
      } else {
        if (cfg->optimizer == KARMA_OPT_ADAM) { p.m.assign(p.n, 0.f); p.v.assign(p.n, 0.f); }
        if (cfg->optimizer == KARMA_OPT_SGD_MOMENTUM) p.m.assign(p.n, 0.f);
      }
      if (r.streamed) {
        if (ok) {
          p.stage_w = r.stage_w_all + p.w_rel;
          if (!r.shared_staging) p.stage_g = r.stage_g_all + p.g_rel;
          else p.stage_g = p.g_rel < r.shared_bytes ? r.stage_w_all + p.g_rel : r.stage_g_all + (p.g_rel - r.shared_bytes);
        }
      } else if (ok) {
        p.stage_g = r.stage_g_all + (p.g_off - r.g_base);
        p.stage_w = r.stage_w_all + (p.w_off - r.w_base);
      }
    }
  }
  pin(&c->stage_in, c->in_bytes);
  pin(&c->stage_lab, c->lab_bytes);
  pin((void**)&c->stage_loss, 256);
  pin(&c->stage_misc, c->misc_bytes);
  for (Record& r : c->rec)
    for (Param& p : r.p) {
      p.chunk_ev.assign((size_t)((p.n + PARAM_CHUNK - 1) / PARAM_CHUNK), nullptr);
      for (auto& e : p.chunk_ev)
        if (ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
          std::fprintf(stderr, "karma_create: hipEventCreate failed\n");
          ok = false;
        }
    }
  if (!ok) { karma_destroy(c); return KARMA_E_HOSTMEM; }
  c->pending_update.assign(c->rec.size(), 0);
  c->update_ns.assign(c->rec.size(), 0);
  if (hipEventCreateWithFlags(&c->weights_uploaded, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&c->program_h2d_done, hipEventDisableTiming) != hipSuccess) {
    karma_destroy(c);
    return KARMA_E_HIP;
  }
  c->pool.reset(new HostPool(cfg->host_threads ? cfg->host_threads : 1));
  *out = c;
  return KARMA_OK;
}

extern "C" void karma_destroy(karma_ctx* c) {
  if (!c) return;
  for (int k = 0; k < 3; ++k) if (c->st[k] || k == 0) (void)hipStreamSynchronize(c->st[k]);
  free_plan_resources(c);
  for (Record& r : c->rec) {
    for (Param& p : r.p)
      for (auto e : p.chunk_ev) if (e) (void)hipEventDestroy(e);
    if (r.grads_ev) (void)hipEventDestroy(r.grads_ev);
    if (r.stage_w_all) (void)hipHostFree(r.stage_w_all);
    if (r.stage_g_all) (void)hipHostFree(r.stage_g_all);
  }
  if (c->stage_in) (void)hipHostFree(c->stage_in);
  if (c->stage_lab) (void)hipHostFree(c->stage_lab);
  if (c->stage_loss) (void)hipHostFree(c->stage_loss);
  if (c->stage_misc) (void)hipHostFree(c->stage_misc);
  for (auto e : c->kev) (void)hipEventDestroy(e);
  if (c->weights_uploaded) (void)hipEventDestroy(c->weights_uploaded);
  if (c->program_h2d_done) (void)hipEventDestroy(c->program_h2d_done);
  delete c;
}

extern "C" const char* karma_last_error(const karma_ctx* c) { return c ? c->err.c_str() : "null context"; }

extern "C" int karma_param_count(const karma_ctx* c, uint32_t layer, uint32_t* n) {
  if (!c || !n || layer >= c->rec.size()) return KARMA_E_INVAL;
  *n = (uint32_t)c->rec[layer].p.size();
  return KARMA_OK;
}

extern "C" int karma_param_size(const karma_ctx* c, uint32_t layer, uint32_t t, uint64_t* n) {
  if (!c || !n || layer >= c->rec.size() || t >= c->rec[layer].p.size()) return KARMA_E_INVAL;
  *n = c->rec[layer].p[t].n;
  return KARMA_OK;
}

extern "C" int karma_set_param(karma_ctx* c, uint32_t layer, uint32_t t, const float* host, uint64_t n) {
  if (!c || !host || layer >= c->rec.size() || t >= c->rec[layer].p.size()) return KARMA_E_INVAL;
  Param& p = c->rec[layer].p[t];
  if (n != p.n) return fail(c, KARMA_E_INVAL, "karma_set_param: element count mismatch");
  int st = finish_all_updates(c);
  if (st) return st;
  std::memcpy(p.master.data(), host, n * sizeof(float));
  if (p.dev_bf16) for (uint64_t i = 0; i < n; ++i) ((uint16_t*)p.stage_w)[i] = f32_to_bf16_rne(host[i]);
  else std::memcpy(p.stage_w, host, n * sizeof(float));
  if (!c->rec[layer].streamed) KARMA_HIP(c, hipMemcpy(c->arena + p.w_off, p.stage_w, p.w_bytes(), hipMemcpyHostToDevice));
  if (p.dev_opt) KARMA_HIP(c, hipMemcpy(c->arena + p.dmaster_off, host, n * sizeof(float), hipMemcpyHostToDevice));
  return KARMA_OK;
}

extern "C" int karma_get_param(karma_ctx* c, uint32_t layer, uint32_t t, float* host, uint64_t n) {
  if (!c || !host || layer >= c->rec.size() || t >= c->rec[layer].p.size()) return KARMA_E_INVAL;
  Param& p = c->rec[layer].p[t];
  if (n != p.n) return fail(c, KARMA_E_INVAL, "karma_get_param: element count mismatch");
  int st = finish_all_updates(c);
  if (st) return st;
  if (p.dev_opt) KARMA_HIP(c, hipMemcpy(p.master.data(), c->arena + p.dmaster_off, n * sizeof(float), hipMemcpyDeviceToHost));
  std::memcpy(host, p.master.data(), n * sizeof(float));
  return KARMA_OK;
}

extern "C" int karma_get_grad(karma_ctx* c, uint32_t layer, uint32_t t, float* host, uint64_t n) {
  if (!c || !host || layer >= c->rec.size() || t >= c->rec[layer].p.size()) return KARMA_E_INVAL;
  Param& p = c->rec[layer].p[t];
  if (n != p.n) return fail(c, KARMA_E_INVAL, "karma_get_grad: element count mismatch");
  if (c->rec[layer].shared_staging)
    return fail(c, KARMA_E_STATE, "karma_get_grad: this record's gradients share the weights' pinned buffer (stream_weights 2)");
  // gradients of streamed weights were copied out by the step itself
  if (!c->rec[layer].streamed) KARMA_HIP(c, hipMemcpy(p.stage_g, c->arena + p.g_off, p.g_bytes(), hipMemcpyDeviceToHost));
  if (p.grad_bf16) for (uint64_t i = 0; i < n; ++i) host[i] = bf16_to_f32(((const uint16_t*)p.stage_g)[i]);
  else std::memcpy(host, p.stage_g, n * sizeof(float));
  return KARMA_OK;
}

extern "C" int karma_get_costs(karma_ctx* c, karma_layer_cost* layers, karma_loss_cost* loss, uint64_t* fixed) {
  if (!c) return KARMA_E_INVAL;
  if (layers) std::memcpy(layers, c->cost.data(), c->L * sizeof(karma_layer_cost));
  if (loss) *loss = c->loss_cost;
  if (fixed) *fixed = c->fixed_bytes;
  return KARMA_OK;
}

extern "C" int karma_set_costs(karma_ctx* c, const karma_layer_cost* layers, const karma_loss_cost* loss,
                               const karma_link* link) {
  if (!c) return KARMA_E_INVAL;
  if (layers)
    for (uint32_t i = 0; i < c->L; ++i) {   // bytes stay the library's own: only times are taken
      c->cost[i].tf_ns = layers[i].tf_ns;
      c->cost[i].tb_ns = layers[i].tb_ns;
      c->cost[i].trc_ns = layers[i].trc_ns;
      c->cost[i].th_ns = layers[i].th_ns;
    }
  if (loss) { c->loss_cost.t_ns = loss->t_ns; c->loss_cost.th_ns = loss->th_ns; }
  if (link) {
    if (!link->bw_h2d || !link->bw_d2h) return KARMA_E_INVAL;
    c->link = *link;
  }
  c->have_times = true;
  return KARMA_OK;
}

extern "C" int karma_refine_host_costs(karma_ctx* c) {
  if (!c) return KARMA_E_INVAL;
  int st = finish_all_updates(c);   // updates a step left pending are timed when they run
  if (st) return st;
  bool any = false;
  for (uint32_t r = 0; r < c->update_ns.size(); ++r) {
    if (c->update_ns[r] <= 0) continue;
    any = true;
    if (r < c->L) c->cost[r].th_ns = c->update_ns[r];
    else c->loss_cost.th_ns = c->update_ns[r];
  }
  return any ? KARMA_OK : fail(c, KARMA_E_STATE, "karma_refine_host_costs: no host update has run yet");
}

extern "C" int karma_plan(karma_ctx* c, uint64_t budget, uint8_t* actions_out, uint8_t* weights_kept_out,
                          karma_plan_summary* summary_out) {
  if (!c) return KARMA_E_INVAL;
  if (budget > c->arena_bytes) return fail(c, KARMA_E_OOM, "budget exceeds the arena handed to karma_create");
  Problem P{c->cost.data(), c->L, c->link, c->loss_cost, budget, c->fixed_bytes, c->skips.data(), (uint32_t)c->skips.size()};
  std::vector<uint8_t> a, kw;
  karma_plan_summary s;
  if (!plan(P, a, kw, &s)) return fail(c, KARMA_E_BUDGET, "no assignment fits the budget");
  int st = install_plan(c, budget, a, kw);
  if (st) return st;
  if (actions_out) std::memcpy(actions_out, a.data(), c->L);
  if (weights_kept_out) std::memcpy(weights_kept_out, kw.data(), c->L);
  if (summary_out) *summary_out = c->summary;
  return KARMA_OK;
}

extern "C" int karma_plan_grouped(karma_ctx* c, uint64_t budget, uint32_t max_group, uint8_t* actions_out,
                                  uint8_t* weights_kept_out, karma_plan_summary* summary_out, uint32_t* group_out) {
  if (!c || !max_group) return KARMA_E_INVAL;
  if (budget > c->arena_bytes) return fail(c, KARMA_E_OOM, "budget exceeds the arena handed to karma_create");
  Problem P{c->cost.data(), c->L, c->link, c->loss_cost, budget, c->fixed_bytes, c->skips.data(), (uint32_t)c->skips.size()};
  std::vector<uint8_t> a, kw;
  karma_plan_summary s;
  uint32_t g = 1;
  if (!plan_grouped(P, max_group, a, kw, &s, &g)) return fail(c, KARMA_E_BUDGET, "no assignment fits the budget");
  int st = install_plan(c, budget, a, kw);
  if (st) return st;
  if (actions_out) std::memcpy(actions_out, a.data(), c->L);
  if (weights_kept_out) std::memcpy(weights_kept_out, kw.data(), c->L);
  if (summary_out) *summary_out = c->summary;
  if (group_out) *group_out = g;
  return KARMA_OK;
}

extern "C" int karma_set_plan(karma_ctx* c, uint64_t budget, const uint8_t* actions, const uint8_t* weights_kept,
                              karma_plan_summary* summary_out) {
  if (!c || !actions) return KARMA_E_INVAL;
  std::vector<uint8_t> a(actions, actions + c->L);
  std::vector<uint8_t> kw(c->L, 0);
  if (weights_kept) kw.assign(weights_kept, weights_kept + c->L);
  int st = install_plan(c, budget, a, kw);
  if (st) return st;
  if (summary_out) *summary_out = c->summary;
  return KARMA_OK;
}

extern "C" int karma_plan_string(karma_ctx* c, char* buf, size_t len) {
  if (!c || !buf) return KARMA_E_INVAL;
  if (!c->planned) return fail(c, KARMA_E_STATE, "no plan");
  std::string s = stage_string(c->ops.data(), (uint32_t)c->ops.size());
  if (s.size() + 1 > len) return KARMA_E_OOM;
  std::memcpy(buf, s.c_str(), s.size() + 1);
  return KARMA_OK;
}

extern "C" int karma_step(karma_ctx* c, const void* in, const void* lab, uint32_t flags, float* loss_out) {
  if (!c || (in == nullptr) != (lab == nullptr)) return KARMA_E_INVAL;
  const int st = run_step(c, in, lab, flags, loss_out, (flags & KARMA_STEP_PROFILE) != 0);
  if (st == KARMA_OK && in) c->inputs_resident = true;
  return st;
}

extern "C" int karma_finish_updates(karma_ctx* c) {
  if (!c) return KARMA_E_INVAL;
  return finish_all_updates(c);
}

extern "C" int karma_get_stats(karma_ctx* c, karma_step_stats* out) {
  if (!c || !out) return KARMA_E_INVAL;
  *out = c->stats;
  return KARMA_OK;
}

extern "C" int karma_get_gemm_stats(karma_ctx* c, uint64_t* launches, double* ms, double* flops) {
  if (!c || !launches || !ms || !flops) return KARMA_E_INVAL;
  *launches = c->gemm_launches;
  *ms = c->gemm_ms;
  *flops = c->gemm_flops;
  return KARMA_OK;
}

extern "C" int karma_get_op_times(karma_ctx* c, karma_op* ops_out, float* ms_out, uint32_t* n_inout) {
  if (!c || !n_inout) return KARMA_E_INVAL;
  if (!c->planned) return fail(c, KARMA_E_STATE, "no plan");
  uint32_t n = (uint32_t)c->ops.size();
  if (*n_inout < n) { *n_inout = n; return KARMA_E_OOM; }
  if (ops_out) std::memcpy(ops_out, c->ops.data(), n * sizeof(karma_op));
  if (ms_out) std::memcpy(ms_out, c->op_ms.data(), n * sizeof(float));
  *n_inout = n;
  return KARMA_OK;
}

extern "C" int karma_get_op_starts(karma_ctx* c, float* start_ms_out, uint32_t* n_inout) {
  if (!c || !n_inout) return KARMA_E_INVAL;
  if (!c->planned) return fail(c, KARMA_E_STATE, "no plan");
  uint32_t n = (uint32_t)c->op_start_ms.size();
  if (*n_inout < n) { *n_inout = n; return KARMA_E_OOM; }
  if (start_ms_out) std::memcpy(start_ms_out, c->op_start_ms.data(), n * sizeof(float));
  *n_inout = n;
  return KARMA_OK;
}

// Profiles the model once (Sec. III-D): an in-core step with events around every op gives
// per-layer times; pinned copies of both directions give the link figures.
extern "C" int karma_measure(karma_ctx* c, uint32_t reps, karma_link* link_out) {
  if (!c) return KARMA_E_INVAL;
  if (!reps) reps = 3;
  std::vector<uint8_t> keep(c->L, KARMA_KEEP), kw(c->L, 0);
  for (uint32_t i = 0; i < c->L; ++i) kw[i] = c->rec[i].streamed ? 1 : 0;
  int st = install_plan(c, c->arena_bytes, keep, kw);
  if (st) return st;
  c->inputs_resident = false;   // the profiling steps below replace the caller's batch
  // inputs: whatever the staging buffers hold (zeros on a fresh context are valid ids / values)
  std::vector<char> in(c->in_bytes ? c->in_bytes : 1, 0), lab(c->lab_bytes ? c->lab_bytes : 1, 0);
  if (c->desc.kind == KARMA_MODEL_GPT) {   // spread token ids over the vocabulary, as real batches do
    int32_t* ids = (int32_t*)in.data();
    int32_t* lb = (int32_t*)lab.data();
    for (uint64_t t = 0; t < c->in_bytes / 4; ++t) {
      ids[t] = (int32_t)((t * 7919u) % c->desc.vocab);
      lb[t] = (int32_t)((t * 104729u + 1) % c->desc.vocab);
    }
  }
  std::vector<std::vector<float>> samples(c->prog.size());
  for (uint32_t r = 0; r < reps + 1; ++r) {
    float loss;
    st = run_step(c, in.data(), lab.data(), 0, &loss, true);
    if (st) return st;
    if (r == 0) continue;   // warm-up
    for (size_t k = 0; k < c->prog.size(); ++k) samples[k].push_back(c->op_ms[k]);
  }
  for (size_t k = 0; k < c->prog.size(); ++k) {
    std::sort(samples[k].begin(), samples[k].end());
    int64_t ns = (int64_t)(samples[k][samples[k].size() / 2] * 1e6);
    if (ns < 1) ns = 1;
    const ProgOp& p = c->prog[k];
    if (p.kind == 'F') { c->cost[p.layer].tf_ns = ns; c->cost[p.layer].trc_ns = ns; }
    else if (p.kind == 'B') c->cost[p.layer].tb_ns = ns;
    else if (p.kind == 'L') c->loss_cost.t_ns = ns;
  }
  // Recompute times: the same step with every record recomputed from its kept input.  Each recompute is then
  // the last of its run and rebuilds the record's internals only (its output still exists as the next
  // record's input), which is what trc prices; inside a run a record is re-run whole and costs tf.
  {
    std::vector<uint8_t> again(c->L, KARMA_RC_KEEP);
    st = install_plan(c, c->arena_bytes, again, kw);
    if (st == KARMA_OK) {
      std::vector<std::vector<float>> rs(c->prog.size());
      for (uint32_t r = 0; r < reps + 1; ++r) {
        float loss;
        st = run_step(c, in.data(), lab.data(), 0, &loss, true);
        if (st) return st;
        if (r == 0) continue;
        for (size_t k = 0; k < c->prog.size(); ++k) rs[k].push_back(c->op_ms[k]);
      }
      for (size_t k = 0; k < c->prog.size(); ++k) {
        const ProgOp& p = c->prog[k];
        if (p.kind != 'R') continue;
        std::sort(rs[k].begin(), rs[k].end());
        int64_t ns = (int64_t)(rs[k][rs[k].size() / 2] * 1e6);
        c->cost[p.layer].trc_ns = std::min<int64_t>(std::max<int64_t>(ns, 1), c->cost[p.layer].tf_ns);
      }
    } else if (st != KARMA_E_BUDGET) {
      return st;
    }
    st = install_plan(c, c->arena_bytes, keep, kw);   // leave the in-core plan installed
    if (st) return st;
  }
  // link: one large and one small pinned copy per direction, on the copy streams
  uint64_t big = std::min<uint64_t>(256ull << 20, (c->arena_bytes - c->fixed_bytes) / 2 / 256 * 256);
  if (big >= (1u << 20)) {
    char* host = nullptr;
    if (hipHostMalloc((void**)&host, big, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return fail(c, KARMA_E_HOSTMEM, "pinned buffer for the link measurement");
    }
    std::memset(host, 0, big);
    hipEvent_t e0, e1;
    KARMA_HIP(c, hipEventCreate(&e0));
    KARMA_HIP(c, hipEventCreate(&e1));
    char* dev = c->act_ptr(0);
    double bw[2] = {0, 0}, lat[2] = {0, 0};
    for (int dir = 0; dir < 2; ++dir) {
      hipStream_t s = c->st[dir == 0 ? 1 : 2];
      for (int pass = 0; pass < 2; ++pass) {
        uint64_t nbytes = pass == 0 ? big : 4096;
        std::vector<float> ms;
        for (uint32_t r = 0; r < reps + 1; ++r) {
          KARMA_HIP(c, hipEventRecord(e0, s));
          if (dir == 0) KARMA_HIP(c, hipMemcpyAsync(dev, host, nbytes, hipMemcpyHostToDevice, s));
          else KARMA_HIP(c, hipMemcpyAsync(host, dev, nbytes, hipMemcpyDeviceToHost, s));
          KARMA_HIP(c, hipEventRecord(e1, s));
          KARMA_HIP(c, hipEventSynchronize(e1));
          float t;
          KARMA_HIP(c, hipEventElapsedTime(&t, e0, e1));
          if (r) ms.push_back(t);
        }
        std::sort(ms.begin(), ms.end());
        double med = ms[ms.size() / 2];
        if (pass == 0) bw[dir] = (double)nbytes / (med * 1e-3);
        else lat[dir] = med * 1e6;
      }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipHostFree(host);
    c->link.bw_h2d = (uint64_t)bw[0];
    c->link.bw_d2h = (uint64_t)bw[1];
    c->link.lat_ns = (int64_t)std::max(lat[0], lat[1]);
  }
  // Host optimiser (Sec. III-G, stage 5) and the link while it runs: the configured update over a scratch
  // parameter tensor on the context's threads, with copies of both directions in flight when the arena has room
  // for them.  Gives the loaded link rates and the update time per parameter, from which each record's th.
  {
    const size_t n = (size_t)16 << 20;
    std::vector<float> w(n, 0.5f), m1(n, 0.f), m2(n, 0.f);
    std::vector<uint16_t> g(n, 0x3c00), out(n);
    const karma_config& cf = c->cfg;
    auto one_pass = [&](uint64_t step) {
      c->pool->parallel_for(n, [&](size_t lo, size_t hi) {
        if (cf.optimizer == KARMA_OPT_ADAM)
          adam_update(w.data() + lo, m1.data() + lo, m2.data() + lo, g.data() + lo, true, hi - lo, cf.lr, cf.beta1, cf.beta2,
                      cf.eps, step, out.data() + lo, true);
        else if (cf.optimizer == KARMA_OPT_SGD_MOMENTUM)
          sgd_momentum_update(w.data() + lo, m1.data() + lo, g.data() + lo, true, hi - lo, cf.lr, cf.beta1, out.data() + lo, true);
        else
          sgd_update(w.data() + lo, g.data() + lo, true, hi - lo, cf.lr, out.data() + lo, true);
      });
    };
    one_pass(1);   // first touch
    char *h_in = nullptr, *h_out = nullptr;
    hipEvent_t a0 = nullptr, a1 = nullptr, b0 = nullptr, b1 = nullptr;
    bool copies = big >= (1u << 20);
    if (copies && (hipHostMalloc((void**)&h_in, big, hipHostMallocDefault) != hipSuccess ||
                   hipHostMalloc((void**)&h_out, big, hipHostMallocDefault) != hipSuccess)) {
      (void)hipGetLastError();
      if (h_in) (void)hipHostFree(h_in);
      h_in = h_out = nullptr;
      copies = false;
    }
    const int rounds = 8;
    if (copies) {
      std::memset(h_in, 0, big);
      std::memset(h_out, 0, big);
      KARMA_HIP(c, hipEventCreate(&a0)); KARMA_HIP(c, hipEventCreate(&a1));
      KARMA_HIP(c, hipEventCreate(&b0)); KARMA_HIP(c, hipEventCreate(&b1));
      char* dev = c->act_ptr(0);
      KARMA_HIP(c, hipEventRecord(a0, c->st[1]));
      KARMA_HIP(c, hipEventRecord(b0, c->st[2]));
      for (int r = 0; r < rounds; ++r) {
        KARMA_HIP(c, hipMemcpyAsync(dev, h_in, big, hipMemcpyHostToDevice, c->st[1]));
        KARMA_HIP(c, hipMemcpyAsync(h_out, dev + big, big, hipMemcpyDeviceToHost, c->st[2]));
      }
      KARMA_HIP(c, hipEventRecord(a1, c->st[1]));
      KARMA_HIP(c, hipEventRecord(b1, c->st[2]));
    }
    uint64_t passes = 0;
    const double t0 = now_ms();
    for (;;) {
      one_pass(2 + passes);
      ++passes;
      if (!copies) { if (passes >= 4) break; continue; }
      const bool in_done = hipEventQuery(a1) == hipSuccess, out_done = hipEventQuery(b1) == hipSuccess;
      (void)hipGetLastError();
      if (in_done || out_done) break;   // once one direction is through, the other is no longer loaded
    }
    const double host_ms = now_ms() - t0;
    const double ns_per_param = host_ms * 1e6 / ((double)passes * (double)n);
    if (copies) {
      KARMA_HIP(c, hipEventSynchronize(a1));
      KARMA_HIP(c, hipEventSynchronize(b1));
      float t_in_ms = 0.f, t_out_ms = 0.f;
      KARMA_HIP(c, hipEventElapsedTime(&t_in_ms, a0, a1));
      KARMA_HIP(c, hipEventElapsedTime(&t_out_ms, b0, b1));
      // never above the idle figure (the tail of the slower direction runs unloaded)
      c->link.bw_h2d_loaded = std::min<uint64_t>(c->link.bw_h2d, (uint64_t)((double)rounds * big / (t_in_ms * 1e-3)));
      c->link.bw_d2h_loaded = std::min<uint64_t>(c->link.bw_d2h, (uint64_t)((double)rounds * big / (t_out_ms * 1e-3)));
      (void)hipEventDestroy(a0); (void)hipEventDestroy(a1); (void)hipEventDestroy(b0); (void)hipEventDestroy(b1);
      (void)hipHostFree(h_in);
      (void)hipHostFree(h_out);
    }
    auto th_of = [&](const Record& r) {
      uint64_t params = 0;
      for (const Param& p : r.p)
        if (!p.dev_opt) params += p.n;
      return (int64_t)((double)params * ns_per_param);
    };
    for (uint32_t i = 0; i < c->L; ++i) c->cost[i].th_ns = th_of(c->rec[i]);
    c->loss_cost.th_ns = th_of(c->rec[c->L]);
  }
  c->have_times = true;
  if (link_out) *link_out = c->link;
  return KARMA_OK;
}
