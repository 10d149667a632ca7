"""ctypes binding of include/karma.h: same names, argument marshalling only.

The library must have been built (paper_2008_11421_amd/build.py); there is no fallback:
a missing library raises ImportError-like OSError on first use."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkarma.so")

KEEP, SWAP, RC_KEEP, RC_SWAP, RC_CHAIN = range(5)
OK, E_INVAL, E_BUDGET, E_OOM, E_HIP, E_STATE, E_HOSTMEM = 0, -1, -2, -3, -4, -5, -6
MODEL_MLP, MODEL_GPT, MODEL_CNN, MODEL_WRN, MODEL_UNET = 1, 2, 3, 4, 5
OPT_SGD, OPT_ADAM, OPT_SGD_MOMENTUM = 1, 2, 3
STEP_APPLY_OPTIMIZER = 1
STEP_PROFILE = 2
STEP_KERNEL_TIMES = 4
GEMM_A_STRIDED, GEMM_B_STRIDED, GEMM_OUT_F32, GEMM_ACCUMULATE = 1, 2, 4, 8
GEMM_GELU_FWD, GEMM_GELU_BWD = 1, 2


class LayerCost(C.Structure):
    _fields_ = [("tf_ns", C.c_int64), ("tb_ns", C.c_int64), ("trc_ns", C.c_int64),
                ("sav_bytes", C.c_uint64), ("out_bytes", C.c_uint64), ("ws_bytes", C.c_uint64),
                ("w_bytes", C.c_uint64), ("g_bytes", C.c_uint64),
                ("th_ns", C.c_int64), ("hg_bytes", C.c_uint64), ("hw_bytes", C.c_uint64)]


class Link(C.Structure):
    _fields_ = [("bw_h2d", C.c_uint64), ("bw_d2h", C.c_uint64), ("lat_ns", C.c_int64),
                ("bw_h2d_loaded", C.c_uint64), ("bw_d2h_loaded", C.c_uint64)]


class LossCost(C.Structure):
    _fields_ = [("t_ns", C.c_int64), ("ws_bytes", C.c_uint64), ("th_ns", C.c_int64), ("hg_bytes", C.c_uint64),
                ("hw_bytes", C.c_uint64)]


class PlanSummary(C.Structure):
    _fields_ = [("makespan_ns", C.c_int64), ("stall_ns", C.c_int64), ("busy_ns", C.c_int64),
                ("recompute_ns", C.c_int64), ("peak_bytes", C.c_uint64), ("bytes_d2h", C.c_uint64),
                ("bytes_h2d", C.c_uint64), ("host_busy_ns", C.c_int64), ("host_end_ns", C.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class Op(C.Structure):
    _fields_ = [("kind", C.c_uint8), ("layer", C.c_uint32), ("start_ns", C.c_int64), ("end_ns", C.c_int64),
                ("off", C.c_int64 * 3)]


class ModelDesc(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("n_layers", C.c_uint32), ("width", C.c_uint32), ("batch", C.c_uint32),
                ("seq", C.c_uint32), ("n_heads", C.c_uint32), ("ffn", C.c_uint32), ("vocab", C.c_uint32),
                ("stream_weights", C.c_uint32), ("stage_blocks", C.c_uint32 * 4), ("split_blocks", C.c_uint32)]


class ConvShape(C.Structure):
    _fields_ = [("n", C.c_uint32), ("h", C.c_uint32), ("w", C.c_uint32), ("c_in", C.c_uint32), ("c_out", C.c_uint32),
                ("r", C.c_uint32), ("s", C.c_uint32), ("stride", C.c_uint32), ("pad", C.c_uint32)]


class Config(C.Structure):
    _fields_ = [("optimizer", C.c_uint32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("host_threads", C.c_uint32), ("device_update_first", C.c_uint32)]


class StepStats(C.Structure):
    _fields_ = [("step_ms", C.c_double), ("compute_busy_ms", C.c_double), ("d2h_ms", C.c_double),
                ("h2d_ms", C.c_double), ("bytes_d2h", C.c_uint64), ("bytes_h2d", C.c_uint64),
                ("arena_peak_bytes", C.c_uint64), ("host_opt_ms", C.c_double), ("updates_deferred", C.c_uint64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class KarmaError(RuntimeError):
    def __init__(self, status, where, detail=""):
        super().__init__("%s failed with status %d %s" % (where, status, detail))
        self.status = status


_lib = None


def lib():
    """Loads libkarma.so (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("libkarma.so is not built: run `python -m paper_2008_11421_amd.build` "
                          "(there is no CPU fallback)")
        # torch ships its own HIP runtime: load it first so that the library binds to the same
        # one (two runtimes in a process do not share allocations)
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        _lib.karma_last_error.restype = C.c_char_p
        _lib.karma_last_error.argtypes = [C.c_void_p]
        _lib.karma_destroy.restype = None
        _lib.karma_destroy.argtypes = [C.c_void_p]
    return _lib


def _layers_array(layers):
    arr = (LayerCost * len(layers))()
    for k, l in enumerate(layers):
        arr[k] = l if isinstance(l, LayerCost) else LayerCost(*[int(v) for v in l])
    return arr


def _check(st, where, ctx=None):
    if st != 0:
        detail = ""
        if ctx is not None:
            msg = lib().karma_last_error(ctx)
            detail = "(" + msg.decode() + ")" if msg else ""
        raise KarmaError(st, where, detail)


# ------------------------------------------------------------------ pure planner
class Skip(C.Structure):
    _fields_ = [("src", C.c_uint32), ("dst", C.c_uint32)]


def _skips_array(skips):
    arr = (Skip * max(1, len(skips)))()
    for k, (src, dst) in enumerate(skips):
        arr[k] = Skip(int(src), int(dst))
    return arr, C.c_uint32(len(skips))


def karma_simulate(layers, link, loss, budget, fixed, actions, want_ops=False, weights_kept=None, skips=None):
    """layers: sequence of (tf, tb, trc, sav, out, ws[, wb, gb[, th, hg, hw]]); link: (bw_h2d, bw_d2h, lat[,
    bw_h2d_loaded, bw_d2h_loaded]); loss: (t, ws[, th, hg, hw]); skips: (src, dst) pairs -> karma_simulate_graph.
    Returns summary dict (and ops list when asked)."""
    if skips is not None:
        return karma_simulate_graph(layers, link, loss, budget, fixed, skips, actions, want_ops, weights_kept)
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    act = (C.c_uint8 * n)(*actions)
    kept = (C.c_uint8 * n)(*weights_kept) if weights_kept is not None else None
    summ = PlanSummary()
    ops = (Op * (8 * n + 2))() if want_ops else None
    nops = C.c_uint32(8 * n + 2)
    st = lib().karma_simulate(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget), C.c_uint64(fixed),
                              act, kept, C.byref(summ), ops, C.byref(nops))
    _check(st, "karma_simulate")
    if want_ops:
        return summ.as_dict(), [ops[k] for k in range(nops.value)]
    return summ.as_dict()


def karma_simulate_graph(layers, link, loss, budget, fixed, skips, actions, want_ops=False, weights_kept=None):
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    sk, nsk = _skips_array(skips)
    act = (C.c_uint8 * n)(*actions)
    kept = (C.c_uint8 * n)(*weights_kept) if weights_kept is not None else None
    summ = PlanSummary()
    cap = 8 * n + 2 + 2 * len(skips)
    ops = (Op * cap)() if want_ops else None
    nops = C.c_uint32(cap)
    st = lib().karma_simulate_graph(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget), C.c_uint64(fixed),
                                    sk, nsk, act, kept, C.byref(summ), ops, C.byref(nops))
    _check(st, "karma_simulate_graph")
    if want_ops:
        return summ.as_dict(), [ops[k] for k in range(nops.value)]
    return summ.as_dict()


def karma_plan_graph(layers, link, loss, budget, fixed, skips):
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    sk, nsk = _skips_array(skips)
    act = (C.c_uint8 * n)()
    kept = (C.c_uint8 * n)()
    summ = PlanSummary()
    st = lib().karma_plan_graph(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget), C.c_uint64(fixed),
                                sk, nsk, act, kept, C.byref(summ))
    _check(st, "karma_plan_graph")
    res = summ.as_dict()
    res["wres"] = list(kept)
    return list(act), res


def karma_plan_grouped_graph(layers, link, loss, budget, fixed, skips, max_group=8):
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    sk, nsk = _skips_array(skips)
    act = (C.c_uint8 * n)()
    kept = (C.c_uint8 * n)()
    summ = PlanSummary()
    g = C.c_uint32()
    st = lib().karma_plan_grouped_graph(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget),
                                        C.c_uint64(fixed), sk, nsk, C.c_uint32(max_group), act, kept, C.byref(summ),
                                        C.byref(g))
    _check(st, "karma_plan_grouped_graph")
    res = summ.as_dict()
    res["wres"] = list(kept)
    return list(act), res, g.value


def karma_plan_pure(layers, link, loss, budget, fixed):
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    act = (C.c_uint8 * n)()
    kept = (C.c_uint8 * n)()
    summ = PlanSummary()
    st = lib().karma_plan_pure(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget), C.c_uint64(fixed),
                               act, kept, C.byref(summ))
    _check(st, "karma_plan_pure")
    res = summ.as_dict()
    res["wres"] = list(kept)
    return list(act), res


def karma_plan_grouped_pure(layers, link, loss, budget, fixed, max_group=8):
    """Planner that also chooses the block granularity: (actions, summary incl. "wres", group size)."""
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    act = (C.c_uint8 * n)()
    kept = (C.c_uint8 * n)()
    summ = PlanSummary()
    g = C.c_uint32()
    st = lib().karma_plan_grouped_pure(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget), C.c_uint64(fixed),
                                       C.c_uint32(max_group), act, kept, C.byref(summ), C.byref(g))
    _check(st, "karma_plan_grouped_pure")
    res = summ.as_dict()
    res["wres"] = list(kept)
    return list(act), res, g.value


class DeviceRates(C.Structure):
    _fields_ = [("matrix_ops_per_s", C.c_uint64), ("other_ops_per_s", C.c_uint64)]


def _model_desc(desc):
    if isinstance(desc, ModelDesc):
        return desc
    desc = dict(desc)
    if "stage_blocks" in desc:
        desc["stage_blocks"] = (C.c_uint32 * 4)(*desc["stage_blocks"])
    return ModelDesc(**desc)


def karma_model_costs(desc, matrix_ops_per_s, other_ops_per_s):
    """Analytic cost records of a model (no GPU): (layers as 8-tuples, (loss t_ns, loss ws_bytes), fixed bytes)."""
    d = _model_desc(desc)
    n = C.c_uint32()
    _check(lib().karma_model_layers(C.byref(d), C.byref(n)), "karma_model_layers")
    arr = (LayerCost * n.value)()
    rates = DeviceRates(int(matrix_ops_per_s), int(other_ops_per_s))
    loss = LossCost()
    fixed = C.c_uint64()
    _check(lib().karma_model_costs(C.byref(d), C.byref(rates), arr, C.byref(n), C.byref(loss), C.byref(fixed)),
           "karma_model_costs")
    layers = [(a.tf_ns, a.tb_ns, a.trc_ns, a.sav_bytes, a.out_bytes, a.ws_bytes, a.w_bytes, a.g_bytes) for a in arr[:n.value]]
    return layers, (loss.t_ns, loss.ws_bytes), fixed.value


def karma_model_skips(desc):
    """Connections between non-consecutive records of a model: [(src, dst), ...] (empty for most kinds)."""
    d = _model_desc(desc)
    n = C.c_uint32(0)
    _check(lib().karma_model_skips(C.byref(d), None, C.byref(n)), "karma_model_skips")
    arr = (Skip * max(1, n.value))()
    _check(lib().karma_model_skips(C.byref(d), arr, C.byref(n)), "karma_model_skips")
    return [(arr[k].src, arr[k].dst) for k in range(n.value)]


def karma_stage_string(ops):
    arr = (Op * len(ops))(*ops)
    buf = C.create_string_buffer(64 * len(ops) + 64)
    _check(lib().karma_stage_string(arr, C.c_uint32(len(ops)), buf, C.c_size_t(len(buf))), "karma_stage_string")
    return buf.value.decode()


# ------------------------------------------------------------------ context
class Context:
    """One model instance.  torch supplies the device slab and the three streams; every
    method is the C entry point of the same name with numpy marshalling."""

    def __init__(self, desc, cfg, arena_bytes, device="cuda:0"):
        import torch
        self.torch = torch
        self.desc = _model_desc(desc)
        self.cfg = cfg if isinstance(cfg, Config) else Config(**cfg)
        self.device = torch.device(device)
        self.arena = torch.empty(int(arena_bytes), dtype=torch.uint8, device=self.device)
        assert self.arena.data_ptr() % 256 == 0
        self.streams = [torch.cuda.Stream(device=self.device) for _ in range(3)]
        self.ctx = C.c_void_p()
        n = C.c_uint32()
        _check(lib().karma_model_layers(C.byref(self.desc), C.byref(n)), "karma_model_layers")
        self.n_layers = n.value
        with torch.cuda.device(self.device):
            st = lib().karma_create(C.byref(self.desc), C.byref(self.cfg), C.c_void_p(self.arena.data_ptr()),
                                    C.c_uint64(self.arena.numel()),
                                    C.c_void_p(self.streams[0].cuda_stream), C.c_void_p(self.streams[1].cuda_stream),
                                    C.c_void_p(self.streams[2].cuda_stream), C.byref(self.ctx))
        _check(st, "karma_create")

    def close(self):
        if self.ctx:
            lib().karma_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, st, where):
        _check(st, where, self.ctx)

    def karma_param_count(self, layer):
        n = C.c_uint32()
        self._chk(lib().karma_param_count(self.ctx, C.c_uint32(layer), C.byref(n)), "karma_param_count")
        return n.value

    def karma_param_size(self, layer, tensor):
        n = C.c_uint64()
        self._chk(lib().karma_param_size(self.ctx, C.c_uint32(layer), C.c_uint32(tensor), C.byref(n)), "karma_param_size")
        return n.value

    def karma_set_param(self, layer, tensor, values):
        a = np.ascontiguousarray(values, dtype=np.float32).reshape(-1)
        self._chk(lib().karma_set_param(self.ctx, C.c_uint32(layer), C.c_uint32(tensor),
                                        a.ctypes.data_as(C.POINTER(C.c_float)), C.c_uint64(a.size)), "karma_set_param")

    def _get(self, fn, name, layer, tensor):
        n = self.karma_param_size(layer, tensor)
        out = np.empty(n, dtype=np.float32)
        self._chk(fn(self.ctx, C.c_uint32(layer), C.c_uint32(tensor), out.ctypes.data_as(C.POINTER(C.c_float)),
                     C.c_uint64(n)), name)
        return out

    def karma_get_param(self, layer, tensor):
        return self._get(lib().karma_get_param, "karma_get_param", layer, tensor)

    def karma_get_grad(self, layer, tensor):
        return self._get(lib().karma_get_grad, "karma_get_grad", layer, tensor)

    def karma_get_costs(self):
        arr = (LayerCost * self.n_layers)()
        loss = LossCost()
        fixed = C.c_uint64()
        self._chk(lib().karma_get_costs(self.ctx, arr, C.byref(loss), C.byref(fixed)), "karma_get_costs")
        layers = [(l.tf_ns, l.tb_ns, l.trc_ns, l.sav_bytes, l.out_bytes, l.ws_bytes, l.w_bytes, l.g_bytes, l.th_ns,
                   l.hg_bytes, l.hw_bytes) for l in arr]
        return layers, (loss.t_ns, loss.ws_bytes, loss.th_ns, loss.hg_bytes, loss.hw_bytes), fixed.value

    def karma_set_costs(self, layers=None, loss=None, link=None):
        arr = _layers_array(layers) if layers is not None else None
        ls = C.byref(LossCost(*[int(v) for v in loss])) if loss is not None else None
        lk = C.byref(Link(*[int(v) for v in link])) if link is not None else None
        self._chk(lib().karma_set_costs(self.ctx, arr, ls, lk), "karma_set_costs")

    def karma_measure(self, reps=3):
        lk = Link()
        self._chk(lib().karma_measure(self.ctx, C.c_uint32(reps), C.byref(lk)), "karma_measure")
        return (lk.bw_h2d, lk.bw_d2h, lk.lat_ns, lk.bw_h2d_loaded, lk.bw_d2h_loaded)

    def karma_refine_host_costs(self):
        self._chk(lib().karma_refine_host_costs(self.ctx), "karma_refine_host_costs")

    def karma_plan(self, budget):
        act = (C.c_uint8 * self.n_layers)()
        kept = (C.c_uint8 * self.n_layers)()
        summ = PlanSummary()
        self._chk(lib().karma_plan(self.ctx, C.c_uint64(budget), act, kept, C.byref(summ)), "karma_plan")
        res = summ.as_dict()
        res["wres"] = list(kept)
        return list(act), res

    def karma_plan_grouped(self, budget, max_group=8):
        act = (C.c_uint8 * self.n_layers)()
        kept = (C.c_uint8 * self.n_layers)()
        summ = PlanSummary()
        g = C.c_uint32()
        self._chk(lib().karma_plan_grouped(self.ctx, C.c_uint64(int(budget)), C.c_uint32(max_group), act, kept,
                                             C.byref(summ), C.byref(g)), "karma_plan_grouped")
        res = summ.as_dict()
        res["wres"] = list(kept)
        return list(act), res, g.value

    def karma_set_plan(self, budget, actions, weights_kept=None):
        act = (C.c_uint8 * self.n_layers)(*actions)
        kept = (C.c_uint8 * self.n_layers)(*weights_kept) if weights_kept is not None else None
        summ = PlanSummary()
        self._chk(lib().karma_set_plan(self.ctx, C.c_uint64(budget), act, kept, C.byref(summ)), "karma_set_plan")
        return summ.as_dict()

    def karma_plan_string(self):
        buf = C.create_string_buffer(1 << 16)
        self._chk(lib().karma_plan_string(self.ctx, buf, C.c_size_t(len(buf))), "karma_plan_string")
        return buf.value.decode()

    def karma_step(self, inputs, labels, flags=0):
        """inputs/labels: numpy arrays of the dtype the model takes (MLP: fp32 / fp32, GPT:
        int32 ids / int32, CNN: fp32 images [n][h][w][3] / int32 classes).  Returns the loss."""
        loss = C.c_float()
        if inputs is None and labels is None:      # the previous step's batch, still resident in HBM
            with self.torch.cuda.device(self.device):
                st = lib().karma_step(self.ctx, None, None, C.c_uint32(flags), C.byref(loss))
            self._chk(st, "karma_step")
            return loss.value
        a = np.ascontiguousarray(inputs, dtype=np.int32 if self.desc.kind == MODEL_GPT else np.float32)
        b = np.ascontiguousarray(labels, dtype=np.float32 if self.desc.kind == MODEL_MLP else np.int32)
        with self.torch.cuda.device(self.device):
            st = lib().karma_step(self.ctx, C.c_void_p(a.ctypes.data), C.c_void_p(b.ctypes.data), C.c_uint32(flags),
                                  C.byref(loss))
        self._chk(st, "karma_step")
        return loss.value

    def karma_finish_updates(self):
        self._chk(lib().karma_finish_updates(self.ctx), "karma_finish_updates")

    def karma_get_stats(self):
        s = StepStats()
        self._chk(lib().karma_get_stats(self.ctx, C.byref(s)), "karma_get_stats")
        return s.as_dict()

    def karma_get_gemm_stats(self):
        n, ms, fl = C.c_uint64(), C.c_double(), C.c_double()
        self._chk(lib().karma_get_gemm_stats(self.ctx, C.byref(n), C.byref(ms), C.byref(fl)), "karma_get_gemm_stats")
        return n.value, ms.value, fl.value

    def karma_get_op_times(self):
        n = C.c_uint32(10 * self.n_layers + 2)
        ops = (Op * n.value)()
        ms = (C.c_float * n.value)()
        self._chk(lib().karma_get_op_times(self.ctx, ops, ms, C.byref(n)), "karma_get_op_times")
        return [(chr(ops[k].kind), ops[k].layer, ops[k].start_ns, ops[k].end_ns, ms[k]) for k in range(n.value)]

    def karma_get_op_starts(self):
        n = C.c_uint32(10 * self.n_layers + 2)
        starts = (C.c_float * n.value)()
        self._chk(lib().karma_get_op_starts(self.ctx, starts, C.byref(n)), "karma_get_op_starts")
        return [starts[k] for k in range(n.value)]
