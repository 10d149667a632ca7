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
MODEL_MLP, MODEL_GPT = 1, 2
OPT_SGD, OPT_ADAM = 1, 2
STEP_APPLY_OPTIMIZER = 1


class LayerCost(C.Structure):
    _fields_ = [("tf_ns", C.c_int64), ("tb_ns", C.c_int64), ("trc_ns", C.c_int64),
                ("sav_bytes", C.c_uint64), ("out_bytes", C.c_uint64), ("ws_bytes", C.c_uint64)]


class Link(C.Structure):
    _fields_ = [("bw_h2d", C.c_uint64), ("bw_d2h", C.c_uint64), ("lat_ns", C.c_int64)]


class LossCost(C.Structure):
    _fields_ = [("t_ns", C.c_int64), ("ws_bytes", C.c_uint64)]


class PlanSummary(C.Structure):
    _fields_ = [("makespan_ns", C.c_int64), ("stall_ns", C.c_int64), ("busy_ns", C.c_int64),
                ("recompute_ns", C.c_int64), ("peak_bytes", C.c_uint64), ("bytes_d2h", C.c_uint64),
                ("bytes_h2d", C.c_uint64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class Op(C.Structure):
    _fields_ = [("kind", C.c_uint8), ("layer", C.c_uint32), ("start_ns", C.c_int64), ("end_ns", C.c_int64),
                ("off", C.c_int64 * 3)]


class ModelDesc(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("n_layers", C.c_uint32), ("width", C.c_uint32), ("batch", C.c_uint32),
                ("seq", C.c_uint32), ("n_heads", C.c_uint32), ("ffn", C.c_uint32), ("vocab", C.c_uint32)]


class Config(C.Structure):
    _fields_ = [("optimizer", C.c_uint32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("host_threads", C.c_uint32)]


class StepStats(C.Structure):
    _fields_ = [("step_ms", C.c_double), ("compute_busy_ms", C.c_double), ("d2h_ms", C.c_double),
                ("h2d_ms", C.c_double), ("bytes_d2h", C.c_uint64), ("bytes_h2d", C.c_uint64),
                ("arena_peak_bytes", C.c_uint64), ("host_opt_ms", C.c_double)]

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
        _lib = C.CDLL(LIB_PATH)
        if hasattr(_lib, "karma_last_error"):
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
def karma_simulate(layers, link, loss, budget, fixed, actions, want_ops=False):
    """layers: sequence of (tf, tb, trc, sav, out, ws); link: (bw_h2d, bw_d2h, lat);
    loss: (t, ws).  Returns summary dict (and ops list when asked)."""
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    act = (C.c_uint8 * n)(*actions)
    summ = PlanSummary()
    ops = (Op * (6 * n + 2))() if want_ops else None
    nops = C.c_uint32(6 * n + 2)
    st = lib().karma_simulate(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget), C.c_uint64(fixed),
                              act, C.byref(summ), ops, C.byref(nops))
    _check(st, "karma_simulate")
    if want_ops:
        return summ.as_dict(), [ops[k] for k in range(nops.value)]
    return summ.as_dict()


def karma_plan_pure(layers, link, loss, budget, fixed):
    n = len(layers)
    arr = _layers_array(layers)
    lk, ls = Link(*[int(v) for v in link]), LossCost(*[int(v) for v in loss])
    act = (C.c_uint8 * n)()
    summ = PlanSummary()
    st = lib().karma_plan_pure(arr, C.c_uint32(n), C.byref(lk), C.byref(ls), C.c_uint64(budget), C.c_uint64(fixed),
                               act, C.byref(summ))
    _check(st, "karma_plan_pure")
    return list(act), summ.as_dict()


def karma_stage_string(ops):
    arr = (Op * len(ops))(*ops)
    buf = C.create_string_buffer(64 * len(ops) + 64)
    _check(lib().karma_stage_string(arr, C.c_uint32(len(ops)), buf, C.c_size_t(len(buf))), "karma_stage_string")
    return buf.value.decode()
