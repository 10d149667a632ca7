"""The host optimiser's update loops (the CPU-side weight update of the out-of-core step) through
their C entry point, against the oracle's fp64 formulas, in both vector builds.  CPU only."""
import ctypes as C

import numpy as np
import pytest

import paper_2008_11421_amd as K
from oracle import nn
import synth_inputs as si

N = 4096 * 5 + 37          # several vector blocks and a ragged tail


def f32(x):
    """The hyper-parameters reach the library as C floats: the oracle gets the same rounded values."""
    return float(np.float32(x))


def fptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def run(opt, w, m, v, g, g_bf16, step, out_bf16, narrow, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8):
    w, m, v = w.copy(), m.copy(), v.copy()
    if g_bf16:
        gb = (nn.bf16_round(g).view(np.uint32) >> 16).astype(np.uint16)
        gp = gb.ctypes.data_as(C.c_void_p)
    else:
        gb = g.astype(np.float32)
        gp = gb.ctypes.data_as(C.c_void_p)
    out = np.zeros(len(w), dtype=np.uint16 if out_bf16 else np.float32)
    st = K.lib().karma_host_update(C.c_uint32(opt), fptr(w), fptr(m), fptr(v), gp, C.c_uint32(int(g_bf16)),
                                   C.c_uint64(len(w)), C.c_float(lr), C.c_float(b1), C.c_float(b2), C.c_float(eps),
                                   C.c_uint64(step), out.ctypes.data_as(C.c_void_p), C.c_uint32(int(out_bf16)),
                                   C.c_uint32(int(narrow)))
    assert st == K.OK
    return w, m, v, out


@pytest.fixture(scope="module")
def data():
    w = si.normal(71, (N,), 0.5).astype(np.float32)
    m = si.normal(72, (N,), 0.01).astype(np.float32)
    v = (si.normal(73, (N,), 0.01) ** 2).astype(np.float32)
    g = si.normal(74, (N,), 0.02).astype(np.float32)
    return w, m, v, g


@pytest.mark.parametrize("g_bf16", [False, True])
@pytest.mark.parametrize("out_bf16", [False, True])
def test_adam_against_oracle_and_both_vector_widths(data, g_bf16, out_bf16):
    w, m, v, g = data
    gg = nn.bf16_round(g) if g_bf16 else g
    ref_w, ref_m, ref_v = nn.adam_update(w.astype(np.float64), m.astype(np.float64), v.astype(np.float64),
                                         gg.astype(np.float64), 3, f32(1e-3), f32(0.9), f32(0.999), f32(1e-8))
    res = [run(K.OPT_ADAM, w, m, v, g, g_bf16, 3, out_bf16, narrow) for narrow in (False, True)]
    for w1, m1, v1, out in res:
        # fp32 arithmetic against the fp64 formulas: a few ulps
        assert np.all(np.abs(m1 - ref_m) <= 3e-7 * (np.abs(m) + np.abs(gg)) + 1e-12)
        assert np.all(np.abs(v1 - ref_v) <= 3e-7 * (np.abs(v) + gg.astype(np.float64) ** 2) + 1e-16)
        assert np.max(np.abs(w1 - ref_w)) <= 1e-3 * 1e-5 + 2e-7 * np.max(np.abs(ref_w))
        if out_bf16:   # the device copy is the master weight rounded to nearest even
            want = (nn.bf16_round(w1).view(np.uint32) >> 16).astype(np.uint16)
            assert np.array_equal(out, want)
        else:
            assert np.array_equal(out, w1)
    # the AVX2 and the AVX-512 build do the same operations per element: identical bits
    for a, b in zip(res[0], res[1]):
        assert np.array_equal(a, b)


def test_sgd_and_momentum(data):
    w, m, _, g = data
    for narrow in (False, True):
        w1, _, _, out = run(K.OPT_SGD, w, m, m, g, False, 1, False, narrow, lr=0.05)
        assert np.allclose(w1, nn.sgd_update(w.astype(np.float64), g.astype(np.float64), f32(0.05)), rtol=2e-7, atol=1e-9)
        assert np.array_equal(out, w1)
        w2, buf, _, _ = run(K.OPT_SGD_MOMENTUM, w, m, m, g, True, 1, True, narrow, lr=0.05, b1=0.9)
        rw, rbuf = nn.sgd_momentum_update(w.astype(np.float64), m.astype(np.float64), nn.bf16_round(g).astype(np.float64),
                                          f32(0.05), f32(0.9))
        assert np.all(np.abs(buf - rbuf) <= 3e-7 * (np.abs(m) + np.abs(g)) + 1e-12) and np.allclose(w2, rw, rtol=3e-7, atol=1e-8)


def test_first_adam_step_moves_every_weight_by_lr(data):
    """Closed form: from zero moments the bias-corrected first step is lr * sign(g) up to eps."""
    w, _, _, g = data
    z = np.zeros_like(w)
    w1, _, _, _ = run(K.OPT_ADAM, w, z, z, g, False, 1, False, False, lr=1e-2)
    big = np.abs(g) > 1e-4
    assert np.allclose((w - w1)[big], 1e-2 * np.sign(g)[big], rtol=1e-3)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("opt", ["sgd", "momentum", "adam"])
def test_update_in_place_of_the_gradient_buffer(data, opt, bf16):
    """out == grad (one element type): every gradient is replaced by its new weight; results equal, bit for bit,
    those of the update into a separate buffer, in both vector builds."""
    w, m, v, g = data
    kind = {"sgd": K.OPT_SGD, "momentum": K.OPT_SGD_MOMENTUM, "adam": K.OPT_ADAM}[opt]
    for narrow in (False, True):
        w0, m0, v0, out0 = run(kind, w, m, v, g, bf16, 2, bf16, narrow)
        w1, m1, v1 = w.copy(), m.copy(), v.copy()
        buf = (nn.bf16_round(g).view(np.uint32) >> 16).astype(np.uint16) if bf16 else g.astype(np.float32)
        bp = buf.ctypes.data_as(C.c_void_p)
        st = K.lib().karma_host_update(C.c_uint32(kind), fptr(w1), fptr(m1), fptr(v1), bp, C.c_uint32(int(bf16)),
                                       C.c_uint64(len(w1)), C.c_float(1e-3), C.c_float(0.9), C.c_float(0.999), C.c_float(1e-8),
                                       C.c_uint64(2), bp, C.c_uint32(int(bf16)), C.c_uint32(int(narrow)))
        assert st == K.OK
        assert np.array_equal(buf, out0) and np.array_equal(w1, w0)
        if opt != "sgd":
            assert np.array_equal(m1, m0)
        if opt == "adam":
            assert np.array_equal(v1, v0)
    # differing element types cannot share a buffer
    st = K.lib().karma_host_update(C.c_uint32(K.OPT_SGD), fptr(w.copy()), None, None, bp, C.c_uint32(1), C.c_uint64(8),
                                   C.c_float(1e-3), C.c_float(0.9), C.c_float(0.999), C.c_float(1e-8), C.c_uint64(1), bp,
                                   C.c_uint32(0), C.c_uint32(0))
    assert st == K.E_INVAL


def test_rejects_bad_arguments(data):
    w, m, v, g = data
    lib = K.lib()
    out = np.zeros(len(w), dtype=np.float32)
    args = (C.c_uint32(0), C.c_uint64(len(w)), C.c_float(1e-3), C.c_float(0.9), C.c_float(0.999), C.c_float(1e-8))
    gp = g.ctypes.data_as(C.c_void_p)
    op = out.ctypes.data_as(C.c_void_p)
    assert lib.karma_host_update(C.c_uint32(7), fptr(w.copy()), fptr(m.copy()), fptr(v.copy()), gp, *args, C.c_uint64(1), op, 0, 0) == K.E_INVAL
    assert lib.karma_host_update(C.c_uint32(K.OPT_ADAM), fptr(w.copy()), None, None, gp, *args, C.c_uint64(1), op, 0, 0) == K.E_INVAL
    assert lib.karma_host_update(C.c_uint32(K.OPT_ADAM), fptr(w.copy()), fptr(m.copy()), fptr(v.copy()), gp, *args, C.c_uint64(0), op, 0, 0) == K.E_INVAL
