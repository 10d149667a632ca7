"""The shared library loads without a GPU and exports every symbol karma.h declares."""
import os
import re

import paper_2008_11421_amd as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    txt = open(os.path.join(ROOT, "include", "karma.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(karma_[a-z0-9_]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 20
    lib = K.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_null_arguments_are_rejected_without_gpu():
    lib = K.lib()
    assert lib.karma_simulate(None, 0, None, None, 0, 0, None, None, None, None) == K.E_INVAL
    assert lib.karma_plan_pure(None, 0, None, None, 0, 0, None, None) == K.E_INVAL
    assert lib.karma_create(None, None, None, 0, None, None, None, None) == K.E_INVAL
    assert lib.karma_step(None, None, None, 0, None) == K.E_INVAL
    assert lib.karma_k_mse_f32(None, None, None, None, None, 0, None) == K.E_INVAL


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: asking bench.py for more ends with a message, before any GPU call."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_entry_module_has_build_and_smoke():
    import importlib.util
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("graft_entry_under_test", os.path.join(root, "__graft_entry__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert callable(mod.build) and callable(mod.smoke)


def test_bench_stall_profile_arithmetic():
    """bench.backward_stalls: idle time of the compute stream before each backward-phase op, per layer, from
    measured starts and durations, and the same from the plan's simulated times."""
    import importlib.util
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)

    class Stub:
        # (kind, layer, simulated start ns, simulated end ns, measured ms); copies (O, I) are not compute ops
        ops = [("F", 0, 0, 10**6, 1.0), ("F", 1, 10**6, 2 * 10**6, 1.0), ("O", 1, 2 * 10**6, 5 * 10**6, 3.0),
               ("L", 2, 2 * 10**6, 3 * 10**6, 1.0), ("I", 1, 5 * 10**6, 8 * 10**6, 3.0),
               ("B", 1, 8 * 10**6, 9 * 10**6, 1.0), ("R", 0, 9 * 10**6, 9 * 10**6 + 500000, 0.5),
               ("B", 0, 9 * 10**6 + 500000, 10**7, 0.5)]
        starts = [0.0, 1.0, 2.0, 2.5, 5.0, 8.25, 9.25, 10.0]

        def karma_get_op_times(self):
            return self.ops

        def karma_get_op_starts(self):
            return self.starts

    ran = []
    out = bench.backward_stalls(Stub(), lambda: ran.append(1), 2)
    assert ran == [1]
    # measured: L starts 0.5 ms after F1 ends; B1 4.75 ms after L ends; R0 at once; B0 0.25 ms after R0 ends
    assert out["by_layer_ms"] == [0.25, 4.75, 0.5] and abs(out["total_ms"] - 5.5) < 1e-9
    # simulated: only B1 waits (5 ms for its swap-in)
    assert abs(out["simulated_total_ms"] - 5.0) < 1e-9
