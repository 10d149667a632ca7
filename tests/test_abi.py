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
