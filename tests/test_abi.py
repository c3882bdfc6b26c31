"""Host-side checks that need no GPU: the shared library builds/loads and exports every entry point
the public header declares; the Python binding declares a prototype for each of them."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "laser.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(laser_[a-z_0-9]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    from paper_2408_05676_amd import build as b
    if not os.path.exists(b.LIB):
        b.build(verbose=False)
    return ctypes.CDLL(b.LIB)


def test_header_declares_the_four_calls():
    names = _declared()
    for n in ("laser_pool_build", "laser_retrieve_drafts", "laser_verify_step", "laser_kv_commit"):
        assert n in names
    assert len(names) >= 15


def test_library_exports_every_declared_symbol(lib):
    missing = [n for n in _declared() if not hasattr(lib, n)]
    assert not missing, missing
    lib.laser_version.restype = ctypes.c_char_p
    assert lib.laser_version().startswith(b"laser")


def test_binding_covers_every_declared_symbol():
    src = open(os.path.join(ROOT, "paper_2408_05676_amd", "binding.py")).read()
    missing = [n for n in _declared() if n not in src]
    assert not missing, missing


def test_argument_errors_without_touching_the_gpu(lib):
    lib.laser_last_error.restype = ctypes.c_char_p
    out = ctypes.c_void_p()
    # n_max out of range is rejected before any device work
    rc = lib.laser_pool_build(None, None, None, ctypes.c_int64(0), 99, None, ctypes.byref(out))
    assert rc == -1 and b"n_max" in lib.laser_last_error()
    assert lib.laser_pool_build(None, None, None, ctypes.c_int64(-1), 2, None, ctypes.byref(out)) == -1
    assert lib.laser_retrieve_drafts(None, None, None, 1, 1, 1, 1, 1, None, None, None, None, None) == -1
    assert lib.laser_kv_commit(None, None, None, 1, None) == -1
    assert lib.laser_model_create(None, None, ctypes.byref(out)) == -1
    assert lib.laser_pool_destroy(None) == 0 and lib.laser_kv_destroy(None) == 0 and lib.laser_model_destroy(None) == 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2408_05676_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f


def test_binding_limits_agree_with_the_header():
    import re as _re
    from paper_2408_05676_amd import binding
    src = open(HEADER).read()
    for name in ("NGRAM", "DRAFT", "TOPK", "TREE", "OWN_TEXT"):
        m = _re.search(r"#define\s+LASER_MAX_%s\s+(\d+)" % name, src)
        assert m and int(m.group(1)) == getattr(binding, "MAX_" + name), name


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU benchmark: --gpus N with N > 1 (or a multi-rank environment) exits with a message
    before anything touches a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
