"""The C-ABI library loads and exports every symbol include/eagle.h declares (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2401_15077_amd as pkg
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2401_15077_amd import build
        build.build()
    return pkg.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "eagle.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(eagle_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(pkg.EXPORTS) == names


def test_workspace_size_and_config_validation(lib):
    s = synth.SHAPES["tiny"]
    par, rk = synth.TREES["T15"]
    cfg = pkg.make_config(s, par, rk, max_seq=256)
    need = lib.eagle_workspace_bytes(ctypes.byref(cfg))
    assert 8_000_000 < need < 400_000_000
    bad = pkg.make_config(s, par, rk, max_seq=256)
    bad.head_dim = 48
    assert lib.eagle_workspace_bytes(ctypes.byref(bad)) == 0
    assert b"head_dim" in lib.eagle_last_error()
    # a tree whose parents do not precede their children is rejected
    bad2 = pkg.make_config(s, np.array([-1, 2, 0], np.int32), np.array([0, 0, 0], np.int32), max_seq=256)
    assert lib.eagle_workspace_bytes(ctypes.byref(bad2)) == 0
    # 7B shape: weights (13.5 GB) + KV + activations
    big = pkg.make_config(synth.SHAPES["llama2-7b"], *synth.TREES["T26"], max_seq=1024)
    n7 = lib.eagle_workspace_bytes(ctypes.byref(big))
    assert 13.4e9 < n7 < 17e9


def test_null_arguments_are_errors_not_crashes(lib):
    assert lib.eagle_prefill(None, 0, None, 0, None) == -1
    assert lib.eagle_step(None, None, None, None) == -1
    assert lib.eagle_init(None, None, 0, None, None) == -1
    assert lib.eagle_version().startswith(b"libeagle")


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N > 1 exits with a message that says so (before touching torch)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr
