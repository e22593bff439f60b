"""The C-ABI library loads and exports every function include/tsp.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "tsp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*\s*|int\s+)(tsp_\w+)\s*\(", text, flags=re.M)
    assert len(names) >= 14
    return names


def test_library_exports_every_declared_symbol():
    from paper_2009_14600_amd import tsp
    if not os.path.exists(tsp.LIB_PATH):
        from paper_2009_14600_amd.build import build_library
        build_library()
    lib = ctypes.CDLL(tsp.LIB_PATH)
    declared = _declared_functions()
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in tsp.h but not exported"
    assert sorted(declared) == sorted(tsp.EXPORTS)


def test_strerror_needs_no_gpu():
    from paper_2009_14600_amd import tsp
    lib = tsp.load_library()
    assert lib.tsp_strerror(0) == b"success"
    assert b"canonical" in lib.tsp_strerror(-3)
    assert lib.tsp_strerror(-99) == b"unknown status"


def test_binding_refuses_to_run_without_gpu():
    import torch
    from paper_2009_14600_amd import tsp
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        tsp.Handle()


def test_bench_refuses_more_than_one_gpu():
    """The path has no multi-GPU part: bench.py says so instead of running."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode == 2
    assert "one GPU" in res.stderr
