"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no GPU): a build of
oracle/spgemm_oracle.c with both sanitizers runs the same products as the ordinary build, on row ranges
that do not start at zero, rectangular shapes, empty rows and empty matrices.  Any out-of-bounds access,
use after free, signed overflow or misaligned pointer aborts the run with a report."""
import os
import subprocess
import tempfile

import numpy as np
import pytest

from paper_2009_14600_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sanitized_binary():
    out = os.path.join(tempfile.mkdtemp(prefix="oracle_san_"), "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-o", out, os.path.join(ROOT, "oracle", "sanitized_check.c"),
           os.path.join(ROOT, "oracle", "spgemm_oracle.c"), "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        pytest.skip("no sanitizer runtime for gcc here: " + res.stderr[-300:])
    return out


def _write_case(path, A, B):
    with open(path, "wb") as f:
        np.array([A.rows, A.cols, A.nnz, B.rows, B.cols, B.nnz], dtype=np.int64).tofile(f)
        for m in (A, B):
            np.asarray(m.row_ptr, dtype=np.int64).tofile(f)
            np.asarray(m.col_idx, dtype=np.int32).tofile(f)
            np.asarray(m.val).astype(np.float16).astype(np.float64).tofile(f)


@pytest.mark.parametrize("maker", [
    lambda: (inputs.config(1, small=True),) * 2,
    lambda: (inputs.config(4, small=True),) * 2,
    lambda: (inputs.random_sparse(57, 23, 0.2, 5, empty_row_fraction=0.3), inputs.random_sparse(23, 91, 0.15, 6)),
    lambda: (inputs.random_sparse(9, 0, 0.5, 7), inputs.random_sparse(0, 4, 0.5, 8)),        # empty inner dimension
    lambda: (inputs.random_sparse(1, 40, 0.9, 9), inputs.random_sparse(40, 1, 0.9, 10)),
])
def test_sanitized_oracle_matches_the_ordinary_build(oracle, sanitized_binary, maker):
    A, B = maker()
    with tempfile.TemporaryDirectory() as d:
        path = os.path.join(d, "case.bin")
        _write_case(path, A, B)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        env.pop("LD_PRELOAD", None)                 # the sanitizer runtime must come first in the process
        res = subprocess.run([sanitized_binary, path], capture_output=True, text=True, timeout=120, env=env)
    assert res.returncode == 0, res.stderr[-2000:]
    products, nnz, col_sum, val_sum, abs_sum = res.stdout.split()
    ref = oracle.spgemm(A, B)
    assert int(products) == ref.products and int(nnz) == ref.nnz
    assert int(col_sum) == int(ref.col.astype(np.int64).sum())
    # the same serial code row by row: the sums of the outputs agree to the last bit
    assert float(val_sum) == float(np.sum(ref.val)) or abs(float(val_sum) - float(np.sum(ref.val))) <= 1e-9 * max(1.0, float(abs_sum))
    assert abs(float(abs_sum) - float(np.sum(ref.mag))) <= 1e-9 * max(1.0, float(abs_sum))
