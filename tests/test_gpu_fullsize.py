"""The five benchmark workloads at full size, in the configuration bench.py times (tsp_spgemm,
A*A, default options).  Needs an MI355X.

All five are compared entry by entry with the oracle.  Workloads 1, 2 and 5 in one piece;
workloads 3 and 4 (0.12 and 2.96 billion entries) in consecutive blocks of rows: the block's
col_idx and val are copied back, the oracle computes the same rows on a thread pool, every
column must be equal and every value inside the tolerance, and the block is dropped.  Before
that their structure is checked on the device at full size (row_ptr monotone, columns strictly
ascending, closed-form or oracle-counted sizes, the checksum identity sum(C) = (1^T A)(A 1)).
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2009_14600_amd import inputs

pytestmark = pytest.mark.gpu

RTOL_S, ATOL = 1e-5, 1e-7


@pytest.fixture(scope="module")
def tsp():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2009_14600_amd import tsp as binding
    binding.load_library()
    return binding


@pytest.fixture(scope="module")
def handle(tsp):
    h = tsp.Handle(validate=True)
    yield h
    h.close()


def _check_values(val, ref, what):
    err = np.abs(val.astype(np.float64) - ref.val)
    bound = RTOL_S * ref.mag + ATOL
    bad = np.nonzero(err > bound)[0]
    assert bad.size == 0, f"{what}: {bad.size} values out of tolerance, first {bad[:5]}"


@pytest.mark.parametrize("index", [1, 2, 5])
def test_full_comparison(tsp, handle, oracle, index):
    A = inputs.config(index)
    print(f"workload {index}: {A.name} rows={A.rows} nnz={A.nnz}", flush=True)
    dA = tsp.to_device(A)
    C = handle.spgemm(dA, dA)
    row_ptr, col, val = C.to_host()
    C.free()
    ref = oracle.spgemm(A, A, threads=8)
    assert np.array_equal(row_ptr, ref.row_ptr) and np.array_equal(col, ref.col)
    _check_values(val, ref, A.name)
    if index == 2:
        assert (ref.nnz, ref.products) == (3397636, 6535176)
    if index == 1:
        assert ref.products == 65536


def _structure_checks_on_device(torch, C, A):
    """row_ptr monotone and consistent, columns in range and strictly ascending inside rows."""
    rp = C.row_ptr
    assert int(rp[0]) == 0 and int(rp[-1]) == C.nnz
    assert bool((rp[1:] >= rp[:-1]).all())
    assert int(C.col_idx.min()) >= 0 and int(C.col_idx.max()) < C.cols
    n = C.nnz
    step = 1 << 28                                     # chunked: the arrays can be billions long
    nonempty = rp[:-1][rp[1:] > rp[:-1]]               # first position of every non-empty row
    for lo in range(0, n - 1, step):
        hi = min(n - 1, lo + step)
        ascending = C.col_idx[lo + 1:hi + 1] > C.col_idx[lo:hi]
        starts = nonempty[(nonempty > lo) & (nonempty <= hi)] - (lo + 1)
        ascending[starts] = True
        assert bool(ascending.all()), f"columns not ascending in entries [{lo},{hi}]"


def _streamed_comparison(oracle, C, A, say, block_entries=120_000_000):
    """Every entry of C against the oracle, block of rows by block of rows.  Returns the number of
    entries compared and the oracle's product count."""
    threads = min(16, os.cpu_count() or 1)
    ops = (oracle._Operand(A), oracle._Operand(A))
    rp = C.row_ptr.cpu().numpy().astype(np.int64)
    assert rp[0] == 0 and rp[-1] == C.nnz
    compared = products = 0
    r0 = 0
    with ThreadPoolExecutor(max_workers=threads) as pool:
        while r0 < C.rows:
            # as many rows as fit the block (at least one)
            r1 = max(r0 + 1, int(np.searchsorted(rp, rp[r0] + block_entries, side="right")) - 1)
            r1 = min(r1, C.rows)
            lo, hi = int(rp[r0]), int(rp[r1])
            col = C.col_idx[lo:hi].cpu().numpy()
            val = C.val[lo:hi].cpu().numpy()
            # sub-blocks of about equal numbers of entries, several per thread
            cuts = np.searchsorted(rp[r0:r1 + 1], np.linspace(lo, hi, 4 * threads + 1)).astype(np.int64) + r0
            cuts[0], cuts[-1] = r0, r1
            cuts = np.unique(cuts)

            def part(k):
                s0, s1 = int(cuts[k]), int(cuts[k + 1])
                ref = oracle.spgemm_rows(A, A, s0, s1, _ops=ops)
                if not np.array_equal(ref.row_ptr + rp[s0], rp[s0:s1 + 1]):
                    return f"rows [{s0},{s1}): row lengths differ", 0, 0
                a, b = int(rp[s0]) - lo, int(rp[s1]) - lo
                if not np.array_equal(col[a:b], ref.col):
                    first = int(np.nonzero(col[a:b] != ref.col)[0][0])
                    return f"rows [{s0},{s1}): column differs at entry {lo + a + first}", 0, 0
                err = np.abs(val[a:b].astype(np.float64) - ref.val)
                bad = np.nonzero(err > RTOL_S * ref.mag + ATOL)[0]
                if bad.size:
                    return f"rows [{s0},{s1}): {bad.size} values out of tolerance, first at entry {lo + a + int(bad[0])}", 0, 0
                return None, ref.nnz, ref.products

            for message, n, p in pool.map(part, range(cuts.shape[0] - 1)):
                assert message is None, message
                compared += n
                products += p
            say(f"rows [{r0},{r1}) of {C.rows}: {compared} of {C.nnz} entries equal to the oracle's")
            r0 = r1
    return compared, products


def _checksum(torch, C, A):
    """sum_ij c_ij = (1^T A)(A 1), within the accumulated fp32 rounding of the entries."""
    v = A.val.astype(np.float64)
    col_sum = np.bincount(A.col_idx, weights=v, minlength=A.cols)
    row_sum = np.bincount(np.repeat(np.arange(A.rows), np.diff(A.row_ptr)), weights=v, minlength=A.rows)
    col_abs = np.bincount(A.col_idx, weights=np.abs(v), minlength=A.cols)
    row_abs = np.bincount(np.repeat(np.arange(A.rows), np.diff(A.row_ptr)), weights=np.abs(v), minlength=A.rows)
    want, scale = float(col_sum @ row_sum), float(col_abs @ row_abs)
    got = float(C.val.sum(dtype=torch.float64))
    assert abs(got - want) <= RTOL_S * scale + ATOL * C.nnz, (got, want, scale)


def test_stencil27_full_size(tsp, handle, oracle, capsys):
    import torch
    A = inputs.config(3)
    assert A.nnz == 81 * A.rows == 26873856
    dA = tsp.to_device(A)
    print("workload 3: multiplying", flush=True)
    C = handle.spgemm(dA, dA)
    st = handle.stats()
    assert C.nnz == 375 * A.rows == 124416000          # 5x5x5 node neighbourhood x 3 dof, periodic grid
    assert bool((C.row_ptr[1:] - C.row_ptr[:-1] == 375).all())
    assert st["a_tiles"] == 559872 and st["c_nnz"] == C.nnz
    print("workload 3: structure", flush=True)
    _structure_checks_on_device(torch, C, A)
    _checksum(torch, C, A)
    def say(text):
        with capsys.disabled():
            print(f"\n  workload 3: {text}", end="", flush=True)
    compared, products = _streamed_comparison(oracle, C, A, say)
    assert compared == C.nnz and products == 81 * 81 * A.rows == 2176782336
    C.free()
    handle.trim()


def test_rmat_full_size(tsp, handle, oracle, capsys):
    import torch
    A = inputs.config(4)
    deg = np.diff(A.row_ptr).astype(np.int64)
    products = int(deg[A.col_idx].sum())
    assert products == int((deg ** 2).sum())           # symmetric 0/1 matrix
    dA = tsp.to_device(A)
    print(f"workload 4: multiplying ({products} products)", flush=True)
    handle.spgemm(dA, dA).free()                       # (the second call with the same operands is the one bench.py times:
    C = handle.spgemm(dA, dA)                          # the counting kernel then keeps its counters for the task-list kernel)
    print(f"workload 4: nnz(C) = {C.nnz}", flush=True)
    assert C.nnz > 2 ** 31                             # needs the 64-bit row_ptr
    counts, _ = oracle.row_nnz(A, A, 0, 256)           # the hub rows: the longest rows of C
    assert np.array_equal((C.row_ptr[1:257] - C.row_ptr[:256]).cpu().numpy(), counts)
    print("workload 4: structure", flush=True)
    _structure_checks_on_device(torch, C, A)
    # 0/1 inputs: every value is a small integer and exact; their sum is the number of products
    total = 0
    for lo in range(0, C.nnz, 1 << 28):
        chunk = C.val[lo:lo + (1 << 28)]
        assert bool((chunk == torch.round(chunk)).all()) and float(chunk.min()) >= 1.0
        total += int(chunk.sum(dtype=torch.float64))
    assert total == products
    def say(text):
        with capsys.disabled():
            print(f"\n  workload 4: {text}", end="", flush=True)
    compared, oracle_products = _streamed_comparison(oracle, C, A, say)
    assert compared == C.nnz == 2962529917 and oracle_products == products == 9487075854
    rng = np.random.default_rng(4)
    diag_rows = rng.integers(0, A.rows, 200)
    for i in diag_rows:                                # c_ii = deg(i)
        lo, hi = int(C.row_ptr[i]), int(C.row_ptr[i + 1])
        if deg[i] == 0:
            assert hi == lo
            continue
        cols = C.col_idx[lo:hi]
        pos = int(torch.searchsorted(cols, int(i)))
        assert int(cols[pos]) == i and float(C.val[lo + pos]) == float(deg[i])
    C.free()
    handle.trim()
