"""The five benchmark workloads at full size, in the configuration bench.py times (tsp_spgemm,
A*A, default options).  Needs an MI355X.

Workloads 1, 2 and 5 are compared entry by entry with the oracle.  Workloads 3 and 4 are too
large for that (0.12 and 2.96 billion entries): their structure is checked on the device at full
size (row_ptr monotone, columns strictly ascending, closed-form or oracle-counted sizes, the
checksum identity sum(C) = (1^T A)(A 1)), and sampled rows, hub rows included, are compared
entry by entry with rows the oracle computes one by one.
"""
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


def _sampled_rows(tsp, oracle, C, A, rows):
    rp = C.row_ptr
    for i in rows:
        lo, hi = int(rp[i]), int(rp[i + 1])
        ref = oracle.spgemm_rows(A, A, int(i), int(i) + 1)
        assert hi - lo == ref.nnz, f"row {i}: {hi - lo} entries, oracle {ref.nnz}"
        assert np.array_equal(C.col_idx[lo:hi].cpu().numpy(), ref.col), f"row {i}: columns differ"
        _check_values(C.val[lo:hi].cpu().numpy(), ref, f"row {i}")


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


def test_stencil27_full_size(tsp, handle, oracle):
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
    print("workload 3: sampled rows", flush=True)
    rng = np.random.default_rng(3)
    rows = np.concatenate([[0, 1, 15, 16, A.rows - 1, 3 * 48 * 48 - 1, 3 * 48 * 48], rng.integers(0, A.rows, 40)])
    _sampled_rows(tsp, oracle, C, A, rows)
    C.free()
    handle.trim()


def test_rmat_full_size(tsp, handle, oracle):
    import torch
    A = inputs.config(4)
    deg = np.diff(A.row_ptr).astype(np.int64)
    products = int(deg[A.col_idx].sum())
    assert products == int((deg ** 2).sum())           # symmetric 0/1 matrix
    dA = tsp.to_device(A)
    print(f"workload 4: multiplying ({products} products)", flush=True)
    C = handle.spgemm(dA, dA)
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
    print("workload 4: sampled rows", flush=True)
    rng = np.random.default_rng(4)
    rows = np.concatenate([[0, 1, 2, 17, A.rows - 1], np.argsort(-deg)[:3], rng.integers(0, A.rows, 30)])
    _sampled_rows(tsp, oracle, C, A, rows)
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
