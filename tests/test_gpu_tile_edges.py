"""The pipeline as the paper lays it out (tsp_spgemm_paper), at tile edges 8, 16 and 32, against the CPU
oracle and against the library's own path.  Needs an MI355X.

The result of the method does not depend on the tile edge (paper Section 2.1.2 fixes 8 for its hardware):
row_ptr and col_idx bit-exact at every edge, values within 1e-5 * sum_k|a_ik||b_kj| + 1e-7; the tile and
task-list counts the call reports equal those of the oracle's tile objects built at the same edge.
"""
import numpy as np
import pytest

from paper_2009_14600_amd import inputs

pytestmark = pytest.mark.gpu

RTOL_S, ATOL = 1e-5, 1e-7
EDGES = (8, 16, 32)


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


def _check(C, ref, what):
    row_ptr, col, val = C.to_host()
    assert np.array_equal(row_ptr, ref.row_ptr), f"{what}: row_ptr differs"
    assert np.array_equal(col, ref.col), f"{what}: col_idx differs"
    err = np.abs(val.astype(np.float64) - ref.val)
    bound = RTOL_S * ref.mag + ATOL
    bad = np.nonzero(err > bound)[0]
    assert bad.size == 0, f"{what}: {bad.size} values out of tolerance, first at {bad[:5]}"


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_small_configs_at_every_tile_edge(tsp, handle, oracle, index):
    A = inputs.config(index, small=True)
    print(f"config {index} small: {A.name} rows={A.rows} nnz={A.nnz}", flush=True)
    dA = tsp.to_device(A)
    ref = oracle.spgemm(A, A, threads=4)
    own = handle.spgemm(dA, dA)
    own_host = own.to_host()
    own.free()
    for T in EDGES:
        print(f"  tile edge {T}", flush=True)
        C = handle.spgemm_paper(dA, dA, T)
        _check(C, ref, f"{A.name}, tile edge {T}")
        got = C.to_host()
        assert np.array_equal(got[0], own_host[0]) and np.array_equal(got[1], own_host[1])
        C.free()


@pytest.mark.parametrize("M,K,N,da,db,seed", [
    (37, 53, 41, 0.2, 0.2, 1), (200, 90, 333, 0.05, 0.1, 2), (33, 1000, 17, 0.02, 0.3, 3),
    (1, 70, 1, 0.5, 0.5, 4), (129, 129, 129, 0.3, 0.01, 5),
])
def test_rectangular_ragged_products(tsp, handle, oracle, M, K, N, da, db, seed):
    A = inputs.random_sparse(M, K, da, 100 + seed, empty_row_fraction=0.2)
    B = inputs.random_sparse(K, N, db, 200 + seed, empty_row_fraction=0.1)
    print(f"rectangular {M}x{K}x{N}: nnz {A.nnz}, {B.nnz}", flush=True)
    ref = oracle.spgemm(A, B, threads=2)
    dA, dB = tsp.to_device(A), tsp.to_device(B)
    for T in EDGES:
        C = handle.spgemm_paper(dA, dB, T)
        assert (C.rows, C.cols) == (M, N)
        _check(C, ref, f"{M}x{K}x{N}, tile edge {T}")
        C.free()


def test_counts_equal_the_tile_objects_of_the_oracle(tsp, handle, oracle):
    """Tiles, candidate pairs, task-list entries and output tiles at every edge: the oracle builds the
    bitmap format and the task list of Algorithm 1 at the same edge (pure Python, so a small product)."""
    A = inputs.random_sparse(150, 170, 0.04, 31)
    B = inputs.random_sparse(170, 140, 0.05, 32)
    dA, dB = tsp.to_device(A), tsp.to_device(B)
    for T in EDGES:
        TA, TB = oracle.bitmap_format(A, T), oracle.bitmap_format(B, T)
        tl = oracle.task_list(TA, TB)
        C = handle.spgemm_paper(dA, dB, T)
        st = handle.stats()
        assert st["a_tiles"] == TA.tile_row.shape[0] and st["b_tiles"] == TB.tile_row.shape[0], T
        assert st["candidate_pairs"] == tl.candidates, T
        assert st["pairs"] == tl.a_tile.shape[0], T
        assert st["c_tiles"] == tl.offsets.shape[0] - 1, T
        assert st["c_nnz"] == C.nnz
        C.free()


def test_fp32_values_int64_row_pointers_stored_zeros_and_cancellation(tsp, handle, oracle):
    rng = np.random.default_rng(77)
    A = inputs.random_sparse(90, 90, 0.1, 41, values="smallint")
    A.val[rng.random(A.nnz) < 0.2] = 0.0                   # stored zeros stay structural
    ref = oracle.spgemm(A, A, threads=2)
    assert (ref.val == 0).any()                             # some sums cancel or are products with zero
    dA = tsp.to_device(A, value_dtype="f32", row_ptr_dtype="i64")
    for T in EDGES:
        C = handle.spgemm_paper(dA, dA, T)
        _check(C, ref, f"fp32/int64 inputs, tile edge {T}")
        C.free()


def test_empty_operands_and_error_codes(tsp, handle):
    import torch
    E = tsp.to_device(inputs.random_sparse(40, 50, 0.0, 1))
    F = tsp.to_device(inputs.random_sparse(50, 30, 0.3, 2))
    for T in EDGES:
        C = handle.spgemm_paper(E, F, T)
        assert C.nnz == 0 and (C.rows, C.cols) == (40, 30)
        assert np.array_equal(C.to_host()[0], np.zeros(41, dtype=np.int64))
        C.free()
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm_paper(F, F, 12)                       # not a tile edge of this build
    assert e.value.status == -1
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm_paper(F, F, 16)                       # 50x30 times 50x30
    assert e.value.status == -2
    bad = tsp.to_device(inputs.random_sparse(40, 40, 0.2, 3))
    cols = bad.col_idx.clone()
    bad.col_idx = torch.flip(cols, dims=[0]).contiguous()   # descending columns
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm_paper(bad, bad, 8)
    assert e.value.status == -3
    bad.col_idx = cols.clone()
    bad.col_idx[5] = -7
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm_paper(bad, bad, 32)
    assert e.value.status == -3
    bad.col_idx = cols
    rp = bad.row_ptr.clone()
    bad.row_ptr[3] = rp[4] + 1                              # non-monotone row_ptr
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm_paper(bad, bad, 16)
    assert e.value.status == -3
    bad.row_ptr = rp
    C = handle.spgemm_paper(bad, bad, 16)                   # the handle still works afterwards
    D = handle.spgemm(bad, bad)
    for x, y in zip(C.to_host()[:2], D.to_host()[:2]):
        assert np.array_equal(x, y)
    C.free()
    D.free()
