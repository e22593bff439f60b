"""tsp_compact_zeros_static (the compaction that allocates nothing) against tsp_compact_zeros, through
the C ABI: two calls in a row on one handle, the second on a smaller matrix, so that what the first call
left in the library's fixed scratch array is still there when the second one runs.  Needs an MI355X."""
import numpy as np
import pytest

from paper_2009_14600_amd import inputs

pytestmark = pytest.mark.gpu


def _matrix_with_zeros(rows, cols, density, seed):
    """Small-integer product whose sums cancel now and then, so that C holds exact zeros to drop."""
    A = inputs.random_sparse(rows, cols, density, seed, empty_row_fraction=0.1, values="smallint")
    B = inputs.random_sparse(cols, rows, density, seed + 1, values="smallint")
    return A, B


def test_static_compaction_equals_the_allocating_one_twice_in_a_row():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2009_14600_amd import tsp
    tsp.load_library()
    handle = tsp.Handle(validate=True)
    removed = []
    for rows, cols, density, seed in [(3000, 700, 0.02, 5), (301, 150, 0.05, 9)]:     # the second is smaller
        A, B = _matrix_with_zeros(rows, cols, density, seed)
        print(f"static compaction: product {rows}x{cols}x{rows}, seed {seed}", flush=True)
        C = handle.spgemm(tsp.to_device(A), tsp.to_device(B))
        want = handle.compact_zeros(C)                                   # the existing entry point
        out_row_ptr = torch.full((rows + 1,), -7, dtype=torch.int64, device="cuda")
        out_col = torch.full((C.nnz + 3,), -7, dtype=torch.int32, device="cuda")
        out_val = torch.full((C.nnz + 3,), -7.0, dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        nnz = handle.compact_zeros_static(C, out_row_ptr, out_col, out_val)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before                   # nothing taken from the handle's allocator
        assert nnz == want.nnz < C.nnz
        assert torch.equal(out_row_ptr, want.row_ptr)
        assert torch.equal(out_col[:nnz], want.col_idx) and torch.equal(out_val[:nnz], want.val)
        assert bool((out_col[nnz:] == -7).all()) and bool((out_val[nnz:] == -7.0).all())   # nothing written past nnz
        removed.append(C.nnz - nnz)
        want.free()
        C.free()
    assert all(r > 0 for r in removed)
    # sizes beyond the fixed scratch array are refused with an error code, nothing is enqueued
    big = tsp.DeviceCSR(tsp_rows := 524289, 4, torch.zeros(tsp_rows + 1, dtype=torch.int64, device="cuda"),
                        torch.zeros(0, dtype=torch.int32, device="cuda"), torch.zeros(0, dtype=torch.float32, device="cuda"))
    with pytest.raises(tsp.TspError) as e:
        handle.compact_zeros_static(big, torch.zeros(tsp_rows + 1, dtype=torch.int64, device="cuda"),
                                    torch.zeros(1, dtype=torch.int32, device="cuda"),
                                    torch.zeros(1, dtype=torch.float32, device="cuda"))
    assert e.value.status == -7
    handle.close()
