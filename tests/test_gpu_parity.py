"""Parity of the HIP path (through the C ABI) against the CPU oracle.  Needs an MI355X.

Bar: row_ptr and col_idx bit-exact; |c - c_ref| <= 1e-5 * sum_k|a_ik||b_kj| + 1e-7 per entry.
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


def assert_matches_oracle(C, ref, what=""):
    row_ptr, col, val = C.to_host()
    assert np.array_equal(row_ptr, ref.row_ptr), f"{what}: row_ptr differs"
    assert np.array_equal(col, ref.col), f"{what}: col_idx differs"
    err = np.abs(val.astype(np.float64) - ref.val)
    bound = RTOL_S * ref.mag + ATOL
    bad = np.nonzero(err > bound)[0]
    assert bad.size == 0, (f"{what}: {bad.size} values out of tolerance, first at {bad[:5]}: "
                           f"got {val[bad[:5]]}, want {ref.val[bad[:5]]}, bound {bound[bad[:5]]}")


def run_and_check(tsp, handle, oracle, A, B=None, **upload):
    dA = tsp.to_device(A, **upload)
    dB = dA if B is None else tsp.to_device(B, **upload)
    C = handle.spgemm(dA, dB)
    try:
        ref = oracle.spgemm(A, A if B is None else B, threads=4)
        assert (C.rows, C.cols) == (A.rows, (A if B is None else B).cols)
        assert_matches_oracle(C, ref, A.name)
        return C.nnz, ref
    finally:
        C.free()


# ------------------------------------------------------------------ small instances of the five workloads
@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_small_configs(tsp, handle, oracle, index):
    A = inputs.config(index, small=True)
    print(f"config {index} small: {A.name} rows={A.rows} nnz={A.nnz}", flush=True)
    run_and_check(tsp, handle, oracle, A)


# ------------------------------------------------------------------ rectangular, ragged, degenerate
@pytest.mark.parametrize("M,K,N,density,seed,kind", [
    (1, 1, 1, 1.0, 1, "uniform"),
    (15, 17, 33, 0.3, 2, "uniform"),
    (100, 37, 250, 0.08, 3, "uniform"),
    (257, 129, 65, 0.05, 4, "smallint"),
    (64, 640, 64, 0.02, 5, "uniform"),
    (500, 500, 500, 0.01, 6, "uniform"),
    (33, 1000, 47, 0.2, 7, "ones"),
    (200, 200, 200, 0.25, 8, "uniform"),      # dense tiles, long segments
])
def test_random_rectangular(tsp, handle, oracle, M, K, N, density, seed, kind):
    A = inputs.random_sparse(M, K, density, seed, empty_row_fraction=0.15, values=kind)
    B = inputs.random_sparse(K, N, density, seed + 50, empty_row_fraction=0.15, values=kind)
    print(f"random {M}x{K}x{N} d={density} {kind}", flush=True)
    run_and_check(tsp, handle, oracle, A, B)


def test_very_wide_tile_rows_take_the_merge_path(tsp, handle, oracle):
    """Tile-rows whose tile columns span more than the converter's LDS bitmap (24576 tile columns
    for wave-sized groups, 131072 for block-sized ones) are converted by the 16-way merge."""
    rng = np.random.default_rng(17)
    n_wide = 2_000_000
    rows = np.repeat(np.arange(40), 30)
    cols = np.concatenate([np.sort(rng.choice(n_wide, 30, replace=False)) for _ in range(40)])
    A = inputs.from_coo(40, n_wide, rows, cols, rng.uniform(-1, 1, rows.shape[0]))
    brow = rng.choice(n_wide, 5000, replace=False)
    B = inputs.from_coo(n_wide, 70, np.concatenate([brow, cols[::7]]),
                        rng.integers(0, 70, brow.shape[0] + cols[::7].shape[0]),
                        rng.uniform(-1, 1, brow.shape[0] + cols[::7].shape[0]))
    nnz, _ = run_and_check(tsp, handle, oracle, A, B)
    assert nnz > 0
    At = inputs.from_coo(n_wide, 40, cols, rows, A.val)            # tall operand, wide inner dimension
    run_and_check(tsp, handle, oracle, At, A)


def test_long_tile_rows_use_block_sized_groups(tsp, handle, oracle):
    A = inputs.random_sparse(64, 3000, 0.6, 71)                    # > 1024 entries per tile-row on average
    B = inputs.random_sparse(3000, 48, 0.05, 72)
    run_and_check(tsp, handle, oracle, A, B)


def test_empty_operands(tsp, handle, oracle):
    for M, K, N in [(0, 5, 7), (5, 0, 7), (5, 7, 0), (20, 30, 40)]:
        A = inputs.random_sparse(M, K, 0.0, 1)
        B = inputs.random_sparse(K, N, 0.3 if M == 20 else 0.0, 2)
        nnz, _ = run_and_check(tsp, handle, oracle, A, B)
        assert nnz == 0


def test_cancellation_and_stored_zeros_keep_their_positions(tsp, handle, oracle):
    A = inputs.from_coo(2, 2, [0, 0, 1], [0, 1, 1], [1.0, 1.0, 2.0])
    B = inputs.from_coo(2, 3, [0, 1, 1], [0, 0, 2], [1.0, -1.0, 0.0])
    nnz, _ = run_and_check(tsp, handle, oracle, A, B)
    assert nnz == 4


def test_fp16_subnormal_inputs_are_not_flushed(tsp, handle, oracle):
    """Products of fp16 subnormals with ordinary values are far above the 1e-7 absolute term,
    so a matrix unit that flushed subnormal inputs would fail here."""
    A = inputs.random_sparse(64, 64, 0.2, 31, values="tiny")
    B = inputs.random_sparse(64, 64, 0.2, 32, values="smallint")
    _, ref = run_and_check(tsp, handle, oracle, A, B)
    assert (ref.mag > 1e-6).sum() > 100


def test_zero_one_inputs_are_exact(tsp, handle, oracle):
    G = inputs.rmat(10, 16, seed=5)
    dG = tsp.to_device(G)
    C = handle.spgemm(dG, dG)
    ref = oracle.spgemm(G, G)
    _, _, val = C.to_host()
    assert np.array_equal(val.astype(np.float64), ref.val)         # integers: no rounding at all
    assert oracle.smape_percent(ref.val, val) == 0.0
    C.free()


def test_fp32_and_int64_inputs(tsp, handle, oracle):
    A = inputs.config(3, small=True)
    run_and_check(tsp, handle, oracle, A, value_dtype="f32", row_ptr_dtype="i64")
    # values that are not fp16 numbers are rounded to nearest even on the device
    import torch
    rng = np.random.default_rng(3)
    A = inputs.random_sparse(90, 70, 0.1, 41)
    v32 = rng.uniform(-2, 2, A.nnz).astype(np.float32)
    dA = tsp.to_device(A, value_dtype="f32")
    dA.val = torch.from_numpy(v32).cuda()
    B = inputs.random_sparse(70, 50, 0.1, 42)
    C = handle.spgemm(dA, tsp.to_device(B))
    A.val = v32.astype(np.float16)
    assert_matches_oracle(C, oracle.spgemm(A, B), "fp32 inputs")
    C.free()


def test_runs_are_bit_identical(tsp, handle):
    A = inputs.config(4, small=True)
    dA = tsp.to_device(A)
    outs = []
    for _ in range(3):
        C = handle.spgemm(dA, dA)
        outs.append(C.to_host())
        C.free()
    for o in outs[1:]:
        assert all(np.array_equal(x, y) for x, y in zip(o, outs[0]))


def test_products_count_and_selection_criteria(tsp, oracle):
    """TSP_OPT_COUNT_PRODUCTS: the library's count of the intermediate products (the FLOP of the benchmark
    metric are twice that) equals the oracle's, for A*A and for a rectangular A*B with 64-bit row pointers;
    off, the field reads -1.  The selection criteria of Section 6.1 are reported for the left operand."""
    h = _variant_handle(tsp, OPT_COUNT_PRODUCTS=1)
    try:
        A = inputs.config(5, small=True)
        dA = tsp.to_device(A)
        h.spgemm(dA, dA).free()
        st = h.stats()
        assert st["products"] == oracle.spgemm(A, A, threads=4).products > 0
        assert abs(st["a_mean_row"] - A.nnz / A.rows) < 1e-3 and st["a_tile_fill"] > 100 and st["well_filled_tiles"] == 1
        assert st["in_paper_regime"] == 0                                  # fewer than 300000 entries
        L = inputs.random_sparse(90, 70, 0.1, 3, empty_row_fraction=0.2)
        R = inputs.random_sparse(70, 200, 0.05, 4)
        h.spgemm(tsp.to_device(L, row_ptr_dtype="i64"), tsp.to_device(R, row_ptr_dtype="i64")).free()
        assert h.stats()["products"] == oracle.spgemm(L, R).products
        h.set_option(tsp.OPT_COUNT_PRODUCTS, 0)
        h.spgemm(dA, dA).free()
        assert h.stats()["products"] == -1
    finally:
        h.close()


# ------------------------------------------------------------------ error paths (forced from the host)
def test_error_codes(tsp, handle):
    import torch
    for key, value in [(tsp.OPT_WORK_ORDER, 3), (tsp.OPT_WORK_ORDER, -1), (tsp.OPT_NUMERIC_RUN, 5), (99, 0)]:
        with pytest.raises(tsp.TspError) as e:                      # option values out of range, unknown option
            handle.set_option(key, value)
        assert e.value.status == -1
    A = tsp.to_device(inputs.random_sparse(20, 30, 0.2, 1))
    B = tsp.to_device(inputs.random_sparse(31, 10, 0.2, 2))
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm(A, B)
    assert e.value.status == -2
    bad = tsp.to_device(inputs.random_sparse(40, 40, 0.2, 3))
    cols = bad.col_idx.clone()
    bad.col_idx = torch.flip(cols, dims=[0]).contiguous()           # descending columns
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm(bad, bad)
    assert e.value.status == -3
    bad.col_idx = cols.clone()
    bad.col_idx[5] = 4000                                           # out of range column
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm(bad, bad)
    assert e.value.status == -3
    bad.col_idx = cols.clone()
    bad.col_idx[5] = -7                                             # negative column: the tile-row leaves the
    with pytest.raises(tsp.TspError) as e:                          # converter's fast path with an empty range
        handle.spgemm(bad, bad)
    assert e.value.status == -3
    first_of_row = int(bad.row_ptr[2])
    bad.col_idx = cols.clone()
    bad.col_idx[first_of_row] = -1                                  # ... also as the first entry of a row
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm(bad, bad)
    assert e.value.status == -3
    bad.col_idx = cols
    rp = bad.row_ptr.clone()
    bad.row_ptr[3] = rp[4] + 1                                      # non-monotone row_ptr
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm(bad, bad)
    assert e.value.status == -3
    bad.row_ptr = rp
    C = handle.spgemm(bad, bad)                                     # the handle still works afterwards
    assert C.nnz > 0
    C.free()


# ------------------------------------------------------------------ phase by phase against the paper's objects
def _decode_groups(view, form, t):
    """Dense 16x16 image (values, occupancy) of tile t from the group storage of one form."""
    mask = int(view[f"{form}_group_mask"][t]) & 0xFFFFFFFF
    off = int(view[f"{form}_group_off"][t]) & 0xFFFFFFFF
    el = view[f"{form}_elements"]
    dense = np.zeros((16, 16), dtype=np.float16)
    stored = 0
    for g in range(32):
        if (mask >> g) & 1:
            vals = el[(off + stored) * 8:(off + stored + 1) * 8]
            h, x = g // 16, g % 16
            if form == "left":
                dense[x, 8 * h:8 * h + 8] = vals
            else:
                dense[8 * h:8 * h + 8, x] = vals
            stored += 1
    return dense


@pytest.mark.parametrize("maker", [
    lambda: (inputs.random_sparse(70, 45, 0.1, 61, empty_row_fraction=0.2), inputs.random_sparse(45, 90, 0.1, 62)),
    lambda: (inputs.config(2, small=True),) * 2,
    lambda: (inputs.config(5, small=True),) * 2,
    lambda: (inputs.config(1, small=True),) * 2,
])
def test_phases_against_paper_objects(tsp, handle, oracle, maker):
    A, B = maker()
    same = A is B
    dA = tsp.to_device(A)
    dB = dA if same else tsp.to_device(B)
    tA = handle.convert(dA)
    tB = tA if same else handle.convert(dB)
    refs, slots = [], []
    for M, tiles in ((A, tA), (B, tB)):
        bm = oracle.bitmap_format(M, 16)
        refs.append(bm)
        view = tiles.view()
        slot = tsp.tile_indices(view).cpu().numpy()      # tile index of the k-th tile in storage order
        slots.append(slot)
        v = {k: (x.cpu().numpy() if hasattr(x, "cpu") else x) for k, x in view.items()}
        n = bm.tile_row.shape[0]
        assert v["ntiles"] == n == slot.shape[0]
        assert v["tile_rows"] == bm.tile_rows and v["tile_cols"] == bm.tile_cols and v["tile_slots"] == M.nnz
        # a tile-row's tiles start at the position of its first entry in the CSR arrays
        first_entry = M.row_ptr[np.minimum(np.arange(bm.tile_rows) * 16, M.rows)]
        assert np.array_equal(v["tile_row_ptr"], first_entry)
        counts = v["tile_row_end"] - v["tile_row_ptr"]
        assert np.array_equal(np.repeat(np.arange(bm.tile_rows), counts), bm.tile_row)
        assert np.array_equal(v["tile_col"][slot], bm.tile_col)
        assert np.array_equal(v["row_mask"].view(np.uint16).reshape(-1, 16)[slot], bm.row_mask.astype(np.uint16))
        for t in range(n):
            occ = np.array([[(int(bm.row_mask[t, r]) >> c) & 1 for c in range(16)] for r in range(16)], dtype=bool)
            want = np.zeros((16, 16), dtype=np.float16)
            want[occ] = bm.elements[bm.index[t]:bm.index[t + 1]]      # ascending slot order = row-major
            for form in ("left", "right"):
                got = _decode_groups(v, form, int(slot[t]))
                assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), (t, form)
    plan = handle.symbolic(tA, tB)
    pv = {k: (x.cpu().numpy() if hasattr(x, "cpu") else x) for k, x in plan.view().items()}
    tl = oracle.task_list(refs[0], refs[1])
    masks, counts = oracle.counting(refs[0], refs[1], tl)
    assert pv["pairs"] == tl.a_tile.shape[0] and pv["c_tiles"] == tl.c_tile_row.shape[0]
    assert pv["candidate_pairs"] == tl.candidates
    assert np.array_equal(pv["pair_off"], tl.offsets)
    # the task list names tiles by their index in the tile arrays
    assert np.array_equal(pv["pair_a"], slots[0][tl.a_tile]) and np.array_equal(pv["pair_b"], slots[1][tl.b_tile])
    assert np.array_equal(pv["c_tile_row"], tl.c_tile_row) and np.array_equal(pv["c_tile_col"], tl.c_tile_col)
    assert np.array_equal(pv["c_row_mask"].view(np.uint16).reshape(-1, 16), masks.astype(np.uint16))
    assert pv["c_nnz"] == counts.sum()
    ref = oracle.spgemm(A, B)
    assert np.array_equal(pv["c_row_ptr"], ref.row_ptr)
    C = handle.numeric(tA, tB, plan)
    assert_matches_oracle(C, ref, "numeric phase")
    C2 = handle.numeric(tA, tB, plan)                                   # a plan can be reused
    assert_matches_oracle(C2, ref, "numeric phase, second use of the plan")
    C.free(); C2.free(); plan.free(); tA.free()
    if not same:
        tB.free()


# ------------------------------------------------------------------ block products without the matrix cores
@pytest.fixture
def vector_handle(tsp):
    """A handle whose multiplication pass runs on the vector ALUs (paper Section 5, the comparison
    build without tensor cores, Algorithm 2)."""
    h = tsp.Handle(validate=True)
    h.set_option(tsp.OPT_MATRIX_CORES, 0)
    yield h
    h.close()


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_vector_alu_numeric_small_configs(tsp, vector_handle, oracle, index):
    A = inputs.config(index, small=True)
    print(f"vector ALU, config {index} small: {A.name} rows={A.rows} nnz={A.nnz}", flush=True)
    run_and_check(tsp, vector_handle, oracle, A)


def test_vector_alu_numeric_rectangular_long_segments_and_subnormals(tsp, vector_handle, oracle):
    A = inputs.random_sparse(200, 1500, 0.2, 31, empty_row_fraction=0.1, values="uniform")   # segments > 64 entries
    B = inputs.random_sparse(1500, 90, 0.2, 32, empty_row_fraction=0.1, values="uniform")
    print("vector ALU, 200x1500x90", flush=True)
    run_and_check(tsp, vector_handle, oracle, A, B)
    T1 = inputs.random_sparse(64, 64, 0.2, 31, values="tiny")        # fp16 subnormals must not be flushed
    T2 = inputs.random_sparse(64, 64, 0.2, 32, values="smallint")
    print("vector ALU, subnormal inputs", flush=True)
    _, ref = run_and_check(tsp, vector_handle, oracle, T1, T2)
    assert (ref.mag > 1e-6).sum() > 100


def test_vector_alu_and_matrix_core_patterns_agree(tsp, handle, vector_handle):
    A = inputs.config(5, small=True)
    dA = tsp.to_device(A)
    C1, C2 = handle.spgemm(dA, dA), vector_handle.spgemm(dA, dA)
    r1, c1, v1 = C1.to_host()
    r2, c2, v2 = C2.to_host()
    C1.free()
    C2.free()
    assert np.array_equal(r1, r2) and np.array_equal(c1, c2)
    assert np.allclose(v1, v2, rtol=1e-4, atol=1e-6)


# ------------------------------------------------------------------ compaction of zeros (Section 4.4)
def _assert_same_csr(C, want, what):
    row_ptr, col, val = C.to_host()
    assert np.array_equal(row_ptr, want.row_ptr), f"{what}: row_ptr differs"
    assert np.array_equal(col, want.col), f"{what}: col_idx differs"
    assert np.array_equal(val.astype(np.float64), want.val), f"{what}: values differ"


@pytest.mark.parametrize("M,K,N,density,seed", [
    (23, 31, 17, 0.3, 1), (300, 200, 500, 0.05, 2), (64, 2000, 64, 0.1, 3), (1, 1, 1, 1.0, 4),
    # rows of thousands of entries (the block takes them one after the other), next to short ones and a ragged last block
    (40, 30, 5000, 0.4, 5), (50, 8, 9000, 0.3, 6)])
def test_compact_zeros_small_integers(tsp, handle, oracle, M, K, N, density, seed):
    """Small-integer values: all sums are exact in fp32 and fp64, so both sides drop the same entries."""
    A = inputs.random_sparse(M, K, density, seed, empty_row_fraction=0.1, values="smallint")
    B = inputs.random_sparse(K, N, density, seed + 9, empty_row_fraction=0.1, values="smallint")
    print(f"compaction {M}x{K}x{N}", flush=True)
    dA, dB = tsp.to_device(A), tsp.to_device(B)
    C = handle.spgemm(dA, dB)
    ref = oracle.spgemm(A, B)
    want = oracle.compact_zeros(ref)
    D = handle.compact_zeros(C)
    try:
        assert C.nnz == ref.nnz and D.nnz == want.nnz
        _assert_same_csr(D, want, "tsp_compact_zeros")
    finally:
        C.free()
        D.free()


def test_compact_zeros_option_cancellation_stored_zeros_and_empty(tsp, oracle):
    h = tsp.Handle(validate=True)
    h.set_option(tsp.OPT_COMPACT_ZEROS, 1)
    try:
        A = inputs.from_coo(2, 2, [0, 0, 1, 1], [0, 1, 0, 1], [1.0, -1.0, 2.0, 0.0], name="cancel")
        B = inputs.from_coo(2, 2, [0, 0, 1, 1], [0, 1, 0, 1], [1.0, 1.0, 1.0, 1.0], name="ones")
        C = h.spgemm(tsp.to_device(A), tsp.to_device(B))
        _assert_same_csr(C, oracle.compact_zeros(oracle.spgemm(A, B)), "option, worked example")
        assert C.nnz == 2
        C.free()
        # 0/1 matrix: nothing cancels, the option changes nothing
        G = inputs.rmat(9, 8, seed=6)
        dG = tsp.to_device(G)
        C = h.spgemm(dG, dG)
        ref = oracle.spgemm(G, G)
        assert C.nnz == ref.nnz
        _assert_same_csr(C, oracle.compact_zeros(ref), "option, 0/1 matrix")
        C.free()
        # all-zero values: every row becomes empty
        Z = inputs.random_sparse(50, 50, 0.2, 8, values="ones")
        Z.val[:] = 0
        dZ = tsp.to_device(Z)
        C = h.spgemm(dZ, dZ)
        assert C.nnz == 0 and int(C.row_ptr.abs().sum()) == 0
        C.free()
        # empty operands
        E = inputs.random_sparse(40, 30, 0.0, 9)
        F = inputs.random_sparse(30, 20, 0.3, 10)
        C = h.spgemm(tsp.to_device(E), tsp.to_device(F))
        assert C.nnz == 0 and (C.rows, C.cols) == (40, 20)
        C.free()
    finally:
        h.close()


def test_compact_zeros_on_a_caller_matrix_with_int32_row_ptr(tsp, handle):
    import torch
    rng = np.random.default_rng(12)
    rows, cols = 1000, 777
    lens = rng.integers(0, 40, rows)
    row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    nnz = int(row_ptr[-1])
    col = np.concatenate([np.sort(rng.choice(cols, n, replace=False)) for n in lens]).astype(np.int32)
    val = rng.integers(-1, 2, nnz).astype(np.float32)          # about a third zeros, some of them -0.0
    val[::7] = -0.0
    val[5] = np.nan
    C = tsp.DeviceCSR(rows, cols, torch.from_numpy(row_ptr).cuda(), torch.from_numpy(col).cuda(),
                      torch.from_numpy(val).cuda())
    D = handle.compact_zeros(C)
    keep = ~(val == 0.0)
    want_ptr = np.concatenate([[0], np.cumsum(keep)])[row_ptr]
    rp, c, v = D.to_host()
    D.free()
    assert np.array_equal(rp, want_ptr) and np.array_equal(c, col[keep])
    assert np.array_equal(v.view(np.uint32), val[keep].view(np.uint32))


def test_compact_zeros_with_more_rows_than_one_prefix_sum_launch_covers(tsp, handle):
    """600,000 rows (the one-launch prefix sum stops at 524,288): the new row_ptr comes from the three-kernel
    scan.  Rows of 0 to 3 entries, a ragged last group of rows, expected result from the definition."""
    import torch
    rng = np.random.default_rng(13)
    rows, cols = 600_003, 50
    lens = rng.integers(0, 4, rows)
    row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    nnz = int(row_ptr[-1])
    first = rng.integers(0, cols - 3, rows)
    col = (np.repeat(first, lens) + (np.arange(nnz) - np.repeat(row_ptr[:-1], lens))).astype(np.int32)
    val = rng.integers(-1, 2, nnz).astype(np.float32)
    C = tsp.DeviceCSR(rows, cols, torch.from_numpy(row_ptr).cuda(), torch.from_numpy(col).cuda(),
                      torch.from_numpy(val).cuda())
    D = handle.compact_zeros(C)
    keep = ~(val == 0.0)
    want_ptr = np.concatenate([[0], np.cumsum(keep)])[row_ptr]
    rp, c, v = D.to_host()
    D.free()
    assert np.array_equal(rp, want_ptr) and np.array_equal(c, col[keep]) and np.array_equal(v, val[keep])


# ------------------------------------------------------------------ precision study (Section 6.4, Eq. 3)
def test_smape_against_full_precision_as_in_the_paper(tsp, handle, oracle):
    """The paper's two observations on synthetic inputs: 0/1 patterns give SMAPE 0 %; real
    fp32 inputs, rounded to fp16 on the device, give a SMAPE of a few hundredths of a percent
    against a full-precision product of the unrounded values."""
    import torch
    G = inputs.rmat(10, 8, seed=3)
    C = handle.spgemm(tsp.to_device(G), tsp.to_device(G))
    _, _, val = C.to_host()
    C.free()
    assert oracle.smape_percent(oracle.spgemm(G, G, full_precision=True).val, val) == 0.0

    rng = np.random.default_rng(63)
    A = inputs.random_sparse(700, 700, 0.02, 41)
    A32 = inputs.CSRMatrix(A.rows, A.cols, A.row_ptr, A.col_idx, rng.uniform(-1, 1, A.nnz).astype(np.float32), "fp32")
    dA = tsp.DeviceCSR(A.rows, A.cols, torch.from_numpy(A32.row_ptr.astype(np.int32)).cuda(),
                       torch.from_numpy(A32.col_idx.astype(np.int32)).cuda(), torch.from_numpy(A32.val).cuda())
    C = handle.spgemm(dA, dA)
    full = oracle.spgemm(A32, A32, full_precision=True)
    assert_matches_oracle(C, oracle.spgemm(A32, A32), "fp32 inputs")     # parity with the fp16-rounded oracle
    _, col, val = C.to_host()
    C.free()
    assert np.array_equal(col, full.col)
    s = oracle.smape_percent(full.val, val)
    print(f"SMAPE against full precision: {s:.4f} %", flush=True)
    assert 0.0 < s < 0.1


# ------------------------------------------------------------------ tile-rows of C wider than the LDS window
@pytest.mark.parametrize("M,K,N,da,db", [(40, 64, 70000, 0.5, 0.05), (40, 1024, 70000, 0.1, 0.004)])
def test_tile_rows_with_more_output_tiles_than_the_symbolic_window(tsp, handle, oracle, M, K, N, da, db):
    """4375 output tiles per tile-row, more than one window of the general task-list kernel holds (4096): such
    a tile-row is worked off window by window (one chunk of A tiles in the first case, several in the second)."""
    A = inputs.random_sparse(M, K, da, 71, values="smallint")
    B = inputs.random_sparse(K, N, db, 72, values="smallint")
    print(f"wide output tile-rows {M}x{K}x{N}", flush=True)
    dA, dB = tsp.to_device(A), tsp.to_device(B)
    C = handle.spgemm(dA, dB)
    st = handle.stats()
    assert st["c_tiles"] > 3 * 4096
    ref = oracle.spgemm(A, B, threads=4)
    assert_matches_oracle(C, ref, "wide output tile-rows")
    C.free()


# ------------------------------------------------------------------ more rows than the one-launch row_ptr covers
def test_band_matrix_with_600000_rows(tsp, handle, oracle):
    """Beyond 524,288 rows row_ptr of C comes from the three-kernel scan instead of the one-launch prefix sum,
    and the sizing scan chains several dozen blocks.  A band matrix keeps the oracle's work small."""
    n = 600_007
    i = np.arange(n)
    rng = np.random.default_rng(600)
    rows = np.concatenate([i, i[:-1], i[1:], i[:-5]])
    cols = np.concatenate([i, i[:-1] + 1, i[1:] - 1, i[:-5] + 5])
    A = inputs.from_coo(n, n, rows, cols, rng.uniform(-1, 1, rows.size), "band 600007")
    print(f"{A.name}: nnz {A.nnz}", flush=True)
    nnz, _ = run_and_check(tsp, handle, oracle, A)
    assert nnz > 2 * A.nnz


# ------------------------------------------------------------------ two tile-rows per wave in the counting kernel
def test_short_tile_rows_against_a_wide_operand(tsp, handle, oracle):
    """Short tile-rows of A against a B too wide for the counting kernel's whole-grid bitmap: the kernel
    that gives each tile-row half a wave.  An odd number of tile-rows (the last half-wave idles), empty
    tile-rows, rows whose candidates lie far apart, and a B with empty tile-rows."""
    rng = np.random.default_rng(123)
    M, K = 16 * 201 - 5, 1 << 18
    rows = np.repeat(np.arange(M), 3)
    cols = rng.integers(0, K, rows.size)
    keep = (rows // 16) % 7 != 3                                       # every seventh tile-row of A empty
    keys = np.unique(rows[keep] * K + cols[keep])
    A = inputs.from_coo(M, K, keys // K, keys % K, rng.uniform(-1, 1, keys.size), "short rows, wide inner dimension")
    i = np.arange(K)
    band = np.concatenate([i, i[:-1], i[1:], i[: K - 700]])
    bcol = np.concatenate([i, i[:-1] + 1, i[1:] - 1, i[: K - 700] + 700])
    live = (band // 16) % 5 != 2                                       # every fifth tile-row of B empty
    B = inputs.from_coo(K, K, band[live], bcol[live], rng.uniform(-1, 1, int(live.sum())), "band")
    print(f"short tile-rows: A {A.rows}x{A.cols} nnz {A.nnz}, B nnz {B.nnz}", flush=True)
    nnz, _ = run_and_check(tsp, handle, oracle, A, B)
    assert nnz > A.nnz
    # enough short tile-rows for the task-list kernel to run the counting pass itself, two tile-rows per
    # wave: 1073 tile-rows, an odd number, the last one ragged
    L = inputs.laplacian_2d(131)
    print(f"short tile-rows: {L.name} rows {L.rows}", flush=True)
    run_and_check(tsp, handle, oracle, L)


def test_short_tile_rows_against_a_very_wide_operand(tsp, handle, oracle):
    """B wider than half a million columns: the counting kernel keeps a tile-row's bitmap in segments of
    1024 tile columns, 16 per tile-row.  Even tile-rows of A are clustered (a few segments), odd ones are
    scattered over more segments than a tile-row may hold and are left to the kernel with the full bitmap."""
    rng = np.random.default_rng(321)
    K = 1 << 20
    tile_rows = 151
    M = 16 * tile_rows - 3
    rows = np.repeat(np.arange(M), 3)
    centre = rng.integers(100, K - 100, tile_rows)                       # one cluster per tile-row
    clustered = centre[rows // 16] + rng.integers(-40, 40, rows.size)
    scattered = rng.integers(0, K, rows.size)
    cols = np.where((rows // 16) % 2 == 0, clustered, scattered)
    keys = np.unique(rows * K + cols)
    A = inputs.from_coo(M, K, keys // K, keys % K, rng.uniform(-1, 1, keys.size), "clustered and scattered tile-rows")
    i = np.arange(K)
    band = np.concatenate([i, i[:-1], i[1:]])
    bcol = np.concatenate([i, i[:-1] + 1, i[1:] - 1])
    B = inputs.from_coo(K, K, band, bcol, rng.uniform(-1, 1, band.size), "band 2^20")
    print(f"very wide operand: A {A.rows}x{A.cols} nnz {A.nnz}, B nnz {B.nnz}", flush=True)
    nnz, _ = run_and_check(tsp, handle, oracle, A, B)
    assert nnz > A.nnz


def test_many_short_tile_rows_whose_candidates_span_two_million_columns(tsp, handle, oracle):
    """More than 1024 tile-rows of A with a few dozen candidate pairs each (the task-list kernel that also
    runs the counting pass, two tile-rows per wave), against a B whose entries sit at both ends of two
    million columns: the bitmap of a tile-row takes nearly 4096 words, two of them no longer fit the
    64 KB of LDS a launch may ask for, and the kernel takes one tile-row per block instead."""
    rng = np.random.default_rng(99)
    M, K, N = 16 * 1025, 200, 2_000_000
    A = inputs.from_coo(M, K, np.arange(M), rng.integers(0, K, M), rng.uniform(-1, 1, M), "one entry per row")
    k = np.arange(K)
    brow = np.concatenate([k, k])
    bcol = np.concatenate([rng.integers(0, 300, K), N - 1 - rng.integers(0, 300, K)])
    B = inputs.from_coo(K, N, brow, bcol, rng.uniform(-1, 1, 2 * K), "both ends of two million columns")
    print(f"wide bitmaps: A {A.rows}x{A.cols} nnz {A.nnz}, B nnz {B.nnz}", flush=True)
    nnz, _ = run_and_check(tsp, handle, oracle, A, B)
    assert nnz == 2 * M


# ------------------------------------------------------------------ heaviest tile-rows first
def test_tile_rows_taken_in_order_of_work(tsp, oracle):
    """The general task-list kernel with its blocks taking the tile-rows heaviest first (forced here; on
    its own the library does that only for large skewed products): a power-law graph, whose hub
    tile-rows are spread over the index range, and a wide product with more tile-rows than one block of
    the ordering kernels covers.  Same result as by index, and as the oracle's."""
    ordered = _variant_handle(tsp, OPT_WORK_ORDER=1)
    by_index = _variant_handle(tsp, OPT_WORK_ORDER=2)
    try:
        G = inputs.rmat(scale=11, edge_factor=12, seed=2024)
        print(f"work order: R-MAT scale 11, nnz {G.nnz}", flush=True)
        dG = tsp.to_device(G)
        C1 = ordered.spgemm(dG, dG)
        assert ordered.stats()["pairs"] > 0
        C2 = by_index.spgemm(dG, dG)
        for x, y in zip(C1.to_host(), C2.to_host()):
            assert np.array_equal(x, y)
        # the same product again: the counting kernel now takes the tile-rows in the order the handle has kept
        # from the first call, and keeps bitmaps and pair counts for the task-list kernel
        C3 = ordered.spgemm(dG, dG)
        for x, y in zip(C1.to_host(), C3.to_host()):
            assert np.array_equal(x, y)
        C3.free()
        assert_matches_oracle(C1, oracle.spgemm(G, G, threads=4), "R-MAT, heaviest tile-rows first")
        C1.free()
        C2.free()
        # 18000 rows: 1125 tile-rows (two blocks of the ordering kernels, the second ragged), of which one
        # in 50 is heavy; a tile-row with thousands of candidate pairs keeps the list kernel out
        rng = np.random.default_rng(91)
        M, K, N = 18000, 600, 3000
        heavy = np.arange(0, M, 50 * 16)[:, None] + np.arange(16)[None, :]
        heavy = heavy[heavy < M]
        rows = np.concatenate([np.repeat(np.arange(M), 2), np.repeat(heavy, 200)])
        cols = np.concatenate([rng.integers(0, K, 2 * M), rng.integers(0, K, 200 * heavy.size)])
        keys = np.unique(rows * K + cols)                                  # no duplicate positions
        rows, cols = keys // K, keys % K
        A = inputs.from_coo(M, K, rows, cols, rng.integers(1, 4, rows.size).astype(np.float64), "skewed rows")
        B = inputs.random_sparse(K, N, 0.05, 92, values="smallint")
        print(f"work order: skewed {M}x{K}x{N}, nnz(A) {A.nnz}", flush=True)
        run_and_check(tsp, ordered, oracle, A, B)
    finally:
        ordered.close()
        by_index.close()


def test_tile_rows_with_very_many_candidates_take_larger_blocks(tsp, oracle):
    """Nearly every tile-row of A meets every tile-row of B in full: about 127 x 127 candidate pairs per
    tile-row, above the 8192 from which the general task-list kernel runs in blocks of 512 threads; so does the counting
    kernel on the second call of the same product, when it keeps the bitmaps and the pairs per tile
    column for the task-list kernel.  Both calls against the oracle."""
    h = tsp.Handle(validate=True)
    try:
        A = inputs.random_sparse(2048, 2048, 0.02, 4711, values="smallint")
        print(f"very many candidates: 2048^2, nnz {A.nnz}", flush=True)
        dA = tsp.to_device(A)
        ref = oracle.spgemm(A, A, threads=4)
        for call in (1, 2):
            C = h.spgemm(dA, dA)
            st = h.stats()
            assert st["candidate_pairs"] >= 8192 * 128, st["candidate_pairs"]
            assert_matches_oracle(C, ref, f"dense tile grid, call {call}")
            C.free()
    finally:
        h.close()


# ------------------------------------------------------------------ output tiles taken in vertical strips
def test_output_tiles_taken_in_vertical_strips(tsp, oracle):
    """The counting and the multiplication kernel with their workgroups taking the output tiles strip by
    strip (forced here, with strips of a few dozen tiles of B; on its own the library does that only for
    large products with long tile-rows): same result, bit for bit, as row-major, and as the oracle's.
    A power-law graph (general task-list kernel and separate counting kernel), a stencil (list kernel with
    the counting pass fused: only the multiplication kernel takes the strips), a rectangular product,
    also with 64-bit addressing and on the vector ALUs."""
    cases = [
        ("R-MAT scale 11", inputs.rmat(scale=11, edge_factor=12, seed=2024), None, {}),
        ("R-MAT scale 10, wide index", inputs.rmat(scale=10, edge_factor=16, seed=5), None, {"OPT_WIDE_INDEX": 1}),
        ("stencil", inputs.config(3, small=True), None, {}),
        ("rectangular", inputs.random_sparse(300, 170, 0.06, 31, empty_row_fraction=0.1),
         inputs.random_sparse(170, 1500, 0.05, 32), {}),
        ("rectangular, vector ALUs", inputs.random_sparse(200, 90, 0.1, 33), inputs.random_sparse(90, 900, 0.08, 34),
         {"OPT_MATRIX_CORES": 0}),
    ]
    for name, A, B, extra in cases:
        for per_strip in (16, 57, 1):
            striped = _variant_handle(tsp, OPT_STRIP_ORDER=per_strip, OPT_NUMERIC_RUN=4, **extra)
            row_major = _variant_handle(tsp, OPT_STRIP_ORDER=2, OPT_NUMERIC_RUN=4, **extra)
            try:
                print(f"strips: {name}, {per_strip} tiles of B per strip", flush=True)
                dA = tsp.to_device(A)
                dB = dA if B is None else tsp.to_device(B)
                C1 = striped.spgemm(dA, dB)
                C2 = row_major.spgemm(dA, dB)
                for x, y in zip(C1.to_host(), C2.to_host()):
                    assert np.array_equal(x, y)
                assert_matches_oracle(C1, oracle.spgemm(A, A if B is None else B, threads=4), f"{name}, strips")
                C1.free()
                C2.free()
            finally:
                striped.close()
                row_major.close()


# ------------------------------------------------------------------ variants of the multiplication kernel
def _variant_handle(tsp, **options):
    h = tsp.Handle(validate=True)
    for name, value in options.items():
        h.set_option(getattr(tsp, name), value)
    return h


def _mesh_cases():
    """Products whose tile-rows of C are short and sparse (at most 60 output tiles, 64 task-list entries
    and 448 entries per tile-row): the multiplication kernel takes a whole tile-row per wave and
    assembles its output in LDS.  Grid edges that are no multiple of 16 give ragged last tile-rows."""
    yield "laplacian 37x37", inputs.laplacian_2d(37), None
    yield "laplacian 64x64", inputs.laplacian_2d(64), None
    yield "laplacian 13x13x13", inputs.laplacian_3d(13), None      # about 20 output tiles per tile-row
    # one inner tile column; 16, 60 and 61 output tiles per tile-row: inside and either side of the limit
    for n_cols, density in ((256, 0.1), (960, 0.025), (976, 0.025)):
        A = inputs.random_sparse(70, 16, 0.07, 91, empty_row_fraction=0.2)
        B = inputs.random_sparse(16, n_cols, density, 92)
        yield f"single inner tile, {n_cols} columns", A, B
    # entries per tile-row either side of 448
    for density in (0.10, 0.12):
        A = inputs.random_sparse(64, 16, 0.0625, 93)
        B = inputs.random_sparse(16, 256, density, 94, values="smallint")
        yield f"single inner tile, density {density}", A, B


@pytest.mark.parametrize("options", [
    {},                                             # automatic choice
    {"OPT_WIDE_INDEX": 1},                          # 64-bit addressing, as for arrays of 4 GiB and more
    {"OPT_NUMERIC_RUN": 4},                         # four tiles per wave whatever the shape of the tile-rows
    {"OPT_NUMERIC_RUN": 8},
    {"OPT_NUMERIC_RUN": 8, "OPT_WIDE_INDEX": 1},
], ids=lambda o: "+".join(f"{k}={v}" for k, v in o.items()) or "automatic")
def test_multiplication_kernel_variants(tsp, oracle, options):
    h = _variant_handle(tsp, **options)
    try:
        for what, A, B in _mesh_cases():
            print(f"{options}: {what}", flush=True)
            run_and_check(tsp, h, oracle, A, B)
        for index in (1, 3, 5):
            A = inputs.config(index, small=True)
            print(f"{options}: config {index} small", flush=True)
            run_and_check(tsp, h, oracle, A)
    finally:
        h.close()


# ------------------------------------------------------------------ a seeded sweep of shapes and densities
def _sweep_cases():
    """Forty products drawn from one seeded generator: sizes from one tile to a few hundred rows, ragged
    edges, densities from almost empty to almost full, empty rows, square and rectangular, the value
    kinds of inputs.random_sparse, and the input types the boundary accepts."""
    rng = np.random.default_rng(20260914)
    for case in range(40):
        M, K, N = (int(x) for x in rng.integers(1, 330, size=3))
        density = float(10.0 ** rng.uniform(-2.5, -0.05))
        kind = ("uniform", "smallint", "ones", "tiny")[int(rng.integers(0, 4))]
        empty = float(rng.choice([0.0, 0.1, 0.5]))
        upload = {"value_dtype": ("f16", "f32")[int(rng.integers(0, 2))],
                  "row_ptr_dtype": ("i32", "i64")[int(rng.integers(0, 2))]}
        yield case, M, K, N, density, kind, empty, upload


def test_seeded_sweep_of_small_products(tsp, handle, oracle):
    for case, M, K, N, density, kind, empty, upload in _sweep_cases():
        A = inputs.random_sparse(M, K, density, 7000 + case, empty_row_fraction=empty, values=kind)
        B = inputs.random_sparse(K, N, density, 8000 + case, empty_row_fraction=empty, values=kind)
        print(f"sweep {case}: {M}x{K}x{N} d={density:.4f} {kind} empty={empty} {upload}", flush=True)
        run_and_check(tsp, handle, oracle, A, B, **upload)


def test_seeded_sweep_with_hub_rows_wide_outputs_and_repeated_calls(tsp, oracle):
    """Forty-eight products of four kinds (square with hub rows and a dense tile grid, which take the general
    task-list kernel; a few rows times a very wide B, whose tile-rows of C pass the symbolic window; tall and
    thin; small and ragged), each multiplied twice on one handle: the second call of a product takes what the
    handle has kept from the first (bitmaps and pair counts from the counting kernel, the order of work)."""
    def make(rng, M, K, d, hubs, name):
        mask = rng.random((M, K)) < d
        for _ in range(hubs):
            mask[rng.integers(0, M)] |= rng.random(K) < min(1.0, 40 * d + 0.2)
        r, c = np.nonzero(mask)
        v = rng.integers(1, 4, r.size).astype(np.float64) if rng.random() < 0.5 else rng.uniform(-1, 1, r.size)
        return inputs.from_coo(M, K, r, c, v, name)

    h = tsp.Handle(validate=True)
    try:
        for case in range(48):
            rng = np.random.default_rng(31_000 + case)
            kind = case % 4
            if kind == 0:
                M = K = N = int(rng.integers(200, 2500))
                da = db = float(10 ** rng.uniform(-2.5, -1.2))
                hubs = int(rng.integers(0, 6))
            elif kind == 1:
                M, K, N = int(rng.integers(1, 300)), int(rng.integers(16, 1500)), int(rng.integers(20000, 90000))
                da, db = float(10 ** rng.uniform(-1.5, -0.3)), float(10 ** rng.uniform(-3.2, -2.0))
                hubs = int(rng.integers(0, 3))
            elif kind == 2:
                M, K, N = int(rng.integers(1000, 20000)), int(rng.integers(1, 200)), int(rng.integers(1, 400))
                da, db = float(10 ** rng.uniform(-2.5, -1)), float(10 ** rng.uniform(-2, -0.5))
                hubs = int(rng.integers(0, 3))
            else:
                M, K, N = (int(x) for x in rng.integers(1, 200, 3))
                da = db = float(10 ** rng.uniform(-2, -0.2))
                hubs = 0
            A = make(rng, M, K, da, hubs, f"A{case}")
            B = A if (kind == 0 and rng.random() < 0.5) else make(rng, K, N, db, hubs, f"B{case}")
            print(f"sweep {case} kind {kind}: {M}x{K}x{B.cols} nnz {A.nnz}, {B.nnz}", flush=True)
            ref = oracle.spgemm(A, B, threads=4)
            dA = tsp.to_device(A)
            dB = dA if B is A else tsp.to_device(B)
            for call in (1, 2):
                C = h.spgemm(dA, dB)
                assert_matches_oracle(C, ref, f"sweep {case}, call {call}")
                C.free()
    finally:
        h.close()


def test_mesh_with_dense_rows(tsp, handle, oracle):
    """A few full rows in an otherwise short-rowed matrix (a constraint row in a mesh problem): their
    tile-rows have far more tiles than a window of the converter and of the task-list kernel holds and go
    through the window-by-window paths of both, inside kernels chosen for the short rows."""
    L = inputs.laplacian_2d(48)
    n = L.rows
    rows = np.repeat(np.arange(n), np.diff(L.row_ptr))
    cols, vals = L.col_idx.astype(np.int64), L.val.astype(np.float64)
    rng = np.random.default_rng(5)
    dense = (7, n // 2 + 3, n - 1)
    keep = ~np.isin(rows, dense)
    rows = np.concatenate([rows[keep]] + [np.full(n, r) for r in dense])
    cols = np.concatenate([cols[keep]] + [np.arange(n) for _ in dense])
    vals = np.concatenate([vals[keep]] + [rng.uniform(-1, 1, n) for _ in dense])
    A = inputs.from_coo(n, n, rows, cols, vals, "laplacian_with_dense_rows")
    nnz, _ = run_and_check(tsp, handle, oracle, A)
    assert nnz > 3 * n
    B = inputs.random_sparse(n, 90, 0.02, 77)
    run_and_check(tsp, handle, oracle, A, B)


@pytest.mark.parametrize("n", [20000, 40000])
def test_band_with_dense_rows(tsp, handle, oracle, n):
    """The same in a band matrix, whose tile-rows the converter gives one wave each: the full rows
    (1250 and 2500 tiles) go window by window inside the kernel built for two entries per lane."""
    i = np.arange(n)
    rng = np.random.default_rng(n)
    dense = (5, n - 40)
    rows = np.concatenate([i, i[:-1], i[1:]])
    cols = np.concatenate([i, i[:-1] + 1, i[1:] - 1])
    keep = ~np.isin(rows, dense)
    rows = np.concatenate([rows[keep]] + [np.full(n, r) for r in dense])
    cols = np.concatenate([cols[keep]] + [i for _ in dense])
    A = inputs.from_coo(n, n, rows, cols, rng.uniform(-1, 1, rows.size), f"band with dense rows {n}")
    print(f"{A.name}: nnz {A.nnz}", flush=True)
    nnz, _ = run_and_check(tsp, handle, oracle, A)
    assert nnz > 2 * n
