"""Pins for the oracle's intermediate objects (bitmap format, task list, counting) against
the dense definition, for the paper's tile edge 8 and the GPU path's 16.  No GPU."""
import numpy as np
import pytest

from paper_2009_14600_amd import inputs
from tests.dense_check import brute_force_product, densify

CASES = [
    (lambda: inputs.random_sparse(37, 29, 0.12, 21, empty_row_fraction=0.2),
     lambda: inputs.random_sparse(29, 45, 0.10, 22, empty_row_fraction=0.2)),
    (lambda: inputs.random_sparse(64, 64, 0.03, 23), lambda: inputs.random_sparse(64, 64, 0.03, 24)),
    (lambda: inputs.laplacian_2d(7), lambda: inputs.laplacian_2d(7)),
    (lambda: inputs.block_clustered(96, 2, 0.5, 16, seed=3), lambda: inputs.block_clustered(96, 2, 0.5, 16, seed=4)),
]


def _tile_dense(bm, t):
    T = bm.T
    out = np.zeros((T, T))
    pat = np.zeros((T, T), dtype=bool)
    e = int(bm.index[t])
    for r in range(T):
        for c in range(T):
            if (int(bm.row_mask[t, r]) >> c) & 1:
                out[r, c] = float(bm.elements[e])
                pat[r, c] = True
                e += 1
    assert e == int(bm.index[t + 1])
    return out, pat


@pytest.mark.parametrize("T", [4, 8, 16])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_bitmap_format_round_trip(oracle, case, T):
    A = CASES[case][0]()
    bm = oracle.bitmap_format(A, T)
    d, p = densify(A)
    dense = np.zeros((bm.tile_rows * T, bm.tile_cols * T))
    pat = np.zeros(dense.shape, dtype=bool)
    key = bm.tile_row * bm.tile_cols + bm.tile_col
    assert np.all(np.diff(key) > 0)                       # COO of tiles, row-major, no duplicates
    for t in range(key.shape[0]):
        td, tp = _tile_dense(bm, t)
        assert tp.any()                                    # only non-empty tiles are kept
        i, j = int(bm.tile_row[t]) * T, int(bm.tile_col[t]) * T
        dense[i:i + T, j:j + T] = td
        pat[i:i + T, j:j + T] = tp
    assert np.array_equal(dense[:A.rows, :A.cols], d) and np.array_equal(pat[:A.rows, :A.cols], p)
    assert not pat[A.rows:].any() and not pat[:, A.cols:].any()
    assert int(bm.index[-1]) == A.nnz


@pytest.mark.parametrize("T", [8, 16])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_task_list_and_counting_against_dense(oracle, case, T):
    A, B = CASES[case][0](), CASES[case][1]()
    TA, TB = oracle.bitmap_format(A, T), oracle.bitmap_format(B, T)
    tl = oracle.task_list(TA, TB)
    _, pa = densify(A)
    _, pb = densify(B)
    ntr, ntk, ntc = TA.tile_rows, TA.tile_cols, TB.tile_cols
    PA = np.zeros((ntr * T, ntk * T), dtype=bool)
    PA[:A.rows, :A.cols] = pa
    PB = np.zeros((ntk * T, ntc * T), dtype=bool)
    PB[:B.rows, :B.cols] = pb
    expect = []          # (I, J, K) with a non-zero boolean tile product, row-major in (I,J), K ascending
    candidates = 0
    for I in range(ntr):
        for J in range(ntc):
            for K in range(ntk):
                a = PA[I * T:(I + 1) * T, K * T:(K + 1) * T]
                b = PB[K * T:(K + 1) * T, J * T:(J + 1) * T]
                if a.any() and b.any():
                    candidates += 1
                    if (a.astype(int) @ b.astype(int)).any():
                        expect.append((I, J, K))
    got = [(int(TA.tile_row[a]), int(TB.tile_col[b]), int(TA.tile_col[a]))
           for a, b in zip(tl.a_tile, tl.b_tile)]
    assert got == expect
    assert all(int(TA.tile_col[a]) == int(TB.tile_row[b]) for a, b in zip(tl.a_tile, tl.b_tile))
    assert tl.candidates == candidates
    cij = sorted({(i, j) for i, j, _ in expect})
    assert list(zip(tl.c_tile_row.tolist(), tl.c_tile_col.tolist())) == cij
    assert tl.offsets[0] == 0 and tl.offsets[-1] == len(expect)
    for c, (i, j) in enumerate(cij):
        assert tl.offsets[c + 1] - tl.offsets[c] == sum(1 for e in expect if e[:2] == (i, j))
    # counting kernel: the accumulated boolean products are exactly the structural pattern of C
    masks, counts = oracle.counting(TA, TB, tl)
    _, _, pat = brute_force_product(A, B)
    PC = np.zeros((ntr * T, ntc * T), dtype=bool)
    PC[:A.rows, :B.cols] = pat
    for c, (i, j) in enumerate(cij):
        block = PC[i * T:(i + 1) * T, j * T:(j + 1) * T]
        got_block = np.array([[(int(masks[c, r]) >> cc) & 1 for cc in range(T)] for r in range(T)], dtype=bool)
        assert np.array_equal(got_block, block) and counts[c] == block.sum() > 0
        PC[i * T:(i + 1) * T, j * T:(j + 1) * T] = False
    assert not PC.any()                                    # every structural entry lies in a listed C tile
    res = oracle.spgemm(A, B)
    assert counts.sum() == res.nnz
