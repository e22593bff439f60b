"""Pins for the CPU oracle: brute force, closed forms, invariants.  No GPU, no HIP library.

The paper prints no worked numeric example in its text (its Fig. 1 example is an image), so
the oracle is pinned by the definition of the sparse product (Section 2.2) evaluated by brute
force, by closed forms, and by identities that hold at any size.
"""
import numpy as np
import pytest

from paper_2009_14600_amd import inputs
from tests.dense_check import brute_force_product, densify, oracle_to_dense


# ---------------------------------------------------------------- brute force, tiny inputs
@pytest.mark.parametrize("M,K,N,density,seed,kind", [
    (1, 1, 1, 1.0, 1, "uniform"),
    (7, 5, 9, 0.4, 2, "uniform"),
    (33, 17, 40, 0.15, 3, "uniform"),
    (40, 40, 40, 0.1, 4, "smallint"),
    (20, 64, 13, 0.3, 5, "tiny"),
    (48, 31, 50, 0.08, 6, "ones"),
    (5, 0, 4, 0.5, 7, "uniform"),
    (0, 4, 4, 0.5, 8, "uniform"),
])
def test_brute_force_dense(oracle, M, K, N, density, seed, kind):
    A = inputs.random_sparse(M, K, density, seed, empty_row_fraction=0.2, values=kind)
    B = inputs.random_sparse(K, N, density, seed + 100, empty_row_fraction=0.2, values=kind)
    res = oracle.spgemm(A, B)
    c_ref, s_ref, pat_ref = brute_force_product(A, B)
    c, s, pat = oracle_to_dense(res, M, N)
    assert np.array_equal(pat, pat_ref)
    # both sum exact fp64 products of fp16 numbers; only the order of additions may differ
    np.testing.assert_allclose(c, c_ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(s, s_ref, rtol=1e-13, atol=0)
    for i in range(M):
        cols = res.col[res.row_ptr[i]:res.row_ptr[i + 1]]
        assert np.all(np.diff(cols) > 0)
    assert res.products == sum(int(B.row_ptr[k + 1] - B.row_ptr[k]) for k in A.col_idx)


def test_cancellation_and_stored_zero_stay_structural(oracle):
    # row 0 of A = [1, 1]; column 0 of B = [1, -1]: the sum cancels; B also stores an explicit 0.0
    A = inputs.from_coo(2, 2, [0, 0, 1], [0, 1, 1], [1.0, 1.0, 2.0])
    B = inputs.from_coo(2, 3, [0, 1, 1], [0, 0, 2], [1.0, -1.0, 0.0])
    res = oracle.spgemm(A, B)
    assert res.row_ptr.tolist() == [0, 2, 4]
    assert res.col.tolist() == [0, 2, 0, 2]
    assert res.val.tolist() == [0.0, 0.0, -2.0, 0.0]
    assert res.mag.tolist() == [2.0, 0.0, 2.0, 0.0]
    assert res.products == 5


# ---------------------------------------------------------------- fp16 decoding and rounding
def _decode_binary16(bits: int) -> float:
    """IEEE 754 binary16 from its fields, written out here so that the pin does not repeat the
    library conversion the oracle uses: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits;
    exponent field 0 = subnormal (no hidden one, exponent -14)."""
    import math
    sign = -1.0 if bits >> 15 else 1.0
    exponent, fraction = (bits >> 10) & 0x1F, bits & 0x3FF
    if exponent == 0:
        return sign * math.ldexp(fraction, -24)
    return sign * math.ldexp(1024 + fraction, exponent - 25)


def test_fp16_decode_all_bit_patterns(oracle):
    """diag(every finite fp16 bit pattern) * I: the oracle's widening of its fp16 inputs (Section
    2.6: the inputs are fp16 numbers) against a decoder by sign, exponent and fraction fields."""
    bits = np.array([b for b in range(65536) if (b >> 10) & 0x1F != 0x1F], dtype=np.uint16)   # finite ones
    n = bits.shape[0]
    assert n == 63488
    expect = np.array([_decode_binary16(int(b)) for b in bits], dtype=np.float64)
    ar = np.arange(n)
    D = inputs.CSRMatrix(n, n, np.arange(n + 1, dtype=np.int32), ar.astype(np.int32), bits.view(np.float16))
    I = inputs.CSRMatrix(n, n, np.arange(n + 1, dtype=np.int32), ar.astype(np.int32),
                         np.ones(n, dtype=np.float16))
    res = oracle.spgemm(D, I)
    assert np.array_equal(res.col, ar)
    assert np.array_equal(res.val, expect)
    nz = expect != 0          # -0.0 accumulates onto +0.0 and comes out +0.0
    assert np.array_equal(np.signbit(res.val[nz]), np.signbit(expect[nz]))
    assert np.array_equal(res.mag, np.abs(expect))
    # spot values fixed by the format itself
    assert _decode_binary16(0x3C00) == 1.0 and _decode_binary16(0x7BFF) == 65504.0
    assert _decode_binary16(0x0001) == 2.0 ** -24 and _decode_binary16(0x0400) == 2.0 ** -14
    assert _decode_binary16(0xC000) == -2.0


def test_fp32_inputs_round_to_nearest_even_fp16(oracle):
    """fp32 inputs are converted to fp16 before use (Section 2.6; Section 6.3 counts the conversion
    into the run time): round to nearest, ties to the even fraction.  Hand-picked values, each
    with the result worked out from the format (spacing 2^-10 in [1,2), 2 in [2048,4096), 2^-24
    among the subnormals)."""
    cases = [
        (1.0 + 2.0 ** -11, 1.0),                         # tie between 1 and 1+2^-10: even fraction 0
        (1.0 + 3.0 * 2.0 ** -11, 1.0 + 2.0 ** -9),       # tie between 1+2^-10 (odd) and 1+2^-9 (even)
        (1.0 + 2.0 ** -11 + 2.0 ** -20, 1.0 + 2.0 ** -10),   # just above the tie: up
        (1.0 + 2.0 ** -11 - 2.0 ** -20, 1.0),            # just below: down
        (2049.0, 2048.0),                                # tie, spacing 2: even multiple
        (2051.0, 2052.0),
        (-2049.0, -2048.0),
        (2.0 ** -25, 0.0),                               # tie between 0 and the smallest subnormal
        (3.0 * 2.0 ** -25, 2.0 ** -23),                  # tie between 2^-24 (odd) and 2^-23 (even)
        (2.0 ** -24 + 2.0 ** -26, 2.0 ** -24),           # subnormal, nearest
        (65504.0, 65504.0),                              # largest finite fp16 stays
        (0.1, 0.0999755859375),                          # 0.1 = 1.6 * 2^-4: fraction 0.6*1024 = 614.4 -> 614
        (1.0 / 3.0, 0.333251953125),                     # 1.3333 * 2^-2: fraction 341.33 -> 341
    ]
    x = np.array([c[0] for c in cases], dtype=np.float32)
    want = np.array([c[1] for c in cases], dtype=np.float64)
    n = x.shape[0]
    ar = np.arange(n, dtype=np.int32)
    D = inputs.CSRMatrix(n, n, np.arange(n + 1, dtype=np.int32), ar, x)
    I = inputs.CSRMatrix(n, n, np.arange(n + 1, dtype=np.int32), ar, np.ones(n, dtype=np.float32))
    res = oracle.spgemm(D, I)
    assert np.array_equal(res.val, want), (res.val, want)
    res = oracle.spgemm(I, D)                            # the right operand takes the same rounding
    assert np.array_equal(res.val, want)
    full = oracle.spgemm(D, I, full_precision=True)      # and the full-precision mode does not round
    assert np.array_equal(full.val, x.astype(np.float64))


# ---------------------------------------------------------------- closed forms
def _identity(n):
    return inputs.CSRMatrix(n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32),
                            np.ones(n, dtype=np.float16))


def test_identity_permutation_diagonal(oracle):
    A = inputs.random_sparse(50, 50, 0.1, 11, empty_row_fraction=0.1)
    n = A.rows
    for res in (oracle.spgemm(A, _identity(n)), oracle.spgemm(_identity(n), A)):
        assert np.array_equal(res.row_ptr, A.row_ptr.astype(np.int64))
        assert np.array_equal(res.col, A.col_idx)
        assert np.array_equal(res.val, A.val.astype(np.float64))
        assert np.array_equal(res.mag, np.abs(A.val.astype(np.float64)))
    rng = np.random.default_rng(5)
    perm = rng.permutation(n)
    P = inputs.from_coo(n, n, np.arange(n), perm, np.ones(n))      # (P A)[i,:] = A[perm[i],:]
    dA, pA = densify(A)
    c, _, pat = oracle_to_dense(oracle.spgemm(P, A), n, n)
    assert np.array_equal(pat, pA[perm]) and np.array_equal(c, dA[perm])
    c, _, pat = oracle_to_dense(oracle.spgemm(A, P), n, n)         # (A P)[:,perm[k]] = A[:,k]
    expect = np.zeros_like(dA)
    expect[:, perm] = dA
    epat = np.zeros_like(pA)
    epat[:, perm] = pA
    assert np.array_equal(pat, epat) and np.array_equal(c, expect)
    scale = 2.0 ** rng.integers(-3, 4, size=n)
    D = inputs.from_coo(n, n, np.arange(n), np.arange(n), scale)
    res = oracle.spgemm(D, A)
    rows = np.repeat(np.arange(n), np.diff(A.row_ptr))
    assert np.array_equal(res.col, A.col_idx)
    assert np.array_equal(res.val, A.val.astype(np.float64) * scale[rows])


def test_transposed_operand_would_fail(oracle):
    """A*B for non-symmetric A, B differs from B*A and from A*B^T: guards the index roles."""
    A = inputs.from_coo(3, 3, [0, 1], [1, 2], [2.0, 3.0])
    B = inputs.from_coo(3, 3, [1, 2], [0, 0], [5.0, 7.0])
    c, _, pat = oracle_to_dense(oracle.spgemm(A, B), 3, 3)
    expect = np.zeros((3, 3))
    expect[0, 0] = 10.0
    expect[1, 0] = 21.0
    assert np.array_equal(c, expect) and np.array_equal(pat, expect != 0)


def test_zero_one_inputs_count_common_neighbours(oracle):
    """0/1 inputs: c_ij is the number of common neighbours, an integer, and exact (the paper's
    SMAPE for such inputs is 0%, Section 6.4)."""
    G = inputs.rmat(8, 8, seed=77)
    res = oracle.spgemm(G, G)
    deg = np.diff(G.row_ptr).astype(np.int64)
    assert np.array_equal(res.val, np.round(res.val)) and np.array_equal(res.val, res.mag)
    rows = np.repeat(np.arange(G.rows), np.diff(res.row_ptr))
    diag = res.val[rows == res.col]
    assert np.array_equal(diag, deg[deg > 0].astype(np.float64))       # c_ii = deg(i), symmetric graph
    assert res.val.sum() == float((deg ** 2).sum()) == float(res.products)
    d, _ = densify(G)
    assert np.array_equal(oracle_to_dense(res, G.rows, G.cols)[0], d @ d)
    assert oracle.smape_percent(res.val, res.val.astype(np.float32)) == 0.0


@pytest.mark.parametrize("maker", [
    lambda: inputs.config(1, small=True), lambda: inputs.config(3, small=True),
    lambda: inputs.config(5, small=True), lambda: inputs.random_sparse(300, 300, 0.03, 9),
])
def test_checksum_identities(oracle, maker):
    """sum_ij c_ij = (1^T A)(B 1) and sum_ij s_ij = (1^T |A|)(|B| 1)."""
    A = maker()
    res = oracle.spgemm(A, A)
    v = A.val.astype(np.float64)
    col_sum = np.bincount(A.col_idx, weights=v, minlength=A.cols)
    row_sum = np.bincount(np.repeat(np.arange(A.rows), np.diff(A.row_ptr)), weights=v, minlength=A.rows)
    col_abs = np.bincount(A.col_idx, weights=np.abs(v), minlength=A.cols)
    row_abs = np.bincount(np.repeat(np.arange(A.rows), np.diff(A.row_ptr)), weights=np.abs(v),
                          minlength=A.rows)
    scale = float(col_abs @ row_abs)
    assert abs(res.val.sum() - float(col_sum @ row_sum)) <= 1e-12 * scale
    assert abs(res.mag.sum() - scale) <= 1e-12 * scale
    assert res.products == int(np.diff(A.row_ptr).astype(np.int64)[A.col_idx].sum())


@pytest.mark.parametrize("g", [5, 12, 37])
def test_laplacian_closed_form(oracle, g):
    """(5-point Laplacian)^2 on a g x g grid: pattern = the 13 offsets with |dx|+|dy| <= 2 that
    stay on the grid; values 16 + (#neighbours) at the centre, -8 at distance 1, +1 straight
    distance 2, +2 diagonal."""
    A = inputs.laplacian_2d(g)
    assert A.nnz == 5 * g * g - 4 * g
    res = oracle.spgemm(A, A)
    offsets = [(dx, dy) for dx in range(-2, 3) for dy in range(-2, 3) if abs(dx) + abs(dy) <= 2]
    assert res.nnz == sum((g - abs(dx)) * (g - abs(dy)) for dx, dy in offsets)
    interior, edge, corner = (g - 2) ** 2, 4 * (g - 2), 4
    assert res.products == interior * 25 + edge * 16 + corner * 9
    rows = np.repeat(np.arange(A.rows), np.diff(res.row_ptr))
    x, y = rows % g, rows // g
    dx, dy = res.col % g - x, res.col // g - y
    nbrs = (x > 0).astype(int) + (x < g - 1) + (y > 0) + (y < g - 1)
    dist = np.abs(dx) + np.abs(dy)
    expect = np.where(dist == 0, 16 + nbrs,
                      np.where(dist == 1, -8, np.where((dx == 0) | (dy == 0), 1, 2))).astype(np.float64)
    assert dist.max() <= 2
    assert np.array_equal(res.val, expect)


def test_laplacian_512_counts(oracle):
    A = inputs.config(2)
    assert (A.rows, A.nnz) == (262144, 1308672)
    counts, products = oracle.row_nnz(A, A)
    assert products == 6535176 and int(counts.sum()) == 3397636


@pytest.mark.parametrize("g", [5, 6])
def test_stencil27_closed_forms(oracle, g):
    n = 3 * g ** 3
    Ap = inputs.stencil27_3d(g, 3, periodic=True)
    assert Ap.nnz == 81 * n
    counts, products = oracle.row_nnz(Ap, Ap)
    assert products == 81 * 81 * n
    assert np.all(counts == 3 * min(g, 5) ** 3)
    At = inputs.stencil27_3d(g, 3, periodic=False)
    assert At.nnz == 9 * (3 * g - 2) ** 3
    counts, products = oracle.row_nnz(At, At)
    assert products == 27 * (2 * 4 + (g - 2) * 9) ** 3
    assert int(counts.sum()) == 9 * (5 * g - 6) ** 3


def test_config1_counts(oracle):
    A = inputs.config(1)
    counts, products = oracle.row_nnz(A, A)
    assert products == 8 * 8 * 1024 and np.all(counts <= 64) and counts.sum() <= 65536


def test_row_range_and_threads_agree(oracle):
    A = inputs.config(4, small=True)
    full = oracle.spgemm(A, A)
    par = oracle.spgemm(A, A, threads=3)
    assert np.array_equal(full.row_ptr, par.row_ptr) and np.array_equal(full.col, par.col)
    assert np.array_equal(full.val, par.val) and full.products == par.products
    part = oracle.spgemm_rows(A, A, 100, 117)
    lo, hi = full.row_ptr[100], full.row_ptr[117]
    assert np.array_equal(part.col, full.col[lo:hi]) and np.array_equal(part.val, full.val[lo:hi])


# ------------------------------------------------------------------ compaction of zeros (Section 4.4)
def test_compaction_worked_example(oracle):
    """A = [[1,-1],[2,0s]], B = [[1,1],[1,1]] (0s = stored zero): A*B = [[0,0],[2,2]] structurally
    full; compaction leaves row 0 empty and row 1 = {(0,2),(1,2)} (computed by hand)."""
    A = inputs.from_coo(2, 2, [0, 0, 1, 1], [0, 1, 0, 1], [1.0, -1.0, 2.0, 0.0], name="cancel")
    B = inputs.from_coo(2, 2, [0, 0, 1, 1], [0, 1, 0, 1], [1.0, 1.0, 1.0, 1.0], name="ones")
    ref = oracle.spgemm(A, B)
    assert ref.nnz == 4 and list(ref.val) == [0.0, 0.0, 2.0, 2.0]
    out = oracle.compact_zeros(ref)
    assert list(out.row_ptr) == [0, 0, 2]
    assert list(out.col) == [0, 1] and list(out.val) == [2.0, 2.0]


@pytest.mark.parametrize("M,K,N,density,seed", [(23, 31, 17, 0.3, 1), (40, 40, 40, 0.2, 2), (8, 64, 8, 0.5, 3)])
def test_compaction_equals_nonzeros_of_the_dense_product(oracle, M, K, N, density, seed):
    """Small-integer values: every sum is exact, so the compacted pattern is exactly the set of
    non-zero entries of the brute-force dense product (many entries cancel)."""
    A = inputs.random_sparse(M, K, density, seed, values="smallint")
    B = inputs.random_sparse(K, N, density, seed + 9, values="smallint")
    c, _, pat = brute_force_product(A, B)
    out = oracle.compact_zeros(oracle.spgemm(A, B))
    want = pat & (c != 0.0)
    assert want.sum() < pat.sum(), "the case should contain cancellations"
    got = np.zeros_like(want)
    for i in range(M):
        cols = out.col[out.row_ptr[i]:out.row_ptr[i + 1]]
        assert np.all(np.diff(cols) > 0)
        got[i, cols] = True
        assert np.array_equal(out.val[out.row_ptr[i]:out.row_ptr[i + 1]], c[i, cols])
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ precision measure (Section 6.4, Eq. 3)
def test_smape_hand_computed(oracle):
    """x = (1, 2), x^ = (1.1, 1.8): 100/2 * (0.1/2.1 + 0.2/3.8) = 5.01253...%; symmetric in its
    arguments; a pair of zeros contributes nothing."""
    want = 50.0 * (0.1 / 2.1 + 0.2 / 3.8)
    assert abs(oracle.smape_percent([1.0, 2.0], [1.1, 1.8]) - want) < 1e-12
    assert abs(oracle.smape_percent([1.1, 1.8], [1.0, 2.0]) - want) < 1e-12
    assert oracle.smape_percent([0.0, 1.0], [0.0, 1.0]) == 0.0
    assert abs(oracle.smape_percent([0.0, 1.0], [0.0, -1.0]) - 50.0) < 1e-12     # opposite signs: a full term


def test_full_precision_reference_differs_only_by_the_fp16_rounding(oracle):
    rng = np.random.default_rng(7)
    A = inputs.random_sparse(60, 50, 0.2, 21)
    A32 = inputs.CSRMatrix(A.rows, A.cols, A.row_ptr, A.col_idx, rng.uniform(-1, 1, A.nnz).astype(np.float32), "fp32")
    full = oracle.spgemm(A32, _t(A32), full_precision=True)
    rounded = oracle.spgemm(A32, _t(A32))
    c, _, _ = brute_force_product(A32, _t(A32))            # dense triple loop on the unrounded values
    got = np.zeros_like(c)
    for i in range(A32.rows):
        got[i, full.col[full.row_ptr[i]:full.row_ptr[i + 1]]] = full.val[full.row_ptr[i]:full.row_ptr[i + 1]]
    assert np.allclose(got, c, rtol=1e-13, atol=1e-15)
    assert np.array_equal(full.col, rounded.col)
    s = oracle.smape_percent(full.val, rounded.val)
    assert 0.0 < s < 0.1, s                               # fp16 rounding: relative 2^-11 per operand at most


def _t(A):
    """Transpose of a CSR matrix (host, any value type)."""
    rows = np.repeat(np.arange(A.rows), np.diff(A.row_ptr))
    order = np.lexsort((rows, A.col_idx))
    row_ptr = np.concatenate([[0], np.cumsum(np.bincount(A.col_idx, minlength=A.cols))]).astype(np.int32)
    return inputs.CSRMatrix(A.cols, A.rows, row_ptr, rows[order].astype(np.int32), np.asarray(A.val)[order], "t")
