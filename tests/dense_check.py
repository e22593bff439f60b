"""Brute-force dense helpers used to pin the oracle (tiny inputs only)."""
import numpy as np


def densify(A):
    """(values float64[rows, cols], stored-pattern bool[rows, cols])."""
    d = np.zeros((A.rows, A.cols), dtype=np.float64)
    p = np.zeros((A.rows, A.cols), dtype=bool)
    for i in range(A.rows):
        for e in range(int(A.row_ptr[i]), int(A.row_ptr[i + 1])):
            d[i, A.col_idx[e]] = float(A.val[e])
            p[i, A.col_idx[e]] = True
    return d, p


def brute_force_product(A, B):
    """Triple loop over the dense forms: values, magnitudes and structural pattern."""
    da, pa = densify(A)
    db, pb = densify(B)
    M, K, N = A.rows, A.cols, B.cols
    c = np.zeros((M, N))
    s = np.zeros((M, N))
    pat = np.zeros((M, N), dtype=bool)
    for i in range(M):
        for k in range(K):
            if not pa[i, k]:
                continue
            for j in range(N):
                if pb[k, j]:
                    pat[i, j] = True
                    c[i, j] += da[i, k] * db[k, j]
                    s[i, j] += abs(da[i, k] * db[k, j])
    return c, s, pat


def oracle_to_dense(res, rows, cols):
    c = np.zeros((rows, cols))
    s = np.zeros((rows, cols))
    pat = np.zeros((rows, cols), dtype=bool)
    for i in range(rows):
        for e in range(int(res.row_ptr[i]), int(res.row_ptr[i + 1])):
            j = res.col[e]
            assert not pat[i, j], "duplicate column in a row"
            pat[i, j] = True
            c[i, j] = res.val[e]
            s[i, j] = res.mag[e]
    return c, s, pat
