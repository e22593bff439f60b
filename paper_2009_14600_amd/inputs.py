"""Seeded synthetic CSR inputs for C = A*A.

This module only *draws inputs*.  It holds none of the spGEMM arithmetic and is
the one piece of code that both the HIP path's tests/bench and the CPU oracle's
tests share.  The paper evaluates A*A on SuiteSparse matrices (Section 5,
Table 1); those files are not redistributable here, so the five generators
below stand in for them: a uniformly random matrix, a 2D 5-point Laplacian, a
3D 27-point stencil with 3x3 node blocks, an R-MAT power-law graph and a
block-clustered matrix.  Every generator can be scaled down for tests.

All matrices are canonical CSR: int32 ``row_ptr``/``col_idx``, strictly
ascending columns per row, values already rounded to IEEE fp16 (round to
nearest even, numpy's float64 -> float16 cast).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 200914600


@dataclass
class CSRMatrix:
    """Host CSR matrix with fp16 values."""

    rows: int
    cols: int
    row_ptr: np.ndarray  # int32[rows + 1]
    col_idx: np.ndarray  # int32[nnz]
    val: np.ndarray      # float16[nnz]
    name: str = ""

    @property
    def nnz(self) -> int:
        return int(self.col_idx.shape[0])

    @property
    def val_bits(self) -> np.ndarray:
        return self.val.view(np.uint16)

    def check_canonical(self) -> None:
        rp = self.row_ptr.astype(np.int64)
        assert rp.shape == (self.rows + 1,) and rp[0] == 0 and rp[-1] == self.nnz
        assert np.all(np.diff(rp) >= 0)
        if self.nnz:
            assert self.col_idx.min() >= 0 and self.col_idx.max() < self.cols
            d = np.diff(self.col_idx.astype(np.int64))
            row_start = np.zeros(self.nnz, dtype=bool)
            starts = rp[:-1][np.diff(rp) > 0]
            row_start[starts] = True
            assert np.all((d > 0) | row_start[1:])


def _uniform_fp16(rng: np.random.Generator, size) -> np.ndarray:
    return rng.uniform(-1.0, 1.0, size=size).astype(np.float16)


def from_coo(rows: int, cols: int, r: np.ndarray, c: np.ndarray, v: np.ndarray,
             name: str = "") -> CSRMatrix:
    """Canonical CSR from duplicate-free COO triplets (any order)."""
    r = np.asarray(r, dtype=np.int64)
    c = np.asarray(c, dtype=np.int64)
    order = np.lexsort((c, r))
    r, c, v = r[order], c[order], np.asarray(v)[order]
    counts = np.bincount(r, minlength=rows)
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    assert row_ptr[-1] < 2**31
    return CSRMatrix(rows, cols, row_ptr.astype(np.int32), c.astype(np.int32),
                     v.astype(np.float16), name)


def random_fixed_per_row(n: int = 1024, per_row: int = 8, seed: int = BASE_SEED + 1,
                         cols: int | None = None) -> CSRMatrix:
    """Exactly ``per_row`` nonzeros per row at uniformly random distinct columns."""
    cols = n if cols is None else cols
    assert per_row <= cols
    rng = np.random.default_rng(seed)
    keys = rng.random((n, cols))
    col = np.sort(np.argpartition(keys, per_row - 1, axis=1)[:, :per_row], axis=1)
    row_ptr = (np.arange(n + 1, dtype=np.int64) * per_row).astype(np.int32)
    val = _uniform_fp16(rng, n * per_row)
    return CSRMatrix(n, cols, row_ptr, col.reshape(-1).astype(np.int32), val,
                     f"random{n}x{cols}_{per_row}per_row")


def laplacian_2d(g: int = 512) -> CSRMatrix:
    """5-point Laplacian on a g x g grid, natural ordering, diagonal 4, off-diagonals -1."""
    n = g * g
    idx = np.arange(n, dtype=np.int64)
    x, y = idx % g, idx // g
    rs, cs, vs = [idx], [idx], [np.full(n, 4.0)]
    for dx, dy in ((-1, 0), (1, 0), (0, -1), (0, 1)):
        ok = (x + dx >= 0) & (x + dx < g) & (y + dy >= 0) & (y + dy < g)
        rs.append(idx[ok])
        cs.append(idx[ok] + dx + dy * g)
        vs.append(np.full(int(ok.sum()), -1.0))
    return from_coo(n, n, np.concatenate(rs), np.concatenate(cs), np.concatenate(vs),
                    f"laplacian2d_{g}")


def laplacian_3d(g: int = 64) -> CSRMatrix:
    """7-point Laplacian on a g x g x g grid, natural ordering, diagonal 6, off-diagonals -1."""
    n = g ** 3
    idx = np.arange(n, dtype=np.int64)
    x, y, z = idx % g, (idx // g) % g, idx // (g * g)
    rs, cs, vs = [idx], [idx], [np.full(n, 6.0)]
    for dx, dy, dz in ((-1, 0, 0), (1, 0, 0), (0, -1, 0), (0, 1, 0), (0, 0, -1), (0, 0, 1)):
        ok = ((x + dx >= 0) & (x + dx < g) & (y + dy >= 0) & (y + dy < g) & (z + dz >= 0) & (z + dz < g))
        rs.append(idx[ok])
        cs.append(idx[ok] + dx + dy * g + dz * g * g)
        vs.append(np.full(int(ok.sum()), -1.0))
    return from_coo(n, n, np.concatenate(rs), np.concatenate(cs), np.concatenate(vs),
                    f"laplacian3d_{g}")


def stencil27_3d(g: int = 48, dof: int = 3, periodic: bool = True,
                 seed: int = BASE_SEED + 3) -> CSRMatrix:
    """27-point stencil on a g^3 grid, ``dof`` unknowns per node, dense dof x dof couplings.

    ``periodic=True`` wraps neighbours around the grid so that every row has
    exactly 27*dof nonzeros (needs g >= 3); otherwise the stencil is truncated
    at the boundary.
    """
    assert (not periodic) or g >= 3
    rng = np.random.default_rng(seed)
    nodes = g ** 3
    idx = np.arange(nodes, dtype=np.int64)
    x, y, z = idx % g, (idx // g) % g, idx // (g * g)
    nb = np.empty((nodes, 27), dtype=np.int64)
    ok = np.ones((nodes, 27), dtype=bool)
    s = 0
    for dz in (-1, 0, 1):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                xx, yy, zz = x + dx, y + dy, z + dz
                if periodic:
                    xx, yy, zz = xx % g, yy % g, zz % g
                else:
                    ok[:, s] = ((xx >= 0) & (xx < g) & (yy >= 0) & (yy < g)
                                & (zz >= 0) & (zz < g))
                nb[:, s] = xx + g * (yy + g * zz)
                s += 1
    nb[~ok] = np.iinfo(np.int64).max
    nb.sort(axis=1)
    cnt = ok.sum(axis=1)                       # neighbours per node
    # one CSR row per (node, d): the node's sorted neighbours, each expanded to dof columns
    per_row = np.repeat(cnt * dof, dof)
    n = nodes * dof
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(per_row, out=row_ptr[1:])
    keep = nb != np.iinfo(np.int64).max        # [nodes, 27]
    cols_node = (nb[:, :, None] * dof + np.arange(dof)[None, None, :])  # [nodes,27,dof]
    keep3 = np.broadcast_to(keep[:, :, None], cols_node.shape)
    cols_node = cols_node.reshape(nodes, 27 * dof)
    keep3 = keep3.reshape(nodes, 27 * dof)
    # every one of the node's dof rows has the same column set
    col_rows = np.repeat(cols_node, dof, axis=0)
    keep_rows = np.repeat(keep3, dof, axis=0)
    col_idx = col_rows[keep_rows].astype(np.int32)
    assert col_idx.shape[0] == row_ptr[-1] < 2**31
    val = _uniform_fp16(rng, col_idx.shape[0])
    return CSRMatrix(n, n, row_ptr.astype(np.int32), col_idx, val,
                     f"stencil27_{g}cubed_dof{dof}_{'periodic' if periodic else 'truncated'}")


def rmat(scale: int = 18, edge_factor: int = 16, abcd=(0.57, 0.19, 0.19, 0.05),
         seed: int = BASE_SEED + 4) -> CSRMatrix:
    """R-MAT graph: 2^scale vertices, edge_factor * 2^scale edge draws, symmetrized,
    self-loops and duplicates removed, every stored value 1.0.  No vertex permutation:
    the hubs sit at the low indices."""
    a, b, c, _ = abcd
    rng = np.random.default_rng(seed)
    n = 1 << scale
    m = n * edge_factor
    r = np.zeros(m, dtype=np.int64)
    col = np.zeros(m, dtype=np.int64)
    for _level in range(scale):
        u = rng.random(m)
        down = u >= a + b                         # quadrants c, d: lower half
        right = ((u >= a) & (u < a + b)) | (u >= a + b + c)   # quadrants b, d: right half
        r = (r << 1) | down
        col = (col << 1) | right
    keep = r != col
    r, col = r[keep], col[keep]
    key = np.unique(np.concatenate([r * n + col, col * n + r]))
    return from_coo(n, n, key // n, key % n, np.ones(key.shape[0]),
                    f"rmat_s{scale}_ef{edge_factor}")


def block_clustered(n: int = 131072, blocks_per_row: int = 4, fill: float = 0.5,
                    block: int = 16, seed: int = BASE_SEED + 5) -> CSRMatrix:
    """Per ``block``-row block-row, ``blocks_per_row`` distinct random block columns, each
    block filled at Bernoulli density ``fill`` with uniform[-1,1] values."""
    assert n % block == 0
    nb = n // block
    assert blocks_per_row <= nb
    rng = np.random.default_rng(seed)
    bc = rng.integers(0, nb, size=(nb, blocks_per_row))
    while True:
        bc.sort(axis=1)
        dup = np.any(np.diff(bc, axis=1) == 0, axis=1)
        if not dup.any():
            break
        bc[dup] = rng.integers(0, nb, size=(int(dup.sum()), blocks_per_row))
    mask = rng.random((nb, blocks_per_row, block, block)) < fill   # [brow, j, r, c]
    # CSR order: brow, r, j (ascending block column), c
    mask_rows = mask.transpose(0, 2, 1, 3)
    cols_full = (bc[:, None, :, None] * block
                 + np.arange(block)[None, None, None, :])          # [brow,1,j,c]
    cols_full = np.broadcast_to(cols_full, mask_rows.shape)
    col_idx = cols_full[mask_rows].astype(np.int32)
    per_row = mask_rows.reshape(n, -1).sum(axis=1)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(per_row, out=row_ptr[1:])
    val = _uniform_fp16(rng, col_idx.shape[0])
    return CSRMatrix(n, n, row_ptr.astype(np.int32), col_idx, val,
                     f"block_clustered_{n}")


def random_sparse(rows: int, cols: int, density: float, seed: int,
                  empty_row_fraction: float = 0.0, values: str = "uniform") -> CSRMatrix:
    """Bernoulli(density) pattern, for small rectangular / ragged test cases.

    values: "uniform" -> uniform[-1,1]; "ones" -> 1.0; "smallint" -> integers in [-3,3]\\{0};
    "tiny" -> fp16 subnormals and values near the bottom of the normal range.
    """
    rng = np.random.default_rng(seed)
    mask = rng.random((rows, cols)) < density
    if empty_row_fraction > 0 and rows:
        mask[rng.random(rows) < empty_row_fraction] = False
    r, c = np.nonzero(mask)
    k = r.shape[0]
    if values == "uniform":
        v = _uniform_fp16(rng, k)
    elif values == "ones":
        v = np.ones(k, dtype=np.float16)
    elif values == "smallint":
        v = rng.integers(1, 4, size=k) * rng.choice([-1, 1], size=k)
    elif values == "tiny":
        v = (rng.integers(1, 3000, size=k).astype(np.uint16)
             | (rng.integers(0, 2, size=k).astype(np.uint16) << 15)).view(np.float16)
    else:
        raise ValueError(values)
    return from_coo(rows, cols, r, c, v, f"random_{rows}x{cols}_d{density}_s{seed}")


def config(index: int, small: bool = False) -> CSRMatrix:
    """The five benchmark workloads (index 1..5).  ``small=True`` gives a reduced instance
    of the same structure that the CPU oracle finishes in well under a second."""
    if index == 1:
        return random_fixed_per_row(1024 if not small else 200, 8)
    if index == 2:
        return laplacian_2d(512 if not small else 37)
    if index == 3:
        return stencil27_3d(48 if not small else 7, 3, periodic=True)
    if index == 4:
        return rmat(18 if not small else 10, 16)
    if index == 5:
        return block_clustered(131072 if not small else 2048)
    raise ValueError("config index must be 1..5")


CONFIG_NAMES = {
    1: "random 1024x1024, 8 nnz/row",
    2: "2D 5-point Laplacian 512x512 grid",
    3: "3D 27-point stencil 48^3 x 3 dof (periodic)",
    4: "R-MAT scale 18, edge factor 16, symmetrized",
    5: "block-clustered 131072, 4 blocks/block-row, 50% fill",
}
