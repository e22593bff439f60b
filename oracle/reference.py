"""CPU oracle for the tiled spGEMM path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this module; the HIP library and its Python binding never do, and this module
imports nothing from them.

Two layers:

* ``spgemm`` / ``spgemm_rows`` / ``row_nnz``: the end result, C = A*B by row-wise
  Gustavson in fp64 (``spgemm_oracle.c``; definition in paper Section 2.2, precision in
  Section 2.6, structural pattern as in Section 4.2).
* ``bitmap_format`` / ``task_list`` / ``counting``: the intermediate objects the paper's
  pipeline names (Section 2.1.2 bitmap format; Section 4.1 and Algorithm 1 (task-list part) task
  list; Section 4.2 counting kernel), written out step by step in numpy for small inputs,
  with the tile edge T as a parameter (the paper uses 8; the GPU path uses 16).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spgemm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_spgemm.so")
_lib = None


def build_lib(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no vendor libraries)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_lib())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_spgemm_row_nnz.restype = i64
        lib.oracle_spgemm_row_nnz.argtypes = [i64, p, p, p, p, i64, i64, p]
        lib.oracle_spgemm_rows.restype = i64
        lib.oracle_spgemm_rows.argtypes = [i64, p, p, p, p, p, p, i64, i64, p, p, p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


class _Operand:
    """Contiguous int64/int32/float64 arrays of a CSR matrix for the C calls."""

    def __init__(self, m, full_precision: bool = False):
        self.rows, self.cols = int(m.rows), int(m.cols)
        self.row_ptr = np.ascontiguousarray(m.row_ptr, dtype=np.int64)
        self.col = np.ascontiguousarray(m.col_idx, dtype=np.int32)
        if full_precision:
            # the values as stored (fp32 or fp64 inputs, not rounded): the "full precision" side of
            # the paper's precision comparison (Section 6.4)
            self.val = np.ascontiguousarray(np.asarray(m.val).astype(np.float64))
        else:
            # the inputs are fp16 numbers (others are rounded to nearest-even fp16 first, Section
            # 2.6); widening them to fp64 is exact
            self.val = np.ascontiguousarray(np.asarray(m.val).astype(np.float16).astype(np.float64))


def row_nnz(A, B, row_begin: int = 0, row_end: int | None = None):
    """(structural nnz of each row of C in the range, products in the range)."""
    a, b = _Operand(A), _Operand(B)
    assert a.cols == b.rows
    row_end = a.rows if row_end is None else row_end
    out = np.zeros(max(row_end - row_begin, 0), dtype=np.int64)
    products = _load().oracle_spgemm_row_nnz(b.cols, _ptr(a.row_ptr), _ptr(a.col), _ptr(b.row_ptr),
                                             _ptr(b.col), row_begin, row_end, _ptr(out))
    if products < 0:
        raise MemoryError
    return out, int(products)


@dataclass
class OracleResult:
    row_begin: int
    row_ptr: np.ndarray   # int64[rows_in_range + 1], relative to the first row in the range
    col: np.ndarray       # int32
    val: np.ndarray       # float64, sum_k a_ik b_kj
    mag: np.ndarray       # float64, sum_k |a_ik||b_kj|
    products: int

    @property
    def nnz(self) -> int:
        return int(self.col.shape[0])


def spgemm_rows(A, B, row_begin: int, row_end: int, _ops=None) -> OracleResult:
    """Rows [row_begin,row_end) of C = A*B."""
    a, b = _ops if _ops is not None else (_Operand(A), _Operand(B))
    assert a.cols == b.rows
    counts = np.zeros(max(row_end - row_begin, 0), dtype=np.int64)
    lib = _load()
    products = lib.oracle_spgemm_row_nnz(b.cols, _ptr(a.row_ptr), _ptr(a.col), _ptr(b.row_ptr),
                                         _ptr(b.col), row_begin, row_end, _ptr(counts))
    if products < 0:
        raise MemoryError
    row_ptr = np.zeros(counts.shape[0] + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    total = int(row_ptr[-1])
    col = np.empty(total, dtype=np.int32)
    val = np.empty(total, dtype=np.float64)
    mag = np.empty(total, dtype=np.float64)
    wrote = lib.oracle_spgemm_rows(b.cols, _ptr(a.row_ptr), _ptr(a.col), _ptr(a.val),
                                   _ptr(b.row_ptr), _ptr(b.col), _ptr(b.val),
                                   row_begin, row_end, _ptr(col), _ptr(val), _ptr(mag))
    if wrote != total:
        raise RuntimeError(f"oracle wrote {wrote} entries, sized {total}")
    return OracleResult(row_begin, row_ptr, col, val, mag, int(products))


def spgemm(A, B, threads: int = 1, full_precision: bool = False) -> OracleResult:
    """All of C = A*B.  threads > 1 runs independent row blocks on a thread pool (the C
    calls release the GIL); every row is still computed by the same serial code, so the
    result does not depend on the thread count.  full_precision: use the stored values
    without the rounding to fp16 (the reference side of the precision study, Section 6.4)."""
    ops = (_Operand(A, full_precision), _Operand(B, full_precision))
    rows = ops[0].rows
    if threads <= 1 or rows < 4 * threads:
        return spgemm_rows(A, B, 0, rows, _ops=ops)
    nblocks = min(rows, threads * 8)
    bounds = np.linspace(0, rows, nblocks + 1).astype(np.int64)
    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(lambda i: spgemm_rows(A, B, int(bounds[i]), int(bounds[i + 1]), _ops=ops),
                              range(nblocks)))
    counts = np.concatenate([np.diff(p.row_ptr) for p in parts])
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return OracleResult(0, row_ptr, np.concatenate([p.col for p in parts]),
                        np.concatenate([p.val for p in parts]), np.concatenate([p.mag for p in parts]),
                        sum(p.products for p in parts))


# --------------------------------------------------------------------------------------
# Intermediate objects of the paper's pipeline, for small inputs.
# --------------------------------------------------------------------------------------

def compact_zeros(res: OracleResult) -> OracleResult:
    """Compaction of zeros (paper Section 4.4; Algorithm 1, the two compaction steps after the
    multiplication kernel): the entries whose accumulated value is zero are removed, the others
    keep their order; rows may become empty.  The decision is taken on the value the oracle
    holds (fp64 sums of exact products), so it equals the GPU's fp32 decision whenever the sums
    are exact in both (small integers, stored zeros), which is what the parity tests use."""
    keep = res.val != 0.0
    before = np.concatenate([[0], np.cumsum(keep)]).astype(np.int64)
    return OracleResult(res.row_begin, before[res.row_ptr], res.col[keep], res.val[keep], res.mag[keep],
                        res.products)


@dataclass
class BitmapMatrix:
    """Bitmap format (paper Section 2.1.2): non-empty T x T tiles in COO order (row-major),
    each with an index into the element array and a bitmap; here the bitmap is kept as T
    row masks (bit c of mask r <-> slot (r,c)), and the tile's elements sit consecutively
    in the element array in ascending slot order r*T+c."""
    T: int
    tile_rows: int
    tile_cols: int
    tile_row: np.ndarray   # int64[ntiles]
    tile_col: np.ndarray   # int64[ntiles]
    index: np.ndarray      # int64[ntiles + 1] offsets into elements
    row_mask: np.ndarray   # uint32[ntiles, T]
    elements: np.ndarray   # float16[nnz]


def bitmap_format(A, T: int = 16) -> BitmapMatrix:
    rp = np.asarray(A.row_ptr, dtype=np.int64)
    col = np.asarray(A.col_idx, dtype=np.int64)
    val = np.asarray(A.val, dtype=np.float16)
    row = np.repeat(np.arange(A.rows, dtype=np.int64), np.diff(rp))
    ntr, ntc = -(-A.rows // T), -(-A.cols // T)
    tr, tc = row // T, col // T
    slot = (row % T) * T + (col % T)
    order = np.lexsort((slot, tc, tr))
    tr, tc, slot, val = tr[order], tc[order], slot[order], val[order]
    key = tr * max(ntc, 1) + tc
    first = np.ones(key.shape[0], dtype=bool)
    first[1:] = key[1:] != key[:-1]
    starts = np.nonzero(first)[0]
    ntiles = starts.shape[0]
    index = np.concatenate([starts, [key.shape[0]]]).astype(np.int64)
    row_mask = np.zeros((ntiles, T), dtype=np.uint32)
    tile_of = np.cumsum(first) - 1
    np.bitwise_or.at(row_mask, (tile_of, slot // T), (np.uint32(1) << (slot % T).astype(np.uint32)))
    return BitmapMatrix(T, ntr, ntc, tr[starts], tc[starts], index, row_mask, val)


def _boolean_tile_product(mask_a: np.ndarray, mask_b: np.ndarray, T: int) -> np.ndarray:
    """Row masks of the boolean product of two T x T 0/1 tiles."""
    out = np.zeros(T, dtype=np.uint32)
    for r in range(T):
        for k in range(T):
            if (int(mask_a[r]) >> k) & 1:
                out[r] |= mask_b[k]
    return out


@dataclass
class TaskList:
    a_tile: np.ndarray     # int64[P] index of the A tile of each entry
    b_tile: np.ndarray     # int64[P]
    offsets: np.ndarray    # int64[n_c_tiles + 1]
    c_tile_row: np.ndarray
    c_tile_col: np.ndarray
    candidates: int        # tile pairs before the zero-product filter


def task_list(TA: BitmapMatrix, TB: BitmapMatrix) -> TaskList:
    """Section 4.1 / Algorithm 1, task-list part: pair every non-empty tile A[I,K] with every
    non-empty tile B[K,J]; drop pairs whose boolean tile product is all zero; sort (stably)
    by B tile column, then by A tile row, so entries of one C tile are consecutive and keep
    ascending K; count entries per distinct (I,J); prefix-sum the counts into offsets."""
    T = TA.T
    b_by_row: dict[int, list[int]] = {}
    for t in range(TB.tile_row.shape[0]):
        b_by_row.setdefault(int(TB.tile_row[t]), []).append(t)
    pa, pb = [], []
    candidates = 0
    for a in range(TA.tile_row.shape[0]):
        for b in b_by_row.get(int(TA.tile_col[a]), []):
            candidates += 1
            if _boolean_tile_product(TA.row_mask[a], TB.row_mask[b], T).any():
                pa.append(a)
                pb.append(b)
    pa = np.asarray(pa, dtype=np.int64)
    pb = np.asarray(pb, dtype=np.int64)
    o = np.argsort(TB.tile_col[pb], kind="stable")
    pa, pb = pa[o], pb[o]
    o = np.argsort(TA.tile_row[pa], kind="stable")
    pa, pb = pa[o], pb[o]
    ci, cj = TA.tile_row[pa], TB.tile_col[pb]
    first = np.ones(pa.shape[0], dtype=bool)
    first[1:] = (ci[1:] != ci[:-1]) | (cj[1:] != cj[:-1])
    starts = np.nonzero(first)[0]
    offsets = np.concatenate([starts, [pa.shape[0]]]).astype(np.int64)
    return TaskList(pa, pb, offsets, ci[starts], cj[starts], candidates)


def counting(TA: BitmapMatrix, TB: BitmapMatrix, tl: TaskList):
    """Section 4.2: per C tile, the 0/1 'simulated' product of the bitmaps of its task-list
    entries, accumulated; returns (row masks uint32[n_c_tiles, T], element count per tile)."""
    T = TA.T
    n = tl.c_tile_row.shape[0]
    masks = np.zeros((n, T), dtype=np.uint32)
    for c in range(n):
        for e in range(tl.offsets[c], tl.offsets[c + 1]):
            masks[c] |= _boolean_tile_product(TA.row_mask[tl.a_tile[e]], TB.row_mask[tl.b_tile[e]], T)
    counts = np.array([sum(bin(int(m)).count("1") for m in masks[c]) for c in range(n)], dtype=np.int64)
    return masks, counts


def smape_percent(x: np.ndarray, x_hat: np.ndarray) -> float:
    """Equation 3: symmetric mean absolute percentage error; a term with x = x_hat = 0
    contributes 0."""
    x = np.asarray(x, dtype=np.float64)
    x_hat = np.asarray(x_hat, dtype=np.float64)
    den = np.abs(x) + np.abs(x_hat)
    num = np.abs(x - x_hat)
    terms = np.divide(num, den, out=np.zeros_like(num), where=den > 0)
    return 100.0 * float(terms.mean()) if terms.size else 0.0
