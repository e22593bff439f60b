"""Thin ctypes binding over libtsp.so (see include/tsp.h).  Argument marshalling only: every step
of the spGEMM path runs in the library's HIP kernels.  PyTorch supplies device memory (through
the allocator callbacks) and the stream.  There is no CPU fallback: if the library has not been
built, or no GPU is present, the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtsp.so")

TSP_I32, TSP_I64 = 0, 1
TSP_F16, TSP_F32 = 0, 1
FORM_LEFT, FORM_RIGHT = 1, 2
OPT_VALIDATE, OPT_PHASE_TIMERS, OPT_WIDE_INDEX, OPT_NUMERIC_RUN, OPT_MATRIX_CORES, OPT_COMPACT_ZEROS = 1, 2, 3, 4, 5, 6
OPT_WORK_ORDER = 7
OPT_STRIP_ORDER = 8
OPT_COUNT_PRODUCTS = 10
OPT_WORKSPACE_CANARIES = 11
PHASES = ("convert", "symbolic", "count", "numeric")
KERNELS = ("convert", "sym_count", "scan_sym", "sym_emit", "count_masks", "row_offsets", "scan_rows", "numeric")

EXPORTS = [
    "tsp_create", "tsp_destroy", "tsp_set_option", "tsp_trim", "tsp_spgemm", "tsp_csr_free",
    "tsp_convert", "tsp_tiles_free", "tsp_tiles_get_view", "tsp_symbolic", "tsp_plan_free",
    "tsp_plan_get_view", "tsp_numeric", "tsp_compact_zeros", "tsp_compact_zeros_static", "tsp_spgemm_paper",
    "tsp_get_stats", "tsp_strerror",
    "tsp_last_hip_error",
]


class TspError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"tsp status {status}: {message}")
        self.status = status


class _Csr(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("val", ctypes.c_void_p),
                ("row_ptr_type", ctypes.c_int32), ("val_type", ctypes.c_int32)]


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p)


class _Allocator(ctypes.Structure):
    _fields_ = [("alloc", _ALLOC_FN), ("free", _FREE_FN), ("user", ctypes.c_void_p)]


class _Stats(ctypes.Structure):
    _fields_ = [("a_tiles", ctypes.c_int64), ("b_tiles", ctypes.c_int64), ("candidate_pairs", ctypes.c_int64),
                ("pairs", ctypes.c_int64), ("c_tiles", ctypes.c_int64), ("c_nnz", ctypes.c_int64),
                ("workspace_bytes", ctypes.c_int64), ("workspace_peak_bytes", ctypes.c_int64),
                ("phase_us", ctypes.c_float * 4), ("total_us", ctypes.c_float),
                ("kernel_us", ctypes.c_float * len(KERNELS)),
                ("products", ctypes.c_int64), ("a_mean_row", ctypes.c_float), ("a_tile_fill", ctypes.c_float),
                ("in_paper_regime", ctypes.c_int32), ("well_filled_tiles", ctypes.c_int32),
                ("workspace_violations", ctypes.c_int64)]


class _TilesView(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("tile_rows", ctypes.c_int64),
                ("tile_cols", ctypes.c_int64), ("ntiles", ctypes.c_int64), ("tile_slots", ctypes.c_int64),
                ("forms", ctypes.c_int32),
                ("tile_row_ptr", ctypes.c_void_p), ("tile_row_end", ctypes.c_void_p),
                ("tile_col", ctypes.c_void_p), ("row_mask", ctypes.c_void_p),
                ("left_group_mask", ctypes.c_void_p), ("right_group_mask", ctypes.c_void_p),
                ("left_head", ctypes.c_void_p), ("right_head", ctypes.c_void_p),
                ("left_elements", ctypes.c_void_p), ("right_elements", ctypes.c_void_p),
                ("left_groups_capacity", ctypes.c_int64), ("right_groups_capacity", ctypes.c_int64)]


class _PlanView(ctypes.Structure):
    _fields_ = [("c_rows", ctypes.c_int64), ("c_cols", ctypes.c_int64), ("c_tile_rows", ctypes.c_int64),
                ("c_tiles", ctypes.c_int64), ("pairs", ctypes.c_int64), ("c_nnz", ctypes.c_int64),
                ("candidate_pairs", ctypes.c_int64),
                ("c_tile_row_ptr", ctypes.c_void_p), ("c_tile_row", ctypes.c_void_p), ("c_tile_col", ctypes.c_void_p),
                ("pair_off", ctypes.c_void_p), ("pair_ab", ctypes.c_void_p),
                ("c_row_mask", ctypes.c_void_p), ("c_row_off", ctypes.c_void_p), ("c_row_ptr", ctypes.c_void_p)]


_lib = None


def load_library():
    """Load libtsp.so; raises if it has not been built (python -m paper_2009_14600_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                           "or python paper_2009_14600_amd/build.py; there is no fallback path")
    # PyTorch-ROCm ships its own HIP runtime; importing torch first makes libtsp.so bind to that
    # one copy (same soname) instead of bringing a second runtime into the process.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    P = ctypes.POINTER
    lib.tsp_create.argtypes = [P(vp), P(_Allocator)]
    lib.tsp_destroy.argtypes = [vp]
    lib.tsp_set_option.argtypes = [vp, ci, i64]
    lib.tsp_trim.argtypes = [vp, vp]
    lib.tsp_spgemm.argtypes = [vp, P(_Csr), P(_Csr), P(_Csr), vp]
    lib.tsp_csr_free.argtypes = [vp, P(_Csr), vp]
    lib.tsp_convert.argtypes = [vp, P(_Csr), ci, P(vp), vp]
    lib.tsp_tiles_free.argtypes = [vp, vp, vp]
    lib.tsp_tiles_get_view.argtypes = [vp, P(_TilesView)]
    lib.tsp_symbolic.argtypes = [vp, vp, vp, P(vp), vp]
    lib.tsp_plan_free.argtypes = [vp, vp, vp]
    lib.tsp_plan_get_view.argtypes = [vp, P(_PlanView)]
    lib.tsp_numeric.argtypes = [vp, vp, vp, vp, P(_Csr), vp]
    lib.tsp_compact_zeros.argtypes = [vp, P(_Csr), P(_Csr), vp]
    lib.tsp_compact_zeros_static.argtypes = [vp, P(_Csr), P(_Csr), vp]
    lib.tsp_spgemm_paper.argtypes = [vp, ci, P(_Csr), P(_Csr), P(_Csr), vp]
    lib.tsp_get_stats.argtypes = [vp, P(_Stats)]
    lib.tsp_strerror.argtypes = [ci]
    lib.tsp_strerror.restype = ctypes.c_char_p
    lib.tsp_last_hip_error.argtypes = [vp]
    for name in EXPORTS:
        if name != "tsp_strerror":
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise TspError(status, load_library().tsp_strerror(status).decode())


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("tsp needs a GPU (torch.cuda.is_available() is False); there is no CPU path")
    return torch


@dataclass
class DeviceCSR:
    """CSR matrix whose arrays are torch tensors on the GPU."""
    rows: int
    cols: int
    row_ptr: "object"
    col_idx: "object"
    val: "object"
    _owner: "object" = None       # Handle that must release the arrays (outputs only)
    _raw: "object" = None

    @property
    def nnz(self) -> int:
        return int(self.col_idx.shape[0])

    def _struct(self) -> _Csr:
        torch = _torch()
        rp_type = {torch.int32: TSP_I32, torch.int64: TSP_I64}[self.row_ptr.dtype]
        v_type = {torch.float16: TSP_F16, torch.uint16: TSP_F16, torch.int16: TSP_F16,
                  torch.float32: TSP_F32}[self.val.dtype]
        assert self.col_idx.dtype == torch.int32
        for t in (self.row_ptr, self.col_idx, self.val):
            assert t.is_cuda and t.is_contiguous()
        return _Csr(self.rows, self.cols, self.nnz, self.row_ptr.data_ptr(), self.col_idx.data_ptr(),
                    self.val.data_ptr(), rp_type, v_type)

    def free(self):
        if self._owner is not None and self._raw is not None:
            self._owner._free_csr(self._raw)
            self._owner = self._raw = None

    def to_host(self):
        """(row_ptr int64, col_idx int32, val) as numpy arrays."""
        return (self.row_ptr.cpu().numpy().astype(np.int64), self.col_idx.cpu().numpy(),
                self.val.cpu().numpy())


def to_device(m, value_dtype: str = "f16", row_ptr_dtype: str = "i32") -> DeviceCSR:
    """Upload a host CSR matrix (inputs.CSRMatrix)."""
    torch = _torch()
    rp = np.asarray(m.row_ptr, dtype=np.int32 if row_ptr_dtype == "i32" else np.int64)
    val = np.asarray(m.val, dtype=np.float16)
    if value_dtype == "f32":
        val = val.astype(np.float32)
    dev = torch.device("cuda", torch.cuda.current_device())
    return DeviceCSR(int(m.rows), int(m.cols), torch.from_numpy(rp.copy()).to(dev),
                     torch.from_numpy(np.asarray(m.col_idx, dtype=np.int32).copy()).to(dev),
                     torch.from_numpy(val.copy()).to(dev))


class Handle:
    """tsp_handle whose device memory comes from PyTorch's caching allocator."""

    def __init__(self, validate: bool = True, phase_timers: bool = False):
        self._lib = load_library()
        torch = _torch()
        self._torch = torch
        self._blocks = {}

        def _alloc(_user, nbytes, _stream):
            try:
                t = torch.empty(int(nbytes), dtype=torch.uint8, device="cuda")
            except Exception:   # out of memory: report NULL to the library
                return None
            self._blocks[t.data_ptr()] = t
            return t.data_ptr()

        def _free(_user, ptr, _stream):
            self._blocks.pop(ptr, None)

        self._alloc_cb, self._free_cb = _ALLOC_FN(_alloc), _FREE_FN(_free)
        self._allocator = _Allocator(self._alloc_cb, self._free_cb, None)
        self._h = ctypes.c_void_p()
        _check(self._lib.tsp_create(ctypes.byref(self._h), ctypes.byref(self._allocator)))
        self.set_option(OPT_VALIDATE, int(validate))
        self.set_option(OPT_PHASE_TIMERS, int(phase_timers))

    # -- plumbing ---------------------------------------------------------------------------
    def _stream(self):
        return ctypes.c_void_p(self._torch.cuda.current_stream().cuda_stream)

    def _view(self, ptr: int, count: int, dtype):
        """Tensor view of `count` elements at device address `ptr` inside one of our blocks."""
        torch = self._torch
        itemsize = torch.empty((), dtype=dtype).element_size()
        if count == 0 or not ptr:
            return torch.empty(0, dtype=dtype, device="cuda")
        for base, block in self._blocks.items():
            if base <= ptr and ptr + count * itemsize <= base + block.numel():
                off = ptr - base
                return block[off:off + count * itemsize].view(dtype)
        raise RuntimeError("device pointer does not belong to this handle")

    def close(self):
        if self._h:
            self._lib.tsp_destroy(self._h)
            self._h = ctypes.c_void_p()
            self._blocks.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, key: int, value: int):
        _check(self._lib.tsp_set_option(self._h, key, value))

    def trim(self):
        _check(self._lib.tsp_trim(self._h, self._stream()))

    def stats(self) -> dict:
        st = _Stats()
        _check(self._lib.tsp_get_stats(self._h, ctypes.byref(st)))
        out = {k: getattr(st, k) for k, _ in _Stats._fields_ if k not in ("phase_us", "kernel_us")}
        out["phase_us"] = {name: st.phase_us[i] for i, name in enumerate(PHASES)}
        out["kernel_us"] = {name: st.kernel_us[i] for i, name in enumerate(KERNELS)}
        return out

    def _wrap_output(self, raw: _Csr) -> DeviceCSR:
        torch = self._torch
        return DeviceCSR(raw.rows, raw.cols, self._view(raw.row_ptr, raw.rows + 1, torch.int64),
                         self._view(raw.col_idx, raw.nnz, torch.int32), self._view(raw.val, raw.nnz, torch.float32),
                         _owner=self, _raw=raw)

    def _free_csr(self, raw: _Csr):
        if self._h:
            _check(self._lib.tsp_csr_free(self._h, ctypes.byref(raw), self._stream()))

    # -- the path -----------------------------------------------------------------------------
    def spgemm(self, A: DeviceCSR, B: DeviceCSR) -> DeviceCSR:
        """C = A*B (tsp_spgemm).  Pass the same object twice for A*A."""
        sa = A._struct()
        sb = sa if B is A else B._struct()
        out = _Csr()
        _check(self._lib.tsp_spgemm(self._h, ctypes.byref(sa), ctypes.byref(sb), ctypes.byref(out), self._stream()))
        return self._wrap_output(out)

    def spgemm_paper(self, A: DeviceCSR, B: DeviceCSR, tile_edge: int) -> DeviceCSR:
        """C = A*B by the paper's own pipeline at a tile edge of 8, 16 or 32 (tsp_spgemm_paper)."""
        sa = A._struct()
        sb = sa if B is A else B._struct()
        out = _Csr()
        _check(self._lib.tsp_spgemm_paper(self._h, int(tile_edge), ctypes.byref(sa), ctypes.byref(sb),
                                          ctypes.byref(out), self._stream()))
        return self._wrap_output(out)

    def compact_zeros(self, C: DeviceCSR) -> DeviceCSR:
        """C without its zero-valued entries (tsp_compact_zeros)."""
        sc = C._struct()
        out = _Csr()
        _check(self._lib.tsp_compact_zeros(self._h, ctypes.byref(sc), ctypes.byref(out), self._stream()))
        return self._wrap_output(out)

    def compact_zeros_static(self, C: DeviceCSR, out_row_ptr, out_col_idx, out_val) -> int:
        """tsp_compact_zeros_static: the compaction into arrays the caller brings (int64[rows+1],
        int32[>= C.nnz], float32[>= C.nnz] tensors on the GPU); returns the new nnz."""
        sc = C._struct()
        out = _Csr(0, 0, 0, out_row_ptr.data_ptr(), out_col_idx.data_ptr(), out_val.data_ptr(), TSP_I64, TSP_F32)
        _check(self._lib.tsp_compact_zeros_static(self._h, ctypes.byref(sc), ctypes.byref(out), self._stream()))
        return int(out.nnz)

    def spgemm_raw(self, sa: _Csr, sb: _Csr):
        """tsp_spgemm on prepared structs; returns the raw output struct (benchmark loop)."""
        out = _Csr()
        _check(self._lib.tsp_spgemm(self._h, ctypes.byref(sa), ctypes.byref(sb), ctypes.byref(out), self._stream()))
        return out

    def convert(self, A: DeviceCSR, forms: int = FORM_LEFT | FORM_RIGHT) -> "Tiles":
        sa = A._struct()
        t = ctypes.c_void_p()
        _check(self._lib.tsp_convert(self._h, ctypes.byref(sa), forms, ctypes.byref(t), self._stream()))
        return Tiles(self, t)

    def symbolic(self, A: "Tiles", B: "Tiles") -> "Plan":
        p = ctypes.c_void_p()
        _check(self._lib.tsp_symbolic(self._h, A._t, B._t, ctypes.byref(p), self._stream()))
        return Plan(self, p)

    def numeric(self, A: "Tiles", B: "Tiles", plan: "Plan") -> DeviceCSR:
        out = _Csr()
        _check(self._lib.tsp_numeric(self._h, A._t, B._t, plan._p, ctypes.byref(out), self._stream()))
        return self._wrap_output(out)


class Tiles:
    """tsp_tiles: a matrix in tile format on the device."""

    def __init__(self, handle: Handle, t):
        self._handle, self._t = handle, t

    def free(self):
        if self._t:
            _check(self._handle._lib.tsp_tiles_free(self._handle._h, self._t, self._handle._stream()))
            self._t = ctypes.c_void_p()

    def view(self) -> dict:
        """Tensor views of the tile arrays (tsp_tiles_view).  The per-tile arrays have tile_slots
        elements; only the indices tile_row_ptr[I] .. tile_row_end[I]-1 of every tile-row hold tiles."""
        h, torch = self._handle, self._handle._torch
        v = _TilesView()
        _check(h._lib.tsp_tiles_get_view(self._t, ctypes.byref(v)))
        n = v.tile_slots
        out = dict(rows=v.rows, cols=v.cols, tile_rows=v.tile_rows, tile_cols=v.tile_cols, ntiles=v.ntiles,
                   tile_slots=n, forms=v.forms,
                   tile_row_ptr=h._view(v.tile_row_ptr, v.tile_rows, torch.int32),
                   tile_row_end=h._view(v.tile_row_end, v.tile_rows, torch.int32),
                   tile_col=h._view(v.tile_col, n, torch.int32),
                   row_mask=h._view(v.row_mask, n * 16, torch.int16),
                   left_group_mask=h._view(v.left_group_mask, n, torch.int32),
                   right_group_mask=h._view(v.right_group_mask, n, torch.int32))
        if v.forms & FORM_LEFT:
            out["left_group_off"] = h._view(v.left_head, n * 2, torch.int32).view(n, 2)[:, 1]
            out["left_elements"] = h._view(v.left_elements, v.left_groups_capacity * 8, torch.float16)
        if v.forms & FORM_RIGHT:
            out["right_group_off"] = h._view(v.right_head, n * 2, torch.int32).view(n, 2)[:, 1]
            out["right_elements"] = h._view(v.right_elements, v.right_groups_capacity * 8, torch.float16)
        return out


def tile_indices(view: dict):
    """The tile indices of a tile matrix in storage order (tile-row by tile-row), as a tensor."""
    torch = _torch()
    begin, end = view["tile_row_ptr"].to(torch.int64), view["tile_row_end"].to(torch.int64)
    counts = end - begin
    starts = torch.repeat_interleave(begin, counts)
    first = torch.cumsum(counts, 0) - counts
    within = torch.arange(int(counts.sum()), device=begin.device) - torch.repeat_interleave(first, counts)
    return starts + within


class Plan:
    """tsp_plan: task list and output pattern of one product."""

    def __init__(self, handle: Handle, p):
        self._handle, self._p = handle, p

    def free(self):
        if self._p:
            _check(self._handle._lib.tsp_plan_free(self._handle._h, self._p, self._handle._stream()))
            self._p = ctypes.c_void_p()

    def view(self) -> dict:
        h, torch = self._handle, self._handle._torch
        v = _PlanView()
        _check(h._lib.tsp_plan_get_view(self._p, ctypes.byref(v)))
        return dict(c_rows=v.c_rows, c_cols=v.c_cols, c_tile_rows=v.c_tile_rows, c_tiles=v.c_tiles, pairs=v.pairs,
                    c_nnz=v.c_nnz, candidate_pairs=v.candidate_pairs,
                    c_tile_row_ptr=h._view(v.c_tile_row_ptr, v.c_tile_rows + 1, torch.int32),
                    c_tile_row=h._view(v.c_tile_row, v.c_tiles, torch.int32),
                    c_tile_col=h._view(v.c_tile_col, v.c_tiles, torch.int32),
                    pair_off=h._view(v.pair_off, v.c_tiles + 1, torch.int64),
                    pair_a=h._view(v.pair_ab, 2 * v.pairs, torch.int32)[0::2],
                    pair_b=h._view(v.pair_ab, 2 * v.pairs, torch.int32)[1::2],
                    c_row_mask=h._view(v.c_row_mask, v.c_tiles * 16, torch.int16),
                    c_row_off=h._view(v.c_row_off, v.c_tiles * 16, torch.int32),
                    c_row_ptr=h._view(v.c_row_ptr, v.c_rows + 1, torch.int64))
