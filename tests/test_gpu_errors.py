"""Error paths of the C ABI, forced from the host: every condition here is one the library detects itself
(on the host, or through its own range checks on the device), so every kernel still runs to its end.
Needs an MI355X."""
import ctypes

import numpy as np
import pytest

from paper_2009_14600_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tsp():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2009_14600_amd import tsp as binding
    binding.load_library()
    return binding


class _FailingHandle:
    """A handle whose allocator callback returns NULL from its k-th call on (k counted from 0)."""

    def __init__(self, tsp, fail_from):
        import torch
        self.calls = 0
        self.blocks = {}

        def alloc(_user, nbytes, _stream):
            k = self.calls
            self.calls += 1
            if k >= fail_from:
                return None
            t = torch.empty(int(nbytes), dtype=torch.uint8, device="cuda")
            self.blocks[t.data_ptr()] = t
            return t.data_ptr()

        def free(_user, ptr, _stream):
            self.blocks.pop(ptr, None)

        self._cb = (tsp._ALLOC_FN(alloc), tsp._FREE_FN(free))
        self._allocator = tsp._Allocator(self._cb[0], self._cb[1], None)
        self.lib = tsp.load_library()
        self.h = ctypes.c_void_p()
        assert self.lib.tsp_create(ctypes.byref(self.h), ctypes.byref(self._allocator)) == 0

    def close(self):
        self.lib.tsp_destroy(self.h)


@pytest.mark.parametrize("maker,tile_edge", [
    (lambda: inputs.config(2, small=True), 0),   # list kernel, whole-tile-row multiplication kernel
    (lambda: inputs.config(4, small=True), 0),   # general task-list kernel, separate counting kernel
    (lambda: inputs.config(1, small=True), 8),   # the paper's pipeline (tsp_spgemm_paper) at two tile edges
    (lambda: inputs.config(5, small=True), 32),
])
def test_allocator_returning_null_at_every_call_site(tsp, maker, tile_edge):
    """tsp_spgemm (tile_edge 0) or tsp_spgemm_paper with an allocator that runs dry after k calls, for every k
    up to the number of calls a successful product makes: status -4 (TSP_ERR_ALLOC_FAILED), *C zeroed, nothing
    leaked (after tsp_trim the handle holds no byte and the allocator has every block back), and the handle
    works again once memory is there."""
    import torch
    A = maker()
    dA = tsp.to_device(A)
    sA = dA._struct()

    def multiply(handle, out):
        if tile_edge:
            return handle.lib.tsp_spgemm_paper(handle.h, tile_edge, ctypes.byref(sA), ctypes.byref(sA), ctypes.byref(out), None)
        return handle.lib.tsp_spgemm(handle.h, ctypes.byref(sA), ctypes.byref(sA), ctypes.byref(out), None)

    ok = _FailingHandle(tsp, fail_from=1 << 30)
    out = tsp._Csr()
    assert multiply(ok, out) == 0
    torch.cuda.synchronize()
    want_nnz, calls = out.nnz, ok.calls
    # what a handle keeps for its whole life (the slots of its chained prefix sums), to tell it from a leak
    assert ok.lib.tsp_csr_free(ok.h, ctypes.byref(out), None) == 0 and ok.lib.tsp_trim(ok.h, None) == 0
    st = tsp._Stats()
    assert ok.lib.tsp_get_stats(ok.h, ctypes.byref(st)) == 0
    kept_bytes, kept_blocks = st.workspace_bytes, len(ok.blocks)
    assert kept_blocks <= 1
    ok.close()
    assert calls >= 10
    for k in range(calls):
        h = _FailingHandle(tsp, fail_from=k)
        out = tsp._Csr(7, 7, 7, 1, 1, 1, 1, 1)
        status = multiply(h, out)
        torch.cuda.synchronize()
        assert status == -4, (k, status)
        assert (out.rows, out.cols, out.nnz, out.row_ptr, out.col_idx, out.val) == (0, 0, 0, None, None, None), k
        assert h.lib.tsp_trim(h.h, None) == 0
        st = tsp._Stats()
        assert h.lib.tsp_get_stats(h.h, ctypes.byref(st)) == 0
        assert st.workspace_bytes in (0, kept_bytes) and len(h.blocks) <= kept_blocks, (k, st.workspace_bytes, len(h.blocks))
        # memory comes back: the same handle multiplies
        h.calls = -(1 << 30)
        out = tsp._Csr()
        assert multiply(h, out) == 0
        torch.cuda.synchronize()
        assert out.nnz == want_nnz
        assert h.lib.tsp_csr_free(h.h, ctypes.byref(out), None) == 0
        h.close()


def test_index_overflow_and_unsupported_span(tsp):
    """-5 (TSP_ERR_INDEX_OVERFLOW): a matrix with 2^31 rows, refused on the host before any array is
    touched.  -7 (TSP_ERR_UNSUPPORTED): a tile-row of C whose candidates lie more than 131072 tile columns
    apart (here 187500), found by the counting kernel's own range check; the handle works afterwards."""
    import torch
    handle = tsp.Handle(validate=True)
    small = tsp.to_device(inputs.random_sparse(20, 20, 0.2, 1))
    s = small._struct()
    huge = tsp._Csr(1 << 31, s.cols, s.nnz, s.row_ptr, s.col_idx, s.val, s.row_ptr_type, s.val_type)
    out = tsp._Csr()
    assert handle._lib.tsp_spgemm(handle._h, ctypes.byref(huge), ctypes.byref(s), ctypes.byref(out), handle._stream()) == -5
    many = tsp._Csr(s.rows, s.cols, 1 << 31, s.row_ptr, s.col_idx, s.val, s.row_ptr_type, s.val_type)
    assert handle._lib.tsp_spgemm(handle._h, ctypes.byref(many), ctypes.byref(s), ctypes.byref(out), handle._stream()) == -5
    N = 3_000_000
    A = inputs.from_coo(16, 16, [0, 3], [0, 5], [1.0, 2.0])
    B = inputs.from_coo(16, N, [0, 0, 5], [0, N - 1, 77], [1.0, 1.0, 1.0])
    with pytest.raises(tsp.TspError) as e:
        handle.spgemm(tsp.to_device(A), tsp.to_device(B))
    assert e.value.status == -7
    C = handle.spgemm(small, small)
    assert C.nnz > 0
    C.free()
    handle.close()
