"""Workspace canaries (TSP_OPT_WORKSPACE_CANARIES): every block the handle hands out carries a guard zone in
front of and behind the part in use; no kernel of either path may change a word of them.  Needs an MI355X."""
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


def _guarded_handle(tsp):
    h = tsp.Handle(validate=True)
    h.set_option(tsp.OPT_WORKSPACE_CANARIES, 1)
    return h


def test_no_kernel_writes_outside_its_arrays(tsp, oracle):
    """The small instances of the five workloads (each twice: the second call takes what the handle kept of
    the first), the paper's pipeline at its three tile edges, the compaction of zeros, ragged rectangular
    products, a product whose tile-rows pass the symbolic window and one with very many candidates per
    tile-row: results as the oracle's, and not one guard word changed."""
    h = _guarded_handle(tsp)
    try:
        cases = [(inputs.config(i, small=True), None) for i in (1, 2, 3, 4, 5)]
        for seed in range(12):
            rng = np.random.default_rng(500 + seed)
            M, K, N = (int(x) for x in rng.integers(1, 300, 3))
            d = float(10 ** rng.uniform(-2.2, -0.3))
            cases.append((inputs.random_sparse(M, K, d, 600 + seed, empty_row_fraction=0.1),
                          inputs.random_sparse(K, N, d, 700 + seed, empty_row_fraction=0.1)))
        cases.append((inputs.random_sparse(40, 64, 0.5, 11), inputs.random_sparse(64, 70000, 0.05, 12)))
        cases.append((inputs.random_sparse(2048, 2048, 0.02, 4711, values="smallint"), None))
        for A, B in cases:
            print(f"canaries: {A.name} {A.rows}x{A.cols}, nnz {A.nnz}", flush=True)
            ref = oracle.spgemm(A, A if B is None else B, threads=4)
            dA = tsp.to_device(A)
            dB = dA if B is None else tsp.to_device(B)
            for call in (1, 2):
                C = h.spgemm(dA, dB)
                row_ptr, col, _ = C.to_host()
                assert np.array_equal(row_ptr, ref.row_ptr) and np.array_equal(col, ref.col)
                if call == 2:
                    Z = h.compact_zeros(C)
                    assert Z.nnz <= C.nnz
                    Z.free()
                C.free()
            if ref.col.size < 2_000_000:
                for T in (8, 16, 32):
                    C = h.spgemm_paper(dA, dB, T)
                    assert np.array_equal(C.to_host()[1], ref.col)
                    C.free()
        h.trim()
        assert h.stats()["workspace_violations"] == 0
    finally:
        h.close()


def test_a_word_changed_next_to_an_array_is_counted(tsp):
    """The check itself: one word behind the values of C and one in front of its column indices are changed
    from the host side (both lie in guard zones of blocks this handle owns); releasing C counts two."""
    import torch
    h = _guarded_handle(tsp)
    try:
        A = tsp.to_device(inputs.random_sparse(60, 60, 0.2, 5))
        C = h.spgemm(A, A)
        assert h.stats()["workspace_violations"] == 0
        behind_values = C._raw.val + ((C.nnz * 4 + 255) // 256) * 256
        in_front_of_columns = C._raw.col_idx - 4
        h._view(behind_values, 1, torch.int32).fill_(7)
        h._view(in_front_of_columns, 1, torch.int32).fill_(7)
        torch.cuda.synchronize()
        C.free()
        assert h.stats()["workspace_violations"] == 2
        # switched off, blocks are handed out as they are, and the count stays
        h.set_option(tsp.OPT_WORKSPACE_CANARIES, 0)
        C = h.spgemm(A, A)
        C.free()
        assert h.stats()["workspace_violations"] == 2
    finally:
        h.close()
