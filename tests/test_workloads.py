"""Structure checks of the seeded input generators (no GPU)."""
import numpy as np
import pytest

from workloads import dense_B, hidden_communities, make_config, rmat_gcn, stencil27


def assert_canonical(A):
    assert A.row_ptr[0] == 0 and A.row_ptr[-1] == A.col_idx.shape[0] == A.val.shape[0]
    assert np.all(np.diff(A.row_ptr) >= 0)
    assert A.col_idx.dtype == np.int32 and A.val.dtype == np.float16 and A.row_ptr.dtype == np.int64
    if A.nnz:
        assert A.col_idx.min() >= 0 and A.col_idx.max() < A.n_cols
        d = np.diff(A.col_idx.astype(np.int64))
        row_end = np.zeros(A.nnz - 1, dtype=bool)
        ends = A.row_ptr[1:-1] - 1
        ends = ends[(ends >= 0) & (ends < A.nnz - 1)]
        row_end[ends] = True
        assert np.all(d[~row_end] > 0)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_reduced_configs_are_canonical_and_seeded(k):
    A, N, dist = make_config(k, small=True)
    assert_canonical(A)
    A2, _, _ = make_config(k, small=True)
    assert A.checksum() == A2.checksum()
    A3, _, _ = make_config(k, seed=1, small=True)
    assert A.checksum() != A3.checksum()


def test_rmat_is_symmetric_with_unit_diagonal_pattern():
    A = rmat_gcn(scale=10, avg_degree=16, seed=0)
    assert_canonical(A)
    rows = np.repeat(np.arange(A.n_rows, dtype=np.int64), A.row_nnz())
    keys = rows * A.n_cols + A.col_idx
    keys_t = np.sort(A.col_idx.astype(np.int64) * A.n_cols + rows)
    assert np.array_equal(keys, keys_t)
    assert np.all(np.isin(np.arange(A.n_rows) * (A.n_cols + 1), keys))
    deg = A.row_nnz().astype(np.float64)
    want = (1.0 / np.sqrt(deg[rows] * deg[A.col_idx])).astype(np.float16)
    assert np.array_equal(A.val.view(np.uint16), want.view(np.uint16))
    assert A.row_nnz().max() > 8 * A.row_nnz().mean()        # heavy tail


def test_stencil_counts():
    A = stencil27(6)
    assert_canonical(A)
    assert A.nnz == (3 * 6 - 2) ** 3 and A.row_nnz().max() == 27 and A.row_nnz().min() == 8
    rows = np.repeat(np.arange(A.n_rows), A.row_nnz())
    diag = A.val[rows == A.col_idx].astype(np.float64)
    off = A.val[rows != A.col_idx].astype(np.float64)
    assert np.all(diag == 26.0) and np.all(np.abs(off + 1.0) <= 0.1 + 1e-3)


def test_hidden_communities_are_hidden_but_recoverable():
    A = hidden_communities(n_comm=16, seed=0)
    assert_canonical(A)
    rc, cc = A.meta["row_comm"], A.meta["col_comm"]
    rows = np.repeat(np.arange(A.n_rows), A.row_nnz())
    same = rc[rows] == cc[A.col_idx]
    assert 0.75 < same.mean() < 0.9          # ~19.2 intra + ~4 long-range per row
    assert np.mean(rc[1:] == rc[:-1]) < 0.2  # neighbours in the given order rarely share a community


def test_dense_B_distributions():
    U = dense_B(1000, 16, "uniform", seed=0).astype(np.float64)
    Z = dense_B(1000, 16, "normal", seed=0).astype(np.float64)
    assert U.min() >= -1 and U.max() <= 1 and abs(U.mean()) < 0.02
    assert abs(Z.std() - 1) < 0.03
