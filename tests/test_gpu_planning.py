"""Planning on the device (Section 3.4, Algorithm 3 step II): the kernel that scores candidate row
pairs must give the host scorer's neighbour lists bit for bit -- same row ids, same affinities --
and therefore the same row order and the same plan."""
import numpy as np
import pytest

from paper_2603_08734_amd import Plan
from paper_2603_08734_amd.binding import RSH_ARR_COUNT, rsh_reorder_knn
from workloads import make_config
from workloads.generators import rmat_gcn

pytestmark = pytest.mark.gpu


def _same_lists(row_ptr, col_idx, n_cols, **kw):
    h_ids, h_sim = rsh_reorder_knn(row_ptr, col_idx, n_cols, device_scoring=0, **kw)
    d_ids, d_sim = rsh_reorder_knn(row_ptr, col_idx, n_cols, device_scoring=1, **kw)
    assert np.array_equal(h_ids, d_ids)
    assert np.array_equal(h_sim.view(np.uint32), d_sim.view(np.uint32))
    return h_ids


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_device_scores_give_the_hosts_neighbour_lists(k):
    A, _, _ = make_config(k, small=True)
    ids = _same_lists(A.row_ptr, A.col_idx, A.n_cols)
    if k != 5:   # config 5's columns are all too frequent to serve as features
        assert (ids >= 0).any()


@pytest.mark.parametrize("kw", [dict(knn_k=1), dict(knn_k=64, alpha=1.0), dict(force_path=2), dict(partition=0, knn_k=3)])
def test_device_scores_under_other_options(kw):
    A, _, _ = make_config(3, small=True)
    _same_lists(A.row_ptr, A.col_idx, A.n_cols, **kw)


def test_device_scores_over_several_blocks_of_rows():
    """More rows than one device table holds (32768), with a ragged last block; heavy-tailed rows."""
    A = rmat_gcn(scale=17, avg_degree=6, seed=21)
    rows = 100_003   # more than three tables, the last one ragged
    ids = _same_lists(A.row_ptr[:rows + 1], A.col_idx[:A.row_ptr[rows]], A.n_cols)
    assert (ids >= 0).sum() > rows


def test_matrices_without_neighbours():
    row_ptr = np.zeros(6, dtype=np.int64)
    _same_lists(row_ptr, np.zeros(0, dtype=np.int32), 7)
    # every row its own column: nobody shares anything
    _same_lists(np.arange(6, dtype=np.int64), np.arange(5, dtype=np.int32), 5)


@pytest.mark.parametrize("k", [2, 4])
def test_plan_does_not_depend_on_where_the_scores_come_from(k):
    A, N, _ = make_config(k, small=True)
    p0 = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, device_scoring=0, min_reuse=1.0)
    p1 = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, device_scoring=1, min_reuse=1.0)
    assert np.array_equal(p0.row_order(), p1.row_order())
    for which in range(RSH_ARR_COUNT):
        assert np.array_equal(p0.array(which), p1.array(which)), which
