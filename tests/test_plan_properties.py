"""Property tests of the host planner on random small matrices and random options (no GPU)."""
import numpy as np
from hypothesis import given, settings, strategies as st

from paper_2603_08734_amd import Plan
from workloads import from_coo


@st.composite
def matrices(draw):
    n_rows = draw(st.integers(1, 70))
    n_cols = draw(st.integers(1, 90))
    density = draw(st.sampled_from([0.0, 0.02, 0.1, 0.4, 1.0]))
    seed = draw(st.integers(0, 2**31 - 1))
    rng = np.random.default_rng(seed)
    mask = rng.random((n_rows, n_cols)) < density
    if draw(st.booleans()) and n_rows > 2:
        mask[rng.integers(0, n_rows)] = True          # one full row
    r, c = np.nonzero(mask)
    vals = rng.standard_normal(r.size)
    vals[rng.random(r.size) < 0.1] = 0.0               # stored zeros must survive
    return from_coo(r, c, vals, n_rows, n_cols)


options = st.fixed_dictionaries({
    "window_rows": st.sampled_from([16, 32, 64]),
    "tile_k": st.sampled_from([16, 32]),
    "partition": st.sampled_from([0, 1]),
    "reorder": st.sampled_from([0, 1]),
    "force_path": st.sampled_from([0, 0, 1, 2]),
    "max_tiles_per_item": st.sampled_from([0, 1, 3]),
    "max_nnz_per_slice": st.sampled_from([0, 17, 40]),
    "xcd_partition_nnz": st.sampled_from([0, -1, 20]),
    "hub_windows": st.sampled_from([0, 1]),
    "long_row_nnz": st.sampled_from([0, 8]),
    "min_reuse": st.sampled_from([0.0, 1.25, 3.0]),
    "tau_nnz": st.sampled_from([-1, 0, 3]),
})


@settings(max_examples=150, deadline=None)
@given(matrices(), options, st.sampled_from([16, 32, 48, 128, 512]))
def test_any_plan_decodes_to_the_input_bit_exactly(A, opts, N):
    p = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, upload=0, **opts)
    row_ptr, col_idx, val, path = p.decode()
    assert np.array_equal(row_ptr, A.row_ptr)
    assert np.array_equal(col_idx, A.col_idx)
    assert np.array_equal(val, A.val.view(np.uint16))
    s = p.stats()
    assert s["nnz_tile"] + s["nnz_irregular"] == A.nnz
    assert int((path == 0).sum()) == s["nnz_tile"]
    assert np.array_equal(np.sort(p.row_order()), np.arange(A.n_rows))
    p.destroy()
