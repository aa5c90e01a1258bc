"""Row-level execution partitioning (paper, Section 3.3.1, Algorithm 1) --
TEST INFRASTRUCTURE ONLY, written with plain Python sets.

The scan walks the rows once.  An empty row is skipped.  For a non-empty head
row r the algorithm looks at the W-row span that starts at r and asks how many
distinct columns that span would lose if r were left out of it.  A row that is
short (at most tau_nnz stored entries) *and* contributes fewer than tau_inc
columns of its own is sent to the residual ("CUDA") set and the scan moves on
by one row; otherwise the whole span becomes a window and the scan jumps past
it.  Rows past the end of the matrix are simply absent from a span.

The paper leaves the threshold estimator undefined (it only says the values
are small, plateau around 4-6 and depend on matrix size and sparsity), so the
thresholds are inputs here; ``estimate_threshold`` is this build's reading.
"""
from __future__ import annotations


def estimate_threshold(n_rows: int, nnz: int) -> tuple[int, int]:
    """(tau_nnz, tau_inc): a quarter of the mean row length clamped to [2, 6]
    (the paper's plateau region), and a column-gain threshold of 2."""
    mean = nnz / n_rows if n_rows else 0.0
    return max(2, min(6, int(mean // 4))), 2


def partition_rows(row_ptr, col_idx, W: int, tau_nnz: int, tau_inc: int):
    """Returns (window_starts, residual_rows), both ascending lists of row ids."""
    n = len(row_ptr) - 1
    cols_of = [set(int(c) for c in col_idx[row_ptr[i]:row_ptr[i + 1]]) for i in range(n)]
    windows, residual = [], []
    r = 0
    while r < n:
        own = cols_of[r]
        if not own:
            r += 1
            continue
        rest = set()
        for q in range(r + 1, min(n, r + W)):
            rest |= cols_of[q]
        gain = len(rest | own) - len(rest)
        if gain < tau_inc and len(own) <= tau_nnz:
            residual.append(r)
            r += 1
        else:
            windows.append(r)
            r += W
    return windows, residual
