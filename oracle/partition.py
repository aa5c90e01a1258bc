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


def own_column_counts(row_ptr, col_idx, W: int) -> list[int]:
    """For every row r: how many of its columns occur in none of the W-1 rows that follow it
    (rows past the end of the matrix are simply absent).  This is the quantity Algorithm 1 calls
    the column gain of a head row: the distinct columns of the span [r, r+W) minus the distinct
    columns of the same span without r, i.e. |S_r \\ (S_{r+1} u ... u S_{r+W-1})|."""
    n = len(row_ptr) - 1
    cols_of = [frozenset(int(c) for c in col_idx[row_ptr[i]:row_ptr[i + 1]]) for i in range(n)]
    own = []
    for r in range(n):
        followers = frozenset().union(*cols_of[r + 1:r + W]) if r + 1 < n and W > 1 else frozenset()
        own.append(len(cols_of[r] - followers))
    return own


def partition_rows(row_ptr, col_idx, W: int, tau_nnz: int, tau_inc: int):
    """Returns (window_starts, residual_rows), both ascending lists of row ids.

    Written as a scan over two per-row quantities computed beforehand -- the row length and the
    row's own-column count (``own_column_counts``) -- which decide, for whichever row the scan
    finds at the head of a span, whether that row leaves for the residual set (short and gaining
    fewer than tau_inc columns) or the span of W rows becomes a window."""
    n = len(row_ptr) - 1
    length = [int(row_ptr[i + 1] - row_ptr[i]) for i in range(n)]
    own = own_column_counts(row_ptr, col_idx, W)
    leaves = [length[r] > 0 and length[r] <= tau_nnz and own[r] < tau_inc for r in range(n)]
    windows, residual = [], []
    head = 0
    while head < n:
        if length[head] == 0:
            head += 1                      # empty rows belong to neither set
        elif leaves[head]:
            residual.append(head)
            head += 1
        else:
            windows.append(head)
            head += W
    return windows, residual
