"""Weighted Jaccard row similarity and the reordering objective (paper,
Section 3.4) -- TEST INFRASTRUCTURE ONLY, plain Python in fp64.

Column j occurring in d_j rows gets weight w_j = d_j ** (-alpha), alpha > 0.
The affinity of two rows is the weight of the columns they share divided by
the weight of the columns either has.  An ordering pi is scored by the sum of
(1 - sim) over consecutive pairs; the reordering heuristic tries to make that
sum small.
"""
from __future__ import annotations

import numpy as np


def column_degree(col_idx, n_cols: int) -> np.ndarray:
    return np.bincount(np.asarray(col_idx, dtype=np.int64), minlength=n_cols).astype(np.int64)


def row_set(row_ptr, col_idx, r: int) -> set:
    return set(int(c) for c in col_idx[row_ptr[r]:row_ptr[r + 1]])


def w_jaccard(set_r: set, set_u: set, degree, alpha: float) -> float:
    union = set_r | set_u
    if not union:
        return 0.0
    num = sum(float(degree[j]) ** (-alpha) for j in sorted(set_r & set_u))
    den = sum(float(degree[j]) ** (-alpha) for j in sorted(union))
    return num / den


def path_cost(row_ptr, col_idx, n_cols: int, order, alpha: float) -> float:
    """sum_{i} (1 - sim(order[i], order[i+1]))."""
    degree = column_degree(col_idx, n_cols)
    total = 0.0
    prev = row_set(row_ptr, col_idx, int(order[0])) if len(order) else set()
    for i in range(1, len(order)):
        cur = row_set(row_ptr, col_idx, int(order[i]))
        total += 1.0 - w_jaccard(prev, cur, degree, alpha)
        prev = cur
    return total
