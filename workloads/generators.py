"""Seeded synthetic sparse workloads shaped like the paper's evaluation inputs.

The paper evaluates on GNN graphs with heavy-tailed row lengths (Section 2.2
and the dataset table of Section 4.1), on scientific matrices from a public
collection, on a row-reordering study, and motivates sparse LLM inference.
None of those datasets is available here, so each family is replaced by a
seeded generator of the same shape.  This module holds *only* input
generation: no SpMM arithmetic, no planning, no tiling.  It is the single
piece of code shared by the CPU oracle's tests and the GPU path's tests.

Every generator draws from one ``numpy.random.default_rng(seed)`` in the
order documented in its docstring, and returns a canonical CSR matrix
(column indices strictly increasing inside each row, no duplicates).
Values are rounded to IEEE binary16 exactly once.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field

import numpy as np


@dataclass
class CSR:
    """Canonical CSR matrix with fp16 values.

    row_ptr : int64 [n_rows+1], col_idx : int32 [nnz], val : float16 [nnz].
    ``meta`` carries generator-side ground truth (never read by the library).
    """

    n_rows: int
    n_cols: int
    row_ptr: np.ndarray
    col_idx: np.ndarray
    val: np.ndarray
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])

    def checksum(self) -> str:
        h = hashlib.sha256()
        h.update(np.ascontiguousarray(self.row_ptr).tobytes())
        h.update(np.ascontiguousarray(self.col_idx).tobytes())
        h.update(np.ascontiguousarray(self.val).view(np.uint16).tobytes())
        return h.hexdigest()[:16]

    def row_nnz(self) -> np.ndarray:
        return np.diff(self.row_ptr)


def csr_from_sorted_keys(keys: np.ndarray, n_rows: int, n_cols: int) -> tuple[np.ndarray, np.ndarray]:
    """keys = row * n_cols + col, sorted and unique -> (row_ptr, col_idx)."""
    rows = keys // n_cols
    cols = (keys - rows * n_cols).astype(np.int32)
    counts = np.bincount(rows, minlength=n_rows).astype(np.int64)
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr, cols


def from_coo(rows, cols, vals, n_rows: int, n_cols: int, meta=None) -> CSR:
    """Build canonical CSR from duplicate-free COO triplets (any order)."""
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.asarray(cols, dtype=np.int64)
    keys = rows * n_cols + cols
    order = np.argsort(keys, kind="stable")
    keys = keys[order]
    if keys.size > 1 and np.any(keys[1:] == keys[:-1]):
        raise ValueError("duplicate (row, col) in COO input")
    row_ptr, col_idx = csr_from_sorted_keys(keys, n_rows, n_cols)
    val = np.asarray(vals)[order].astype(np.float16)
    return CSR(n_rows, n_cols, row_ptr, col_idx, val, meta or {})


# --------------------------------------------------------------------------
# 1. tiny uniform
# --------------------------------------------------------------------------
def uniform_rows(n_rows=4096, n_cols=4096, per_row=16, seed=0) -> CSR:
    """Each row holds ``per_row`` distinct uniform-random columns, values U[-1,1].

    Draw order: (1) an n_rows x n_cols matrix of float64 keys whose per-row
    ``per_row`` smallest entries select the columns; (2) nnz uniform values.
    """
    rng = np.random.default_rng(seed)
    per_row = min(per_row, n_cols)
    keys = rng.random((n_rows, n_cols))
    cols = np.argpartition(keys, per_row - 1, axis=1)[:, :per_row] if per_row < n_cols else np.tile(np.arange(n_cols), (n_rows, 1))
    cols = np.sort(cols, axis=1).astype(np.int32)
    row_ptr = np.arange(n_rows + 1, dtype=np.int64) * per_row
    val = rng.uniform(-1.0, 1.0, size=n_rows * per_row).astype(np.float16)
    return CSR(n_rows, n_cols, row_ptr, cols.reshape(-1), val, {"family": "uniform"})


# --------------------------------------------------------------------------
# 2. R-MAT power-law graph, GCN-normalised
# --------------------------------------------------------------------------
def rmat_gcn(scale=20, avg_degree=16, a=0.57, b=0.19, c=0.19, seed=0) -> CSR:
    """R-MAT graph on 2**scale vertices, symmetrised, deduplicated, self-loops
    added, values D^-1/2 (A+I) D^-1/2 rounded once to fp16.

    ``avg_degree * 2**scale`` directed edges are drawn; every edge takes
    ``scale`` recursive quadrant choices with probabilities (a, b, c, 1-a-b-c),
    no noise and no vertex relabelling.  Draw order: one float32 vector of
    length n_edges per recursion level, most significant bit first.
    D is the row sum of the 0/1 pattern after symmetrisation and self-loops.
    """
    rng = np.random.default_rng(seed)
    n = 1 << scale
    n_edges = avg_degree * n
    src = np.zeros(n_edges, dtype=np.int64)
    dst = np.zeros(n_edges, dtype=np.int64)
    ab, abc = a + b, a + b + c
    for _ in range(scale):
        u = rng.random(n_edges, dtype=np.float32)
        row_bit = u >= ab                      # quadrants c, d
        col_bit = ((u >= a) & (u < ab)) | (u >= abc)   # quadrants b, d
        src = (src << 1) | row_bit
        dst = (dst << 1) | col_bit
    diag = np.arange(n, dtype=np.int64)
    keys = np.concatenate([src * n + dst, dst * n + src, diag * n + diag])
    del src, dst
    keys = np.unique(keys)
    row_ptr, col_idx = csr_from_sorted_keys(keys, n, n)
    del keys
    deg = np.diff(row_ptr).astype(np.float64)
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(row_ptr))
    val = (1.0 / np.sqrt(deg[rows] * deg[col_idx])).astype(np.float16)
    return CSR(n, n, row_ptr, col_idx, val, {"family": "rmat_gcn", "scale": scale})


# --------------------------------------------------------------------------
# 3. 27-point stencil on a cubic grid, natural ordering
# --------------------------------------------------------------------------
def stencil27(n=96, jitter=True, seed=0) -> CSR:
    """27-point Laplacian-style matrix on an n^3 grid, row = (z*n + y)*n + x.

    Centre coefficient 26.0; each in-grid neighbour -1.0 (+ U[-0.1, 0.1] when
    ``jitter``).  Draw order: one uniform per stored off-diagonal entry, in
    CSR order.  nnz = (3n-2)^3.
    """
    rng = np.random.default_rng(seed)
    idx = np.arange(n, dtype=np.int32)
    z, y, x = np.meshgrid(idx, idx, idx, indexing="ij")
    z, y, x = z.reshape(-1), y.reshape(-1), x.reshape(-1)
    n_rows = n ** 3
    cols = np.empty((n_rows, 27), dtype=np.int32)
    valid = np.empty((n_rows, 27), dtype=bool)
    k = 0
    for dz in (-1, 0, 1):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                zz, yy, xx = z + dz, y + dy, x + dx
                ok = (zz >= 0) & (zz < n) & (yy >= 0) & (yy < n) & (xx >= 0) & (xx < n)
                cols[:, k] = (zz * n + yy) * n + xx
                valid[:, k] = ok
                k += 1
    counts = valid.sum(axis=1).astype(np.int64)
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    is_centre = np.zeros((n_rows, 27), dtype=bool)
    is_centre[:, 13] = True
    col_idx = cols[valid]
    centre = is_centre[valid]
    val = np.full(col_idx.shape[0], -1.0, dtype=np.float64)
    if jitter:
        off = ~centre
        val[off] += rng.uniform(-0.1, 0.1, size=int(off.sum()))
    val[centre] = 26.0
    return CSR(n_rows, n_rows, row_ptr, col_idx.astype(np.int32), val.astype(np.float16),
               {"family": "stencil27", "grid": n})


# --------------------------------------------------------------------------
# 4. hidden-locality community matrix
# --------------------------------------------------------------------------
def hidden_communities(n_comm=8192, comm_size=64, density=0.30, long_range=4,
                       permute=True, seed=0) -> CSR:
    """Block-diagonal communities hidden by random row and column permutations.

    Draw order: (1) n_comm x comm_size x comm_size float32 Bernoulli(density)
    field; (2) n x long_range uniform column indices; (3) row permutation;
    (4) column permutation; (5) one N(0,1) value per stored entry in final CSR
    order.  ``meta['row_comm'][r]`` is the planted community of output row r.
    """
    rng = np.random.default_rng(seed)
    n = n_comm * comm_size
    blk = rng.random((n_comm, comm_size, comm_size), dtype=np.float32) < density
    cid, ri, ci = np.nonzero(blk)
    rows = cid.astype(np.int64) * comm_size + ri
    cols = cid.astype(np.int64) * comm_size + ci
    del blk, cid, ri, ci
    lr_cols = rng.integers(0, n, size=(n, long_range), dtype=np.int64)
    lr_rows = np.repeat(np.arange(n, dtype=np.int64), long_range)
    if permute:
        p_r = rng.permutation(n).astype(np.int64)
        p_c = rng.permutation(n).astype(np.int64)
    else:
        p_r = np.arange(n, dtype=np.int64)
        p_c = np.arange(n, dtype=np.int64)
    all_rows = p_r[np.concatenate([rows, lr_rows])]
    all_cols = p_c[np.concatenate([cols, lr_cols.reshape(-1)])]
    keys = np.unique(all_rows * n + all_cols)
    row_ptr, col_idx = csr_from_sorted_keys(keys, n, n)
    val = rng.standard_normal(keys.shape[0]).astype(np.float16)
    row_comm = np.empty(n, dtype=np.int32)
    row_comm[p_r] = (np.arange(n) // comm_size).astype(np.int32)
    col_comm = np.empty(n, dtype=np.int32)
    col_comm[p_c] = (np.arange(n) // comm_size).astype(np.int32)
    return CSR(n, n, row_ptr, col_idx, val,
               {"family": "hidden_communities", "row_comm": row_comm, "col_comm": col_comm,
                "comm_size": comm_size})


# --------------------------------------------------------------------------
# 5. pruned LLM weight
# --------------------------------------------------------------------------
def pruned_weight(n_rows=28672, n_cols=8192, keep=0.20, row_jitter=0.5, std=0.02, seed=0) -> CSR:
    """Unstructured random mask; row r keeps each entry with probability
    keep * (1 + u_r), u_r ~ U[-row_jitter, row_jitter]; values N(0, std).

    Draw order: (1) n_rows uniforms u_r; (2) mask field in chunks of 1024
    rows (float32); (3) one normal per stored entry in CSR order.
    """
    rng = np.random.default_rng(seed)
    p_row = keep * (1.0 + rng.uniform(-row_jitter, row_jitter, size=n_rows))
    col_chunks, counts = [], np.zeros(n_rows, dtype=np.int64)
    for r0 in range(0, n_rows, 1024):
        r1 = min(n_rows, r0 + 1024)
        m = rng.random((r1 - r0, n_cols), dtype=np.float32) < p_row[r0:r1, None].astype(np.float32)
        rr, cc = np.nonzero(m)
        counts[r0:r1] = np.bincount(rr, minlength=r1 - r0)
        col_chunks.append(cc.astype(np.int32))
    col_idx = np.concatenate(col_chunks) if col_chunks else np.zeros(0, np.int32)
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    val = (rng.standard_normal(col_idx.shape[0]) * std).astype(np.float16)
    return CSR(n_rows, n_cols, row_ptr, col_idx, val, {"family": "pruned_weight"})


# --------------------------------------------------------------------------
# dense operand
# --------------------------------------------------------------------------
def dense_B(n_rows: int, n_cols: int, dist: str = "uniform", seed: int = 1) -> np.ndarray:
    """Row-major fp16 dense matrix; dist = 'uniform' (U[-1,1]) or 'normal' (N(0,1))."""
    rng = np.random.default_rng(seed)
    if dist == "uniform":
        out = np.empty((n_rows, n_cols), dtype=np.float16)
        step = max(1, (1 << 24) // max(1, n_cols))
        for r0 in range(0, n_rows, step):
            r1 = min(n_rows, r0 + step)
            out[r0:r1] = rng.uniform(-1.0, 1.0, size=(r1 - r0, n_cols)).astype(np.float16)
        return out
    if dist == "normal":
        out = np.empty((n_rows, n_cols), dtype=np.float16)
        step = max(1, (1 << 24) // max(1, n_cols))
        for r0 in range(0, n_rows, step):
            r1 = min(n_rows, r0 + step)
            out[r0:r1] = rng.standard_normal((r1 - r0, n_cols)).astype(np.float16)
        return out
    raise ValueError(dist)


# --------------------------------------------------------------------------
# the five named configurations (full size) and reduced versions of each
# --------------------------------------------------------------------------
CONFIGS = {
    1: dict(name="tiny_uniform_4096", N=32, B_dist="uniform"),
    2: dict(name="rmat_gcn_2e20", N=128, B_dist="normal"),
    3: dict(name="stencil27_96", N=64, B_dist="uniform"),
    4: dict(name="hidden_communities_524288", N=256, B_dist="uniform"),
    5: dict(name="pruned_llm_28672x8192", N=128, B_dist="normal"),
}


def make_config(k: int, seed: int = 0, small: bool = False) -> tuple[CSR, int, str]:
    """Return (A, N, B_dist) for configuration k (1..5).

    ``small=True`` keeps the recipe but shrinks the matrix so that the CPU
    oracle finishes in well under a second (used by tests on machines with
    no GPU and by the per-element parity tests).
    """
    cfg = CONFIGS[k]
    if k == 1:
        A = uniform_rows(4096 if not small else 512, 4096 if not small else 512, 16, seed)
    elif k == 2:
        A = rmat_gcn(20 if not small else 12, 16, seed=seed)
    elif k == 3:
        A = stencil27(96 if not small else 14, True, seed)
    elif k == 4:
        A = hidden_communities(8192 if not small else 48, 64, 0.30, 4, True, seed)
    elif k == 5:
        A = (pruned_weight(28672, 8192, seed=seed) if not small
             else pruned_weight(448, 1024, seed=seed))
    else:
        raise KeyError(k)
    A.meta["config"] = k
    A.meta["name"] = cfg["name"] + ("_small" if small else "")
    return A, cfg["N"], cfg["B_dist"]
