"""Pins for the CPU SpMM oracle (no GPU).

The oracle is checked against things it does not itself define: numpy's
binary16 decoding, a brute-force dense product, closed forms, algebraic
invariants and scipy's sparse product.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import spmm as oracle
from workloads import dense_B, from_coo, make_config, stencil27

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_csr(rng, n_rows, n_cols, density, empty_rows=(), full_rows=()):
    mask = rng.random((n_rows, n_cols)) < density
    for r in empty_rows:
        mask[r, :] = False
    for r in full_rows:
        mask[r, :] = True
    rows, cols = np.nonzero(mask)
    vals = rng.uniform(-2, 2, size=rows.shape[0])
    return from_coo(rows, cols, vals, n_rows, n_cols)


def dense_of(A):
    D = np.zeros((A.n_rows, A.n_cols), dtype=np.float64)
    rows = np.repeat(np.arange(A.n_rows), A.row_nnz())
    D[rows, A.col_idx] = A.val.astype(np.float64)
    return D


def test_half_decoding_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.half_bits_to_double(bits)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


@pytest.mark.parametrize("shape", [(1, 1, 1), (7, 5, 3), (33, 64, 16), (64, 17, 9), (40, 40, 1)])
def test_against_bruteforce_dense_product(shape):
    n_rows, n_cols, N = shape
    rng = np.random.default_rng(123 + n_rows)
    A = random_csr(rng, n_rows, n_cols, 0.3, empty_rows=[0] if n_rows > 2 else [],
                   full_rows=[n_rows - 1] if n_rows > 2 else [])
    B = rng.uniform(-1, 1, size=(n_cols, N)).astype(np.float16)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    D = dense_of(A)
    want = D @ B.astype(np.float64)
    want_S = np.abs(D) @ np.abs(B.astype(np.float64))
    # both are fp64 sums of the same exact products; only the order may differ
    assert np.all(np.abs(C - want) <= 1e-13 * want_S + 1e-300)
    assert np.all(np.abs(S - want_S) <= 1e-13 * want_S + 1e-300)
    if n_rows > 2:
        assert np.all(C[0] == 0) and np.all(S[0] == 0)


def test_non_square_operands_not_transposed():
    # a single entry at (row 1, col 3) picks row 3 of B into row 1 of C
    A = from_coo([1], [3], [2.0], 2, 5)
    B = np.arange(5 * 4, dtype=np.float64).reshape(5, 4).astype(np.float16)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert np.array_equal(C[1], 2.0 * B[3].astype(np.float64))
    assert np.all(C[0] == 0)
    assert np.array_equal(S[1], 2.0 * np.abs(B[3].astype(np.float64)))


def test_identity_gives_B_exactly():
    n, N = 50, 24
    A = from_coo(np.arange(n), np.arange(n), np.ones(n), n, n)
    B = dense_B(n, N, "normal", seed=5)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert np.array_equal(C, B.astype(np.float64))
    assert np.array_equal(S, np.abs(B.astype(np.float64)))


def test_permutation_matrix_gathers_rows():
    rng = np.random.default_rng(3)
    n, N = 37, 8
    perm = rng.permutation(n)
    A = from_coo(np.arange(n), perm, np.ones(n), n, n)
    B = dense_B(n, N, "uniform", seed=6)
    C, _, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert np.array_equal(C, B.astype(np.float64)[perm])


def test_single_entry_rows_are_exact_products():
    rng = np.random.default_rng(4)
    n, m, N = 20, 30, 16
    cols = rng.integers(0, m, size=n)
    vals = rng.standard_normal(n).astype(np.float16)
    A = from_coo(np.arange(n), cols, vals, n, m)
    B = dense_B(m, N, "normal", seed=7)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    want = vals.astype(np.float64)[:, None] * B.astype(np.float64)[cols]
    assert np.array_equal(C, want)
    assert np.array_equal(S, np.abs(want))


def test_subnormal_halves_are_kept():
    tiny = np.array([1, 2, 0x3ff], dtype=np.uint16).view(np.float16)   # subnormal binary16
    A = from_coo([0, 0, 0], [0, 1, 2], tiny, 1, 3)
    B = np.array([[1.0], [1.0], [1.0]], dtype=np.float16)
    C, _, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert C[0, 0] == (1 + 2 + 1023) * 2.0 ** -24


def test_stencil_closed_form_rowsums():
    table = {}
    with open(os.path.join(GOLDEN, "stencil_rowsums.txt")) as f:
        for line in f:
            if line.startswith("boundary_coords"):
                t = line.split()
                table[int(t[1])] = float(t[3])
    n = 7
    A = stencil27(n, jitter=False)
    B = np.ones((A.n_cols, 3), dtype=np.float16)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    idx = np.arange(n)
    z, y, x = np.meshgrid(idx, idx, idx, indexing="ij")
    on_edge = lambda a: ((a == 0) | (a == n - 1)).astype(int)
    e = (on_edge(z) + on_edge(y) + on_edge(x)).reshape(-1)
    want = np.array([table[int(k)] for k in e])
    assert np.array_equal(C, np.repeat(want[:, None], 3, axis=1))
    assert np.array_equal(S[:, 0], 26.0 + (26.0 - want))
    assert A.nnz == (3 * n - 2) ** 3
    assert (e == 0).sum() == (n - 2) ** 3 and (e == 3).sum() == 8


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_against_scipy_on_reduced_configs(k):
    A, N, dist = make_config(k, small=True)
    N = min(N, 32)
    B = dense_B(A.n_cols, N, dist, seed=11)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    M = sp.csr_matrix((A.val.astype(np.float64), A.col_idx, A.row_ptr), shape=(A.n_rows, A.n_cols))
    want = M @ B.astype(np.float64)
    want_S = abs(M) @ np.abs(B.astype(np.float64))
    assert np.all(np.abs(C - want) <= 1e-12 * want_S + 1e-300)
    assert np.all(np.abs(S - want_S) <= 1e-12 * want_S + 1e-300)


def test_scale_is_product_of_absolute_values_and_bounds_C():
    rng = np.random.default_rng(9)
    A = random_csr(rng, 30, 40, 0.2)
    B = dense_B(40, 8, "normal", seed=2)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    C_abs, _, _ = oracle.spmm(A.row_ptr, A.col_idx, np.abs(A.val), np.abs(B))
    assert np.array_equal(S, C_abs)
    assert np.all(np.abs(C) <= S)


def test_linearity_on_disjoint_supports_and_power_of_two_scaling():
    rng = np.random.default_rng(10)
    n, m, N = 25, 31, 8
    mask = rng.random((n, m)) < 0.3
    pick = rng.random((n, m)) < 0.5
    r1, c1 = np.nonzero(mask & pick)
    r2, c2 = np.nonzero(mask & ~pick)
    v1 = rng.standard_normal(r1.size)
    v2 = rng.standard_normal(r2.size)
    A1 = from_coo(r1, c1, v1, n, m)
    A2 = from_coo(r2, c2, v2, n, m)
    A12 = from_coo(np.concatenate([r1, r2]), np.concatenate([c1, c2]), np.concatenate([v1, v2]), n, m)
    B = dense_B(m, N, "uniform", seed=3)
    C1, S1, _ = oracle.spmm(A1.row_ptr, A1.col_idx, A1.val, B)
    C2, S2, _ = oracle.spmm(A2.row_ptr, A2.col_idx, A2.val, B)
    C12, S12, _ = oracle.spmm(A12.row_ptr, A12.col_idx, A12.val, B)
    assert np.all(np.abs(C12 - (C1 + C2)) <= 1e-13 * S12 + 1e-300)
    assert np.all(np.abs(S12 - (S1 + S2)) <= 1e-13 * S12 + 1e-300)
    C4, _, _ = oracle.spmm(A12.row_ptr, A12.col_idx, (A12.val.astype(np.float32) * 4).astype(np.float16), B)
    assert np.array_equal(C4, 4.0 * C12)


def test_row_subset_matches_full_and_threads_do_not_change_bits():
    A, N, dist = make_config(2, small=True)
    B = dense_B(A.n_cols, 16, dist, seed=1)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B, threads=1)
    Cp, Sp, used = oracle.spmm(A.row_ptr, A.col_idx, A.val, B, threads=4)
    assert used == 4
    assert np.array_equal(C, Cp) and np.array_equal(S, Sp)
    rows = np.array([0, 5, 17, A.n_rows - 1, 5], dtype=np.int64)
    Cs, Ss, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B, rows=rows)
    assert np.array_equal(Cs, C[rows]) and np.array_equal(Ss, S[rows])


def test_exact_rational_check_on_tiny_case():
    # every binary16 value is a dyadic rational: check one output against exact arithmetic
    A = from_coo([0, 0, 0], [0, 2, 3], np.array([0.1, -2.5, 3.0], dtype=np.float16), 1, 4)
    B = np.array([[0.3], [9.0], [1.5], [-0.7]], dtype=np.float16)
    C, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    fr = lambda h: Fraction(float(h))
    exact = sum(fr(a) * fr(B[c, 0]) for a, c in zip(A.val, A.col_idx))
    assert Fraction(C[0, 0]) == exact     # three products of 11-bit numbers sum exactly in fp64
