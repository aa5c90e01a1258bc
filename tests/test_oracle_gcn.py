"""Pins for the GCN-layer oracle (no GPU): finite differences, dense closed forms, special cases."""
import numpy as np
import pytest

from oracle import gcn
from workloads import from_coo


def small_problem(seed, n=9, d_in=5, d_out=4, density=0.35):
    rng = np.random.default_rng(seed)
    mask = rng.random((n, n)) < density
    mask[2, :] = False                       # an empty row
    rows, cols = np.nonzero(mask)
    A = from_coo(rows, cols, rng.uniform(-1.5, 1.5, size=rows.size), n, n)
    H = rng.normal(size=(n, d_in))
    W = rng.normal(size=(d_in, d_out))
    b = rng.normal(size=d_out)
    G = rng.normal(size=(n, d_out))
    return A, H, W, b, G


def dense_of(A):
    D = np.zeros((A.n_rows, A.n_cols))
    for i in range(A.n_rows):
        for p in range(A.row_ptr[i], A.row_ptr[i + 1]):
            D[i, A.col_idx[p]] = float(A.val[p])
    return D


def loss(A, H, W, b, relu, G):
    Y, _ = gcn.layer_forward(A.row_ptr, A.col_idx, A.val, A.n_cols, H, W, b, relu)
    return float((Y * G).sum())


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_backward_matches_central_differences(seed, relu):
    A, H, W, b, G = small_problem(seed)
    dH, dW, db = gcn.layer_backward(A.row_ptr, A.col_idx, A.val, A.n_cols, H, W, b, relu, G)
    eps = 1e-6

    def numeric(X, grad):
        out = np.zeros_like(X)
        for idx in np.ndindex(*X.shape):
            keep = X[idx]
            X[idx] = keep + eps
            up = loss(A, H, W, b, relu, G)
            X[idx] = keep - eps
            dn = loss(A, H, W, b, relu, G)
            X[idx] = keep
            out[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(grad, out, rtol=1e-5, atol=1e-6)

    numeric(H, dH)
    numeric(W, dW)
    numeric(b, db)


@pytest.mark.parametrize("relu", [False, True])
def test_forward_is_the_dense_formula(relu):
    A, H, W, b, _ = small_problem(3)
    D = dense_of(A)
    Z = np.zeros((A.n_rows, W.shape[1]))
    for i in range(A.n_rows):                     # the layer equation, written element by element
        for j in range(W.shape[1]):
            s = b[j]
            for k in range(A.n_cols):
                for l in range(H.shape[1]):
                    s += D[i, k] * H[k, l] * W[l, j]
            Z[i, j] = s
    want = np.maximum(Z, 0) if relu else Z
    for order in ("AH_W", "A_HW"):
        Y, Zo = gcn.layer_forward(A.row_ptr, A.col_idx, A.val, A.n_cols, H, W, b, relu, order)
        np.testing.assert_allclose(Zo, Z, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(Y, want, rtol=1e-12, atol=1e-12)


def test_identity_adjacency_is_a_dense_layer():
    rng = np.random.default_rng(4)
    n = 7
    A = from_coo(np.arange(n), np.arange(n), np.ones(n), n, n)
    H, W, b = rng.normal(size=(n, 3)), rng.normal(size=(3, 6)), rng.normal(size=6)
    Y, _ = gcn.layer_forward(A.row_ptr, A.col_idx, A.val, n, H, W, b, True)
    np.testing.assert_allclose(Y, np.maximum(H @ W + b, 0), rtol=1e-13, atol=1e-13)


def test_empty_row_gives_activation_of_bias():
    A, H, W, b, _ = small_problem(5)
    Y, _ = gcn.layer_forward(A.row_ptr, A.col_idx, A.val, A.n_cols, H, W, b, True)
    np.testing.assert_array_equal(Y[2], np.maximum(b, 0))


@pytest.mark.parametrize("relu", [False, True])
def test_product_epilogue_special_cases(relu):
    rng = np.random.default_rng(6)
    n, N = 8, 16
    cols = rng.permutation(n)
    scale = rng.uniform(-2, 2, size=n)
    A = from_coo(np.arange(n), cols, scale, n, n)         # one entry per row: a scaled row gather
    B = rng.normal(size=(n, N))
    b = rng.normal(size=N)
    a = A.val.astype(np.float64)
    Z, S = gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, n, B, b, relu)
    want = a[:, None] * B[A.col_idx] + b
    np.testing.assert_allclose(Z, np.maximum(want, 0) if relu else want, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(S, np.abs(a)[:, None] * np.abs(B[A.col_idx]) + np.abs(b), rtol=1e-14)
    Z0, S0 = gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, n, B, None, relu)
    want0 = a[:, None] * B[A.col_idx]
    np.testing.assert_allclose(Z0, np.maximum(want0, 0) if relu else want0, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(S0, np.abs(want0), rtol=1e-14)


def test_product_epilogue_matches_dense_product():
    A, H, _, _, _ = small_problem(7)
    b = np.linspace(-1, 1, H.shape[1])
    Z, S = gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, A.n_cols, H, b, True)
    D = dense_of(A)
    np.testing.assert_allclose(Z, np.maximum(D @ H + b, 0), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S, np.abs(D) @ np.abs(H) + np.abs(b), rtol=1e-13, atol=1e-13)
