"""Oracle of the GCN layer built on the sparse-dense product (paper, Section 4.4).

TEST INFRASTRUCTURE ONLY.  Plain numpy in fp64, no blocking, no fusion.

The layer equation of Section 4.4 is H' = sigma(A H W) with A sparse and sigma the
activation of a graph convolutional network (ReLU in hidden layers, the identity in
the last one); a bias b is added before sigma as in the usual formulation.  The
equation fixes no association: both (A H) W and A (H W) are written out below and
must agree in fp64 up to rounding.

Functions:
  product_epilogue   act(A B + b): the product the sparse kernels deliver when the
                     bias, the activation and the rounding of the output are applied
                     on the way out.  Also returns S = |A||B| + |b|, the scale of
                     the accumulation error bound.
  layer_forward      Z = A H W + b, Y = act(Z), both association orders.
  layer_backward     gradients of L = sum(Y * G) for a given G with respect to H, W
                     and b, derived by the chain rule: dZ = G * [Z > 0] (or G),
                     dW = (A H)^T dZ, dH = A^T (dZ W^T), db = column sums of dZ.

Pins (tests/test_oracle_gcn.py): central finite differences of L on tiny inputs (they
use layer_forward only, so a wrong transpose, mask or missing term in layer_backward
fails); A = I reduces the layer to act(H W + b) written densely; both association
orders agree; a one-entry-per-row A makes the product a scaled row gather.
"""
from __future__ import annotations

import numpy as np
import scipy.sparse as sp


def _csr64(row_ptr, col_idx, val, n_cols):
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    return sp.csr_matrix((np.asarray(val, dtype=np.float64), np.asarray(col_idx, dtype=np.int64), row_ptr),
                         shape=(row_ptr.size - 1, n_cols))


def product_epilogue(row_ptr, col_idx, val, n_cols, B, bias=None, relu=False):
    """Return (act(A B + bias), S) in fp64; S = |A||B| + |bias| elementwise."""
    A = _csr64(row_ptr, col_idx, val, n_cols)
    B = np.asarray(B, dtype=np.float64)
    Z = A @ B
    S = abs(A) @ np.abs(B)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        Z = Z + b[None, :]
        S = S + np.abs(b)[None, :]
    if relu:
        Z = np.maximum(Z, 0.0)
    return Z, S


def layer_forward(row_ptr, col_idx, val, n_cols, H, W, bias=None, relu=True, order="AH_W"):
    """Return (Y, Z): Z = A H W + bias in the given association order, Y = act(Z)."""
    A = _csr64(row_ptr, col_idx, val, n_cols)
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    if order == "AH_W":
        Z = (A @ H) @ W
    elif order == "A_HW":
        Z = A @ (H @ W)
    else:
        raise ValueError(order)
    if bias is not None:
        Z = Z + np.asarray(bias, dtype=np.float64)[None, :]
    Y = np.maximum(Z, 0.0) if relu else Z
    return Y, Z


def layer_backward(row_ptr, col_idx, val, n_cols, H, W, bias, relu, G):
    """Gradients of L = sum(Y * G): returns (dH, dW, db) in fp64."""
    A = _csr64(row_ptr, col_idx, val, n_cols)
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    _, Z = layer_forward(row_ptr, col_idx, val, n_cols, H, W, bias, relu)
    dZ = G * (Z > 0.0) if relu else G
    AH = A @ H
    dW = AH.T @ dZ
    dH = A.T @ (dZ @ W.T)
    db = dZ.sum(axis=0)
    return dH, dW, db
