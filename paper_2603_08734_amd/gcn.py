"""GCN layers H' = act(A H W + b) on the sparse kernels (paper, Section 4.4).

The sparse products -- A times a dense operand in the forward pass, A^T times a dense operand in
the backward pass -- run through ``rsh_spmm_f16``; the two small dense products per pass are plain
library GEMMs (``torch.matmul`` on binary16 operands, fp32 accumulation).  Two association orders:

  "A_HW": Y = act(A (H W) + b)   the GEMM shrinks the features first; bias, activation and the
                                 rounding to binary16 are fused into the sparse kernels
  "AH_W": Y = act((A H) W + b)   the order the paper's layer equation is written in; the sparse
                                 kernels deliver A H in binary16 for the GEMM

A plan is bound to the feature width of the sparse product's dense operand (d_out for "A_HW", d_in
for "AH_W"; forward and backward use the same width), so all layers of a network that share a
width share two plans: one of A, one of A^T (built on the first backward pass).  ``Adjacency``
holds the matrix and hands out the plans.  Without the HIP library every call fails: there is no
CPU path.
"""
from __future__ import annotations

import torch

from .binding import Plan


class Adjacency:
    """A fixed sparse A (CSR, binary16 values) and its plans by (feature width, transposed)."""

    def __init__(self, row_ptr, col_idx, val_f16, n_cols: int, symmetric: bool = False, **plan_opts):
        """symmetric=True (the caller vouches that A equals its transpose, values included, as the
        normalised adjacency of an undirected graph does): the backward pass reuses the plan of A."""
        self._csr = (row_ptr, col_idx, val_f16, int(n_cols))
        self._opts = dict(plan_opts)
        self._symmetric = bool(symmetric)
        self._plans: dict[tuple[int, bool], Plan] = {}

    def plan(self, width: int, transposed: bool = False) -> Plan:
        key = (int(width), bool(transposed) and not self._symmetric)
        if key not in self._plans:
            row_ptr, col_idx, val, n_cols = self._csr
            self._plans[key] = Plan(row_ptr, col_idx, val, n_cols, key[0], transpose=1 if transposed else 0, **self._opts)
        return self._plans[key]

    def destroy(self) -> None:
        for p in self._plans.values():
            p.destroy()
        self._plans.clear()


class _SparseProduct(torch.autograd.Function):
    """X (binary16, [n_cols, N]) -> binary16(act(A X + bias)); backward through A^T."""

    @staticmethod
    def forward(ctx, adj, X, bias, relu):
        X = X.contiguous()
        plan = adj.plan(X.shape[1])
        Y = torch.empty((plan.n_rows, plan.N), dtype=torch.float16, device=X.device)
        plan.spmm_f16(X, Y, bias, relu)
        ctx.adj, ctx.relu, ctx.has_bias = adj, relu, bias is not None
        ctx.save_for_backward(Y if relu else None)
        return Y

    @staticmethod
    def backward(ctx, dY):
        (Y,) = ctx.saved_tensors
        dZ = dY.to(torch.float16)
        if ctx.relu:
            dZ = dZ * (Y > 0)
        dZ = dZ.contiguous()
        plan_t = ctx.adj.plan(dZ.shape[1], transposed=True)
        dX = torch.empty((plan_t.n_rows, plan_t.N), dtype=torch.float16, device=dZ.device)
        plan_t.spmm_f16(dZ, dX, None, False)
        dbias = dZ.sum(dim=0, dtype=torch.float32) if ctx.has_bias else None
        return None, dX, dbias, None


class _DenseProduct(torch.autograd.Function):
    """H W with library GEMMs.  The weight gradient H^T dZ reduces over all rows of the graph into a
    d_in x d_out result; as one GEMM that is a single output tile (one workgroup streams the whole
    of H), so it is issued as a batched GEMM over row slabs whose partial results are then added."""

    @staticmethod
    def forward(ctx, H, W):
        ctx.save_for_backward(H, W)
        return H @ W

    @staticmethod
    def backward(ctx, dZ):
        H, W = ctx.saved_tensors
        dH = dZ @ W.t() if ctx.needs_input_grad[0] else None
        dW = None
        if ctx.needs_input_grad[1]:
            n = H.shape[0]
            slabs = 256      # the largest power of two that divides n and leaves slabs of 64 rows or more
            while slabs > 1 and (n % slabs or n // slabs < 64):
                slabs //= 2
            if slabs > 1:
                part = torch.bmm(H.view(slabs, n // slabs, -1).transpose(1, 2), dZ.reshape(slabs, n // slabs, -1))
                dW = part.sum(dim=0, dtype=torch.float32).to(W.dtype)
            else:
                dW = H.t() @ dZ
        return dH, dW


class GCNLayer:
    """One layer on an ``Adjacency``; layers of equal width share its plans."""

    def __init__(self, adjacency, d_in: int, d_out: int, order: str | None = None):
        if order is None:
            order = "A_HW" if d_out <= d_in else "AH_W"
        if order not in ("A_HW", "AH_W"):
            raise ValueError(order)
        self.adj, self.order, self.d_in, self.d_out = adjacency, order, int(d_in), int(d_out)
        self.width = self.d_out if order == "A_HW" else self.d_in
        self.adj.plan(self.width)          # plan now, not inside the first forward pass

    def __call__(self, H, W, bias=None, relu: bool = True):
        """H: binary16 [n_cols, d_in]; W: binary16 [d_in, d_out]; bias: fp32 [d_out] or None."""
        assert H.dtype == torch.float16 and W.dtype == torch.float16 and tuple(W.shape) == (self.d_in, self.d_out)
        if self.order == "A_HW":
            return _SparseProduct.apply(self.adj, _DenseProduct.apply(H, W), bias, relu)
        M = _SparseProduct.apply(self.adj, H, None, False)
        Z = _DenseProduct.apply(M, W)
        if bias is not None:
            Z = Z.float() + bias
        return (torch.relu(Z) if relu else Z).to(torch.float16)
