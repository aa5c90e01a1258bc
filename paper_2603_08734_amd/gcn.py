"""One GCN layer H' = act(A H W + b) on the sparse kernels (paper, Section 4.4).

The sparse products -- A times a dense operand in the forward pass, A^T times a dense operand in
the backward pass -- run through ``rsh_spmm_f16``; the two small dense products per pass are plain
library GEMMs (``torch.matmul`` on binary16 operands, fp32 accumulation).  Two association orders:

  "A_HW": Y = act(A (H W) + b)   the GEMM shrinks the features first; bias, activation and the
                                 rounding to binary16 are fused into the sparse kernels
  "AH_W": Y = act((A H) W + b)   the order the paper's layer equation is written in; the sparse
                                 kernels deliver A H in binary16 for the GEMM

Plans are bound to the feature width of the sparse product's dense operand: d_out for "A_HW",
d_in for "AH_W" (forward and backward use the same width).  The plan of A^T is built on the first
backward pass.  Without the HIP library every call fails: there is no CPU path.
"""
from __future__ import annotations

import torch

from .binding import Plan


class _SparseProduct(torch.autograd.Function):
    """X (binary16, [n_cols, N]) -> binary16(act(A X + bias)); backward through A^T."""

    @staticmethod
    def forward(ctx, layer, X, bias, relu):
        X = X.contiguous()
        Y = torch.empty((layer.fwd.n_rows, layer.fwd.N), dtype=torch.float16, device=X.device)
        layer.fwd.spmm_f16(X, Y, bias, relu)
        ctx.layer, ctx.relu, ctx.has_bias = layer, relu, bias is not None
        ctx.save_for_backward(Y if relu else None)
        return Y

    @staticmethod
    def backward(ctx, dY):
        (Y,) = ctx.saved_tensors
        dZ = dY.to(torch.float16)
        if ctx.relu:
            dZ = dZ * (Y > 0)
        dZ = dZ.contiguous()
        plan_t = ctx.layer.transposed_plan()
        dX = torch.empty((plan_t.n_rows, plan_t.N), dtype=torch.float16, device=dZ.device)
        plan_t.spmm_f16(dZ, dX, None, False)
        dbias = dZ.sum(dim=0, dtype=torch.float32) if ctx.has_bias else None
        return None, dX, dbias, None


class GCNLayer:
    """A fixed sparse A (CSR, binary16 values) and the two plans its layer needs."""

    def __init__(self, row_ptr, col_idx, val_f16, n_cols: int, d_in: int, d_out: int, order: str | None = None,
                 **plan_opts):
        if order is None:
            order = "A_HW" if d_out <= d_in else "AH_W"
        if order not in ("A_HW", "AH_W"):
            raise ValueError(order)
        self.order, self.d_in, self.d_out = order, int(d_in), int(d_out)
        self._csr = (row_ptr, col_idx, val_f16, int(n_cols))
        self._opts = dict(plan_opts)
        self.width = self.d_out if order == "A_HW" else self.d_in
        self.fwd = Plan(row_ptr, col_idx, val_f16, n_cols, self.width, **plan_opts)
        self._bwd = None

    def transposed_plan(self) -> Plan:
        if self._bwd is None:
            row_ptr, col_idx, val, n_cols = self._csr
            self._bwd = Plan(row_ptr, col_idx, val, n_cols, self.width, transpose=1, **self._opts)
        return self._bwd

    def __call__(self, H, W, bias=None, relu: bool = True):
        """H: binary16 [n_cols, d_in]; W: binary16 [d_in, d_out]; bias: fp32 [d_out] or None."""
        assert H.dtype == torch.float16 and W.dtype == torch.float16 and tuple(W.shape) == (self.d_in, self.d_out)
        if self.order == "A_HW":
            return _SparseProduct.apply(self, H @ W, bias, relu)
        M = _SparseProduct.apply(self, H, None, False)
        Z = M @ W
        if bias is not None:
            Z = Z.float() + bias
        return (torch.relu(Z) if relu else Z).to(torch.float16)

    def destroy(self) -> None:
        self.fwd.destroy()
        if self._bwd is not None:
            self._bwd.destroy()
            self._bwd = None
