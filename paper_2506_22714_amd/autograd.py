"""Differentiable SpMM / SDDMM / edge softmax on top of the C ABI (training use of the operators, Section 5.5 of the
paper).  Only argument marshalling and the chain rule live here; every product runs in the library's kernels:

  C = A B            dB = A^T dC                 (SpMM on the plan of the transposed pattern)
                     dA_p = <dC_i, B_j>          (SDDMM without A's values)
  out_p = A_p <X_i, Y_j>
                     dX = (A o dout) Y,  dY = (A o dout)^T X,  dA_p = dout_p <X_i, Y_j>
  alpha = softmax_row(scale * s)
                     ds_p = scale alpha_p (dalpha_p - sum_row alpha dalpha)
"""
from __future__ import annotations

import torch

from . import binding as lb


class SparseMatrix:
    """A sparse pattern on the device with the plan of A and of A^T (both built by the device planner).  Values are
    passed to every call (they are what training changes); the plans only hold the current ones."""

    def __init__(self, M: int, Kc: int, rowptr: torch.Tensor, col: torch.Tensor, dtype=torch.float16, **opts):
        self.M, self.Kc, self.dtype = int(M), int(Kc), dtype
        self.rowptr, self.col = rowptr, col
        self.nnz = int(col.numel())
        ones = torch.ones(self.nnz, dtype=dtype, device=col.device)
        self.plan = lb.Plan.from_device_csr(M, Kc, rowptr, col, ones, resident=True, keep_host_copy=False, **opts)
        rowptr_t, col_t, perm_t = lb.transpose_csr(M, Kc, rowptr, col)
        self.perm_t = perm_t.long()
        self.plan_t = lb.Plan.from_device_csr(Kc, M, rowptr_t, col_t, ones, resident=True, keep_host_copy=False, **opts)

    def close(self):
        self.plan.close()
        self.plan_t.close()


def _feature_ok(n: int) -> bool:
    return n in (32, 64, 128)


class _SpMM(torch.autograd.Function):
    @staticmethod
    def forward(ctx, sm: SparseMatrix, vals: torch.Tensor, B: torch.Tensor):
        sm.plan.set_values(vals.detach().contiguous(), lb.OP_SPMM)
        ctx.sm = sm
        ctx.save_for_backward(vals, B)
        return sm.plan.spmm(B.detach().contiguous())

    @staticmethod
    def backward(ctx, dC):
        sm = ctx.sm
        vals, B = ctx.saved_tensors
        dC16 = dC.to(sm.dtype).contiguous()
        dvals = dB = None
        if ctx.needs_input_grad[2]:
            sm.plan_t.set_values(vals.detach()[sm.perm_t].contiguous(), lb.OP_SPMM)
            dB = sm.plan_t.spmm(dC16).to(B.dtype)
        if ctx.needs_input_grad[1]:
            if not _feature_ok(B.shape[1]):
                raise RuntimeError("gradient with respect to the sparse values needs N in {32, 64, 128}")
            dvals = sm.plan.sddmm(dC16, B.detach().contiguous(), pattern_only=True).to(vals.dtype)
        return None, dvals, dB


class _SDDMM(torch.autograd.Function):
    @staticmethod
    def forward(ctx, sm: SparseMatrix, vals: torch.Tensor, X: torch.Tensor, Y: torch.Tensor):
        sm.plan.set_values(vals.detach().contiguous(), lb.OP_SDDMM)
        ctx.sm = sm
        ctx.save_for_backward(vals, X, Y)
        return sm.plan.sddmm(X.detach().contiguous(), Y.detach().contiguous())

    @staticmethod
    def backward(ctx, dout):
        sm = ctx.sm
        vals, X, Y = ctx.saved_tensors
        Xc, Yc = X.detach().contiguous(), Y.detach().contiguous()
        g = (dout * vals.detach().float()).to(sm.dtype).contiguous()
        dvals = dX = dY = None
        if ctx.needs_input_grad[2]:
            sm.plan.set_values(g, lb.OP_SPMM)
            dX = sm.plan.spmm(Yc).to(X.dtype)
        if ctx.needs_input_grad[3]:
            sm.plan_t.set_values(g[sm.perm_t].contiguous(), lb.OP_SPMM)
            dY = sm.plan_t.spmm(Xc).to(Y.dtype)
        if ctx.needs_input_grad[1]:
            dvals = (dout * sm.plan.sddmm(Xc, Yc, pattern_only=True)).to(vals.dtype)
        return None, dvals, dX, dY


class _EdgeSoftmax(torch.autograd.Function):
    @staticmethod
    def forward(ctx, sm: SparseMatrix, scores: torch.Tensor, scale: float):
        alpha = sm.plan.edge_softmax(scores.detach().float().contiguous(), scale,
                                     out=torch.empty(sm.nnz, dtype=sm.dtype, device=scores.device))
        ctx.sm, ctx.scale = sm, scale
        ctx.save_for_backward(alpha)
        return alpha

    @staticmethod
    def backward(ctx, dalpha):
        (alpha,) = ctx.saved_tensors
        return None, ctx.sm.plan.edge_softmax_backward(alpha, dalpha.float().contiguous(), ctx.scale), None


def spmm(sm: SparseMatrix, vals: torch.Tensor, B: torch.Tensor) -> torch.Tensor:
    """C = A B with A's values `vals` (CSR order); fp32 result."""
    return _SpMM.apply(sm, vals, B)


def sddmm(sm: SparseMatrix, vals: torch.Tensor, X: torch.Tensor, Y: torch.Tensor) -> torch.Tensor:
    """out_p = vals_p <X_i, Y_j> on A's pattern (CSR order); fp32 result."""
    return _SDDMM.apply(sm, vals, X, Y)


def edge_softmax(sm: SparseMatrix, scores: torch.Tensor, scale: float = 1.0) -> torch.Tensor:
    """Row-wise softmax of `scale * scores` over A's pattern; result in the matrix's value type."""
    return _EdgeSoftmax.apply(sm, scores, scale)
