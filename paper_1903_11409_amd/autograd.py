"""Autograd glue: the batched product as a differentiable PyTorch operation.

Argument marshalling only: the forward pass is one ``bspmm_run`` launch, the backward pass one
``bspmm_run_transposed`` launch on the same plan (the gradient with respect to the dense
operand, ``dB_i = A_i^T dY_i``; the adjacency values are constants of the layer, as in the
paper's graph-convolution layer, Sec. II-A / Sec. IV-D).
"""
import torch

from . import bspmm as K


class BatchedSpMM(torch.autograd.Function):
    """``C = BatchedSpMM.apply(plan, B)`` with ``plan`` a :class:`bspmm.Plan`; ``B`` is the packed
    dense input (``n_b_rows x F`` fp32 on the plan's device), ``C`` the packed output."""

    @staticmethod
    def forward(ctx, plan, B, n_c_rows=None):
        if B.dtype != torch.float32 or not B.is_cuda:
            raise TypeError("BatchedSpMM needs an fp32 CUDA tensor")
        B = B.contiguous()
        rows = int(n_c_rows) if n_c_rows is not None else int(B.shape[0])
        C = torch.zeros((rows, plan.F), dtype=torch.float32, device=B.device)
        plan.run(B, C)
        ctx.plan = plan
        ctx.n_b_rows = int(B.shape[0])
        return C

    @staticmethod
    def backward(ctx, dY):
        dY = dY.contiguous()
        G = torch.zeros((ctx.n_b_rows, ctx.plan.F), dtype=torch.float32, device=dY.device)
        ctx.plan.run_transposed(dY, G)
        return None, G, None


def batched_spmm(plan: K.Plan, B, n_c_rows=None):
    """Functional form of :class:`BatchedSpMM`.  Rows of the output that belong to no operation
    are zero (``n_c_rows`` defaults to the number of rows of ``B``)."""
    return BatchedSpMM.apply(plan, B, n_c_rows)
