"""Differentiable OT cost: OT_h(C) = min_X <C,X> + h(X) over the transport polytope.

Section "Backpropagation through regularized OT-costs": a solution X* of problem (1) is a
subgradient of OT_h with respect to C, and the gradient when the solution is unique (for instance
with the quadratic term).  The forward pass is one solve of the HIP library; the backward pass
hands the plan it returned to autograd, scaled by the incoming gradient.  No solver arithmetic
lives here.
"""
from __future__ import annotations

import torch

from .binding import Solver


class _OTCost(torch.autograd.Function):
    @staticmethod
    def forward(ctx, C, solver, p, q, solve_kwargs):
        res = solver.solve(C.detach(), p, q, **solve_kwargs)
        ctx.save_for_backward(res.X)
        ctx.result = res
        return torch.tensor(res.objective, dtype=torch.float64, device=C.device)

    @staticmethod
    def backward(ctx, grad_out):
        (X,) = ctx.saved_tensors
        return (grad_out.to(X.dtype) * X), None, None, None, None


def ot_cost(solver: Solver, C: torch.Tensor, p: torch.Tensor, q: torch.Tensor, **solve_kwargs) -> torch.Tensor:
    """OT_h(C) as a float64 scalar tensor whose gradient with respect to C is the transport plan.

    solve_kwargs go to Solver.solve (reg_kind, lam, mu, row_class, num_classes, max_iters, tol, ...).
    The solver must have been created with compute_gap on (the default): the value is the
    objective the library evaluates at the returned plan.  The plan is as accurate as the solve:
    pass a tolerance and an iteration budget that fit the use.
    """
    return _OTCost.apply(C, solver, p, q, solve_kwargs)
