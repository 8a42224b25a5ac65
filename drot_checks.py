"""fp64 checks of a returned triple (X, phi, varphi) in plain PyTorch -- test and benchmark infrastructure.

Independent of both solvers: this module imports neither the HIP binding nor the CPU oracle and
shares no code with them.  It evaluates, from the definitions, what any candidate solution of

    min <C,X> + h(X)   s.t.  X 1_n = p,  X^T 1_m = q,  X >= 0                    (problem (1))

can be judged by at any size: nonnegativity, the two marginal residual norms of the stopping
criterion (Appendix C), the objective, and the duality gap of Appendix C with u = phi/rho,
v = varphi/rho, W = [u 1^T + 1 v^T - C]_+:

    gap = <C,X> + h(X) - (p^T u + q^T v) + h*(W),

with the closed-form conjugates h*(W) = ||W||_F^2/(2 lambda) (quadratic) and
sum_g max(||W_g||_2 - mu, 0)^2/(2 lambda) (group lasso plus quadratic); where h* is an indicator
(h = 0, or group lasso with lambda = 0) its violation is returned as the dual residual instead.
The matrices are walked in row blocks, widened to fp64 block by block, on whatever device they
live on.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch


@dataclass
class Fp64Terms:
    min_entry: float      # min_ij X_ij
    r_row: float          # ||X 1 - p||_2
    r_col: float          # ||X^T 1 - q||_2
    cost: float           # <C, X>
    h: float              # h(X)
    dual_linear: float    # p^T u + q^T v
    h_conj: float         # h*(W) where finite, else 0
    dual_res: float       # violation of the dual constraint where h* is an indicator, else 0
    nnz: int              # entries of X that are not zero

    @property
    def objective(self) -> float:
        return self.cost + self.h

    @property
    def gap(self) -> float:
        return self.cost + self.h - self.dual_linear + self.h_conj


def fp64_terms(C: torch.Tensor, X: torch.Tensor, p: torch.Tensor, q: torch.Tensor, phi: torch.Tensor,
               varphi: torch.Tensor, rho: float, reg_kind: int = 0, lam: float = 0.0, mu: float = 0.0,
               row_class: Optional[torch.Tensor] = None, num_classes: int = 0, block_rows: int = 2048) -> Fp64Terms:
    """All of the above for one (X, phi, varphi); reg_kind 0 none, 1 quadratic, 2 group lasso (+ quadratic)."""
    m, n = X.shape
    dev = X.device
    f64 = torch.float64
    u = phi.to(f64) / rho
    v = varphi.to(f64) / rho
    col = torch.zeros(n, dtype=f64, device=dev)
    rows = torch.empty(m, dtype=f64, device=dev)
    cost = xx = ww = 0.0
    nnz = 0
    min_entry = float("inf")
    gx = gw = None
    if reg_kind == 2:
        gx = torch.zeros((num_classes, n), dtype=f64, device=dev)
        gw = torch.zeros((num_classes, n), dtype=f64, device=dev)
    for i0 in range(0, m, block_rows):
        i1 = min(i0 + block_rows, m)
        Xb = X[i0:i1].to(f64)
        Cb = C[i0:i1].to(f64)
        Wb = (u[i0:i1, None] + v[None, :] - Cb).clamp_(min=0.0)
        rows[i0:i1] = Xb.sum(dim=1)
        col += Xb.sum(dim=0)
        # (pairs with an infinite cost carry no mass: they add nothing to <C,X>)
        cost += float(torch.where(Xb > 0, Cb * Xb, torch.zeros_like(Xb)).sum())
        xx += float((Xb * Xb).sum())
        ww += float((Wb * Wb).sum())
        nnz += int((Xb != 0).sum())
        min_entry = min(min_entry, float(Xb.min()))
        if reg_kind == 2:
            cls = row_class[i0:i1].long()
            gx.index_add_(0, cls, Xb * Xb)
            gw.index_add_(0, cls, Wb * Wb)
    r_row = float((rows - p.to(f64)).norm())
    r_col = float((col - q.to(f64)).norm())
    dual_linear = float((p.to(f64) * u).sum() + (q.to(f64) * v).sum())
    h = h_conj = dual_res = 0.0
    if reg_kind == 0 or (reg_kind == 1 and lam <= 0.0):
        dual_res = ww ** 0.5
    elif reg_kind == 1:
        h = 0.5 * lam * xx
        h_conj = ww / (2.0 * lam)
    else:
        excess = (gw.sqrt() - mu).clamp_(min=0.0)
        e2 = float((excess * excess).sum())
        h = mu * float(gx.sqrt().sum()) + 0.5 * lam * xx
        if lam > 0.0:
            h_conj = e2 / (2.0 * lam)
        else:
            dual_res = e2 ** 0.5
    return Fp64Terms(min_entry=min_entry, r_row=r_row, r_col=r_col, cost=cost, h=h, dual_linear=dual_linear,
                     h_conj=h_conj, dual_res=dual_res, nnz=nnz)


def fixed_point_defect(C: torch.Tensor, X: torch.Tensor, phi: torch.Tensor, varphi: torch.Tensor, rho: float,
                       lam: float, block_rows: int = 2048) -> float:
    """max_ij | rho*lam*X_ij - [phi_i + varphi_j - rho*C_ij]_+ | in fp64 (quadratic regularizer).

    At a fixed point of X <- [X + phi 1^T + 1 varphi^T - rho C]_+ / (1 + rho*lam) the expression
    vanishes; it is the optimality condition X = [u (+) v - C]_+ / lam multiplied through by
    rho*lam, so no small number is divided by.
    """
    m, _ = X.shape
    f64 = torch.float64
    worst = 0.0
    for i0 in range(0, m, block_rows):
        i1 = min(i0 + block_rows, m)
        T = (phi[i0:i1, None].to(f64) + varphi[None, :].to(f64) - rho * C[i0:i1].to(f64)).clamp_(min=0.0)
        worst = max(worst, float((rho * lam * X[i0:i1].to(f64) - T).abs().max()))
    return worst
