"""Shared helpers of the GPU parity tests: run both sides on the same fp32 inputs and compare.

Tolerances (the bar the benchmark definition states, fp32 arithmetic on the GPU, fp64 oracle):
  * plan:       max_ij |X_gpu - X_oracle| <= 1e-4 * max_ij |X_oracle|
                (the elementwise error is normalised by the plan's scale: entries are produced by
                cancelling terms of size rho*C, so fp32 cannot hold a relative error on the tiniest ones)
  * objective:  |obj_gpu - obj_oracle| <= 1e-5 * |obj_oracle|, both evaluated in fp64 from the plans
  * residuals:  | ||X1-p|| - ||X1-p||_oracle | <= 1e-6, same for the column residual
  * support:    entries positive on one side and zero on the other are below 5e-5 of the plan's scale and few
  * large entries (>= 1e-2 * max): per-entry relative error <= 8e-3
"""
from __future__ import annotations

import numpy as np
import torch

PLAN_TOL = 1e-4
OBJ_TOL = 1e-5
RES_TOL = 1e-6
# support mismatches (an entry > 0 on one side, == 0 on the other): how large such an entry may be
# relative to the largest entry of the plan (it is at most the plan error at that entry; the bar is half
# of PLAN_TOL; measured: none on the five configurations, single entries of up to 1.2e-5 elsewhere), and
# how many there may be
SUPPORT_TOL = 5e-5
SUPPORT_COUNT_FRAC = 2e-2
SUPPORT_COUNT_MIN = 8
# per-entry relative error on the entries >= BIG_ENTRY * max: there an absolute error of PLAN_TOL * max is
# a relative one of at most PLAN_TOL / BIG_ENTRY = 1e-2; the bar asked of those entries is a little tighter
# (measured: 1e-5 .. 1e-3 after the configurations' fixed iteration counts, 4.8e-3 after the 20800 iterations
# of the second configuration's run to 1e-5, on entries right at the threshold)
BIG_ENTRY = 1e-2
REL_TOL_BIG = 8e-3
LAST_STATS = {}  # what the last assert_parity measured beyond its return value (for the test logs)


def to_dev(P):
    dev = torch.device("cuda:0")
    C = torch.from_numpy(P.C).to(dev)
    if P.forbidden is not None:  # the library's convention for constrained OT: +inf cost on the forbidden pairs
        C = torch.where(torch.from_numpy(P.forbidden).to(dev), torch.full_like(C, float("inf")), C)
    p = torch.from_numpy(P.p).to(dev)
    q = torch.from_numpy(P.q).to(dev)
    rc = None if P.row_class is None else torch.from_numpy(P.row_class).to(dev)
    return C, p, q, rc


def gpu_solve(solver, P, max_iters, tol=0.0, stepsize=0.0, stream=None, X_out=None):
    C, p, q, rc = to_dev(P)
    W = None if P.weights is None else torch.from_numpy(P.weights).to(C.device)
    res = solver.solve(C, p, q, stepsize=stepsize, reg_kind=P.reg_kind, lam=P.lam, mu=P.mu, row_class=rc,
                       num_classes=P.num_classes, max_iters=max_iters, tol=tol, stream=stream, X_out=X_out, weights=W)
    phi, varphi = solver.duals(P.m, P.n, C.device)
    torch.cuda.synchronize()
    return res, res.X.cpu().numpy(), phi.cpu().numpy(), varphi.cpu().numpy()


def oracle_solve(oracle, P, max_iters, tol=0.0, check_every=1, stepsize=None):
    rho = float(P.rho) if stepsize is None else float(np.float32(stepsize))
    return oracle.solve(P.C, P.p, P.q, rho=rho, reg_kind=P.reg_kind, lam=float(np.float32(P.lam)),
                        mu=float(np.float32(P.mu)), row_class=P.row_class, num_classes=P.num_classes,
                        max_iters=max_iters, tol=tol, check_every=check_every, weights=P.weights,
                        forbidden=P.forbidden)


def fp64_terms(oracle, P, X, phi, varphi, stepsize=None):
    rho = float(P.rho) if stepsize is None else float(np.float32(stepsize))
    return oracle.objective_gap(P.C, X, P.p, P.q, phi, varphi, rho, reg_kind=P.reg_kind,
                                lam=float(np.float32(P.lam)), mu=float(np.float32(P.mu)), row_class=P.row_class,
                                num_classes=P.num_classes, weights=P.weights, forbidden=P.forbidden)


def residuals(P, X):
    X = np.asarray(X, dtype=np.float64)
    r = X.sum(1) - P.p.astype(np.float64)
    s = X.sum(0) - P.q.astype(np.float64)
    return float(np.linalg.norm(r)), float(np.linalg.norm(s))


def assert_parity(oracle, P, gres, Xg, phig, varphig, ores, stepsize=None, check_gap=True, label=""):
    """Element-by-element comparison of the GPU iterate with the oracle's, to the stated bar."""
    Xo = ores.X
    assert Xg.shape == Xo.shape
    assert np.isfinite(Xg).all(), label
    assert (Xg >= 0).all(), label
    scale = np.abs(Xo).max()
    diff = np.abs(Xg.astype(np.float64) - Xo)
    err = diff.max()
    assert err <= PLAN_TOL * scale, f"{label}: plan error {err:.3e} vs scale {scale:.3e} (ratio {err / scale:.2e})"
    # support: entries that are positive on one side and exactly zero on the other.  fp32 produces an
    # entry as the clamp of a sum of terms of size rho*|C|, |phi|, |varphi|, so one that the fp64
    # iteration leaves within the rounding of those terms of zero may land on the other side of the
    # clamp; such entries must be that small (far below the plan's tolerance) and few
    sg, so = Xg > 0, Xo > 0
    mism = sg != so
    nmism = int(np.count_nonzero(mism))
    nnz = max(int(np.count_nonzero(so)), 1)
    mism_mag = float(np.maximum(Xg[mism].max(initial=0.0), Xo[mism].max(initial=0.0)))
    assert mism_mag <= SUPPORT_TOL * scale, f"{label}: {nmism} support mismatches, largest entry {mism_mag:.3e} vs scale {scale:.3e}"
    assert nmism <= max(SUPPORT_COUNT_MIN, SUPPORT_COUNT_FRAC * nnz), f"{label}: {nmism} support mismatches of {nnz} nonzeros"
    # relative error where it means something: on the entries that are at least a hundredth of the largest
    big = Xo >= BIG_ENTRY * scale
    rel_big = float((diff[big] / Xo[big]).max()) if big.any() else 0.0
    assert rel_big <= REL_TOL_BIG, f"{label}: relative error {rel_big:.3e} on entries >= {BIG_ENTRY:g} * max"
    LAST_STATS.update(support_mismatches=nmism, nonzeros=nnz, largest_mismatched_entry=mism_mag / scale,
                      rel_err_big_entries=rel_big, frob=float(np.sqrt((diff * diff).sum()) / np.sqrt((Xo * Xo).sum())))
    # dual vectors: same normalisation (they are O(rho) like the plan's increments)
    pscale = max(np.abs(ores.phi).max(), np.abs(ores.varphi).max())
    perr = max(np.abs(phig - ores.phi).max(), np.abs(varphig - ores.varphi).max())
    assert perr <= PLAN_TOL * pscale, f"{label}: dual vector error {perr:.3e} vs {pscale:.3e}"
    # objective in fp64 from each plan
    tg = fp64_terms(oracle, P, Xg, phig, varphig, stepsize)
    to = fp64_terms(oracle, P, Xo, ores.phi, ores.varphi, stepsize)
    assert abs(tg.objective - to.objective) <= OBJ_TOL * abs(to.objective), \
        f"{label}: objective {tg.objective} vs {to.objective}"
    # marginal residuals in fp64 from each plan, and the ones the library reports
    rg, sg = residuals(P, Xg)
    ro, so = residuals(P, Xo)
    assert abs(rg - ro) <= RES_TOL and abs(sg - so) <= RES_TOL, f"{label}: residuals {rg},{sg} vs {ro},{so}"
    assert abs(gres.r_row - ro) <= RES_TOL and abs(gres.r_col - so) <= RES_TOL, \
        f"{label}: reported residuals {gres.r_row},{gres.r_col} vs {ro},{so}"
    if check_gap:
        # the library's own objective / gap / dual residual vs the fp64 evaluation at its iterate
        assert abs(gres.objective - tg.objective) <= OBJ_TOL * abs(tg.objective) + 1e-12, \
            f"{label}: reported objective {gres.objective} vs {tg.objective}"
        gap_scale = max(abs(tg.cost), abs(tg.dual_linear), abs(tg.h_conj), 1e-30)
        assert abs(gres.gap - tg.gap) <= 2e-5 * gap_scale, f"{label}: reported gap {gres.gap} vs {tg.gap}"
        assert abs(gres.dual_res - tg.dual_res) <= 2e-5 * max(tg.dual_res, gap_scale), \
            f"{label}: reported dual residual {gres.dual_res} vs {tg.dual_res}"
    return err / scale
