"""The plain-torch fp64 checks (drot_checks.py) against the oracle's evaluation of the same quantities,
and against values worked out by hand: two routes written separately must agree on every term."""
import numpy as np
import pytest
import torch

import drot_checks
import drot_inputs


@pytest.mark.parametrize("kind,lam,mu", [(0, 0.0, 0.0), (1, 0.3, 0.0), (2, 0.2, 0.07), (2, 0.0, 0.05)])
def test_terms_agree_with_the_oracle(oracle, kind, lam, mu):
    P = drot_inputs.random_problem(37, 53, seed=4100 + kind, reg_kind=kind, lam=lam, mu=mu, num_classes=4,
                                   sorted_classes=False)
    rng = np.random.default_rng(4200)
    # an arbitrary nonnegative sparse X and arbitrary dual vectors: the formulas, not a solution
    X = (np.outer(P.p, P.q) * rng.uniform(0.0, 3.0, size=(P.m, P.n)) * (rng.uniform(size=(P.m, P.n)) < 0.3)).astype(np.float32)
    rho = float(P.rho)
    phi = (rho * rng.uniform(0.0, 0.8, size=P.m)).astype(np.float32)
    varphi = (rho * rng.uniform(0.0, 0.8, size=P.n)).astype(np.float32)
    lam32, mu32 = float(np.float32(lam)), float(np.float32(mu))
    o = oracle.objective_gap(P.C, X, P.p, P.q, phi, varphi, rho, reg_kind=kind, lam=lam32, mu=mu32,
                             row_class=P.row_class, num_classes=P.num_classes)
    rc = None if P.row_class is None else torch.from_numpy(P.row_class)
    t = drot_checks.fp64_terms(torch.from_numpy(P.C), torch.from_numpy(X), torch.from_numpy(P.p), torch.from_numpy(P.q),
                               torch.from_numpy(phi), torch.from_numpy(varphi), rho, reg_kind=kind, lam=lam32, mu=mu32,
                               row_class=rc, num_classes=P.num_classes, block_rows=16)
    for a, b in ((t.cost, o.cost), (t.h, o.h), (t.dual_linear, o.dual_linear), (t.h_conj, o.h_conj), (t.gap, o.gap),
                 (t.dual_res, o.dual_res)):
        assert abs(a - b) <= 1e-12 * max(1.0, abs(b)), (a, b)
    X64 = X.astype(np.float64)
    assert abs(t.r_row - np.linalg.norm(X64.sum(1) - P.p)) <= 1e-15
    assert abs(t.r_col - np.linalg.norm(X64.sum(0) - P.q)) <= 1e-15
    assert t.nnz == int(np.count_nonzero(X)) and t.min_entry == 0.0


def test_terms_by_hand_on_a_two_by_two_problem():
    # C = [[0, 1], [1, 0]], X = diag(1/2, 1/2), u = v = (1/4, 1/4) => W = [u_i + v_j - C_ij]_+ = [[1/2, 0], [0, 1/2]]
    C = torch.tensor([[0.0, 1.0], [1.0, 0.0]])
    X = torch.tensor([[0.5, 0.0], [0.0, 0.5]])
    p = q = torch.tensor([0.5, 0.5])
    rho = 0.5
    phi = varphi = torch.tensor([0.125, 0.125])  # u = v = 1/4
    t = drot_checks.fp64_terms(C, X, p, q, phi, varphi, rho, reg_kind=1, lam=2.0)
    assert t.cost == 0.0 and t.h == pytest.approx(0.5 * 2.0 * 0.5)      # (lambda/2) * (1/4 + 1/4)
    assert t.dual_linear == pytest.approx(0.5)                           # 4 * (1/2 * 1/4)
    assert t.h_conj == pytest.approx(0.5 / 4.0)                          # ||W||^2 / (2 lambda) = (1/2) / 4
    assert t.gap == pytest.approx(0.5 - 0.5 + 0.125)
    assert t.r_row == 0.0 and t.r_col == 0.0 and t.dual_res == 0.0
    t0 = drot_checks.fp64_terms(C, X, p, q, phi, varphi, rho, reg_kind=0)
    assert t0.dual_res == pytest.approx(0.5 ** 0.5) and t0.h == 0.0 and t0.h_conj == 0.0
    # group lasso, both rows in one class: groups are the two columns, ||X_g|| = 1/2 each, ||W_g|| = 1/2 each
    rc = torch.tensor([0, 0], dtype=torch.int32)
    tg = drot_checks.fp64_terms(C, X, p, q, phi, varphi, rho, reg_kind=2, lam=2.0, mu=0.25, row_class=rc, num_classes=1)
    assert tg.h == pytest.approx(0.25 * 1.0 + 0.5)
    assert tg.h_conj == pytest.approx(2 * (0.25 ** 2) / 4.0)


def test_fixed_point_defect_vanishes_at_the_oracles_fixed_point(oracle):
    P = drot_inputs.random_problem(12, 15, seed=4300, reg_kind=1, lam=5.0)
    lam = float(np.float32(P.lam))
    r = oracle.solve(P.C, P.p, P.q, rho=float(P.rho), reg_kind=1, lam=lam, max_iters=200000, tol=1e-13, check_every=10)
    d = drot_checks.fixed_point_defect(torch.from_numpy(P.C), torch.from_numpy(r.X), torch.from_numpy(r.phi),
                                       torch.from_numpy(r.varphi), float(P.rho), lam)
    assert d <= 1e-12 * float(P.rho)
    # and one iterate earlier it is bounded by (1 + rho*lambda) times the step to the next iterate
    a = oracle.solve(P.C, P.p, P.q, rho=float(P.rho), reg_kind=1, lam=lam, max_iters=40)
    b = oracle.solve(P.C, P.p, P.q, rho=float(P.rho), reg_kind=1, lam=lam, max_iters=41)
    d = drot_checks.fixed_point_defect(torch.from_numpy(P.C), torch.from_numpy(a.X), torch.from_numpy(a.phi),
                                       torch.from_numpy(a.varphi), float(P.rho), lam)
    assert d <= (1.0 + float(P.rho) * lam) * np.abs(a.X - b.X).max() + 1e-15
