"""Pins of the CPU oracle against things other than itself (no GPU needed).

Every check here compares the oracle with something the paper or the mathematics fixes:
dense least squares, brute force over permutations, an LP solver, the smooth dual solved by
L-BFGS, numerical minimisation of the prox objective and of the conjugate's supremum, the
O(m+n) vector recursion the paper prints as eq. (6), and the closed-form early iterates of
Appendix B.  A plausible slip in the oracle (a sign, a 1/m vs 1/n, a dropped rho, a transposed
operand) fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.optimize as sopt

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_problem(m, n, seed, uniform=False):
    rng = np.random.default_rng(seed)
    C = rng.uniform(0.0, 1.0, size=(m, n)).astype(np.float32)
    C /= C.max()
    if uniform:
        p, q = np.full(m, 1.0 / m), np.full(n, 1.0 / n)
    else:
        p = rng.uniform(0.5, 1.5, m)
        q = rng.uniform(0.5, 1.5, n)
        p, q = p / p.sum(), q / q.sum()
    return C, p, q


# ---------------------------------------------------------------------------------------------
# projection onto the marginal constraints (Section 2.1, the closed form of eq. (5))
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("m,n", [(3, 5), (4, 4), (7, 2), (1, 6), (5, 1)])
def test_projection_equals_dense_least_squares(oracle, m, n):
    rng = np.random.default_rng(10 * m + n)
    V = rng.normal(size=(m, n))
    p = rng.uniform(0.5, 1.5, m)
    q = rng.uniform(0.5, 1.5, n)
    p, q = p / p.sum(), q / q.sum()
    # constraint matrix of vec(Z) (row-major): m row-sum rows, n column-sum rows
    A = np.zeros((m + n, m * n))
    for i in range(m):
        A[i, i * n:(i + 1) * n] = 1.0
    for j in range(n):
        A[m + j, j::n] = 1.0
    b = np.concatenate([p, q])
    v = V.ravel()
    z_ls = v - np.linalg.pinv(A) @ (A @ v - b)  # Euclidean projection onto {A z = b}
    Z, cr, cc = oracle.project_marginals(V, p, q)
    assert np.allclose(Z.ravel(), z_ls, atol=1e-12)
    assert np.allclose(Z.sum(1), p, atol=1e-13) and np.allclose(Z.sum(0), q, atol=1e-13)
    # the correction is a sum of a row-constant and a column-constant matrix
    assert np.allclose(Z - V, cr[:, None] + cc[None, :], atol=1e-14)
    # idempotent
    Z2, _, _ = oracle.project_marginals(Z, p, q)
    assert np.allclose(Z2, Z, atol=1e-13)


# ---------------------------------------------------------------------------------------------
# unregularized problem: optimum of the LP
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", [3, 4, 5, 6, 7])
def test_unregularized_optimum_equals_best_permutation(oracle, n):
    # uniform marginals, square: the LP optimum is attained at a permutation matrix / n (Birkhoff)
    C, p, q = _rand_problem(n, n, 100 + n, uniform=True)
    best = min(sum(float(C[i, s[i]]) for i in range(n)) for s in itertools.permutations(range(n))) / n
    rho = oracle.default_stepsize(n, n)
    res = oracle.solve(C, p, q, max_iters=30000)
    g = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho)
    assert abs(g.objective - best) < 1e-10
    assert abs(g.dual_linear - best) < 1e-10  # strong duality: dual value equals the optimum
    assert abs(g.gap) < 1e-10 and g.dual_res < 1e-10
    assert res.X.min() >= 0.0
    assert max(res.res_row[-1], res.res_col[-1]) < 1e-10


@pytest.mark.parametrize("m,n,seed", [(5, 8, 1), (12, 9, 2), (10, 10, 3)])
def test_unregularized_optimum_equals_lp_solver(oracle, m, n, seed):
    C, p, q = _rand_problem(m, n, seed)
    A_eq = np.zeros((m + n, m * n))
    for i in range(m):
        A_eq[i, i * n:(i + 1) * n] = 1.0
    for j in range(n):
        A_eq[m + j, j::n] = 1.0
    lp = sopt.linprog(C.astype(np.float64).ravel(), A_eq=A_eq[:-1], b_eq=np.concatenate([p, q])[:-1],
                      bounds=(0, None), method="highs")
    assert lp.status == 0
    rho = oracle.default_stepsize(m, n)
    res = oracle.solve(C, p, q, max_iters=60000)
    g = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho)
    assert abs(g.objective - lp.fun) < 1e-9
    # u = phi/rho, v = varphi/rho are Kantorovich potentials: dual feasible, dual value = optimum
    u, v = res.phi / rho, res.varphi / rho
    assert (u[:, None] + v[None, :] - C).max() < 1e-9
    assert abs(p @ u + q @ v - lp.fun) < 1e-9
    assert max(res.res_row[-1], res.res_col[-1]) < 1e-9


# ---------------------------------------------------------------------------------------------
# quadratic regularization
# ---------------------------------------------------------------------------------------------
def _solve_quadratic_dual(C, p, q, lam):
    """max_{u,v} p.u + q.v - ||[u (+) v - C]_+||^2 / (2 lam) with L-BFGS; X* = [u (+) v - C]_+ / lam."""
    m, n = C.shape
    C = C.astype(np.float64)

    def negdual(w):
        u, v = w[:m], w[m:]
        W = np.maximum(u[:, None] + v[None, :] - C, 0.0)
        val = p @ u + q @ v - (W ** 2).sum() / (2 * lam)
        gu = p - W.sum(1) / lam
        gv = q - W.sum(0) / lam
        return -val, -np.concatenate([gu, gv])

    out = sopt.minimize(negdual, np.zeros(m + n), jac=True, method="L-BFGS-B",
                        options=dict(maxiter=20000, maxfun=200000, ftol=1e-18, gtol=1e-13, maxcor=50))
    u, v = out.x[:m], out.x[m:]
    return np.maximum(u[:, None] + v[None, :] - C, 0.0) / lam, -out.fun


@pytest.mark.parametrize("m,n,lam,seed", [(6, 9, 0.5, 5), (10, 7, 2.0, 6)])
def test_quadratic_solution_equals_smooth_dual_solution(oracle, m, n, lam, seed):
    C, p, q = _rand_problem(m, n, seed)
    X_dual, dual_val = _solve_quadratic_dual(C, p, q, lam)
    rho = 0.2
    res = oracle.solve(C, p, q, rho=rho, reg_kind=oracle.REG_QUADRATIC, lam=lam, max_iters=40000)
    assert np.abs(res.X - X_dual).max() < 1e-7
    g = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho, reg_kind=oracle.REG_QUADRATIC, lam=lam)
    assert abs(g.objective - dual_val) < 1e-8
    assert abs(g.gap) < 1e-10
    # KKT: X* = [u (+) v - C]_+ / lam with u = phi/rho, v = varphi/rho
    u, v = res.phi / rho, res.varphi / rho
    assert np.abs(res.X - np.maximum(u[:, None] + v[None, :] - C, 0.0) / lam).max() < 1e-10
    # strongly convex => unique => independent of the stepsize
    res2 = oracle.solve(C, p, q, rho=0.05, reg_kind=oracle.REG_QUADRATIC, lam=lam, max_iters=80000)
    assert np.abs(res2.X - res.X).max() < 1e-9


def test_quadratic_prox_is_a_scaling(oracle):
    rng = np.random.default_rng(3)
    V = np.abs(rng.normal(size=(4, 6)))
    out = oracle.prox_h(V, 0.3, reg_kind=oracle.REG_QUADRATIC, lam=0.7)
    # argmin_x (lam/2) x^2 + (x - v)^2 / (2 rho)  =>  x = v / (1 + rho lam)
    assert np.allclose(out, V / (1 + 0.3 * 0.7), atol=1e-15)


# ---------------------------------------------------------------------------------------------
# group lasso (+ quadratic)
# ---------------------------------------------------------------------------------------------
def _prox_objective(x, v, rho, lam, mu):
    return mu * np.linalg.norm(x) + 0.5 * lam * (x @ x) + ((x - v) @ (x - v)) / (2 * rho)


@pytest.mark.parametrize("lam", [0.0, 0.8])
def test_group_lasso_prox_minimises_its_objective(oracle, lam):
    rng = np.random.default_rng(11)
    m, n, ncls = 7, 5, 3
    row_class = np.array([0, 2, 1, 1, 0, 2, 2], dtype=np.int32)  # not sorted on purpose
    V = np.abs(rng.normal(size=(m, n))) * rng.uniform(0.05, 1.0, size=(1, n))
    rho, mu = 0.4, 0.9
    out = oracle.prox_h(V, rho, reg_kind=oracle.REG_GROUP_LASSO, lam=lam, mu=mu, row_class=row_class, num_classes=ncls)
    n_zero_groups = 0
    for c in range(ncls):
        rows = np.where(row_class == c)[0]
        for j in range(n):
            v, x = V[rows, j], out[rows, j]
            f_x = _prox_objective(x, v, rho, lam, mu)
            # numerical minimiser from a few starts (objective is convex; nonsmooth only at 0)
            best = min(sopt.minimize(_prox_objective, x0, args=(v, rho, lam, mu), method="Nelder-Mead",
                                     options=dict(xatol=1e-10, fatol=1e-14, maxiter=20000)).fun
                       for x0 in (v, 0.5 * v, 1e-3 * np.ones_like(v)))
            assert f_x <= best + 1e-10
            assert f_x <= _prox_objective(np.zeros_like(v), v, rho, lam, mu) + 1e-15
            for _ in range(20):  # and no nearby point is better
                assert f_x <= _prox_objective(x + 1e-4 * rng.normal(size=x.shape), v, rho, lam, mu) + 1e-12
            n_zero_groups += int(not x.any())
    assert 0 < n_zero_groups < ncls * n  # both branches of the threshold were exercised


def test_group_lasso_prox_special_cases(oracle):
    rng = np.random.default_rng(12)
    m, n = 6, 8
    V = np.abs(rng.normal(size=(m, n)))
    V[2, 3] = 0.0
    rho, lam, mu = 0.25, 0.6, 0.5
    rc = np.array([0, 0, 1, 1, 1, 2], dtype=np.int32)
    # mu = 0 -> the quadratic prox
    a = oracle.prox_h(V, rho, reg_kind=oracle.REG_GROUP_LASSO, lam=lam, mu=0.0, row_class=rc, num_classes=3)
    assert np.allclose(a, V / (1 + rho * lam), atol=1e-15)
    # every row its own class -> groups are single entries -> elementwise soft threshold
    single = np.arange(m, dtype=np.int32)
    b = oracle.prox_h(V, rho, reg_kind=oracle.REG_GROUP_LASSO, lam=lam, mu=mu, row_class=single, num_classes=m)
    assert np.allclose(b, np.maximum(V - rho * mu, 0.0) / (1 + rho * lam), atol=1e-15)
    # lam = 0 -> textbook block soft threshold x = max(1 - rho mu/||v||, 0) v
    c = oracle.prox_h(V, rho, reg_kind=oracle.REG_GROUP_LASSO, lam=0.0, mu=mu, row_class=rc, num_classes=3)
    for cls in range(3):
        rows = np.where(rc == cls)[0]
        for j in range(n):
            v = V[rows, j]
            assert np.allclose(c[rows, j], max(1 - rho * mu / np.linalg.norm(v), 0.0) * v, atol=1e-15)
    # an all-zero group stays zero (no 0/0), zeros stay zero and signs are kept (Lemma A.1)
    Vz = V.copy()
    Vz[0:2, 1] = 0.0
    d = oracle.prox_h(Vz, rho, reg_kind=oracle.REG_GROUP_LASSO, lam=lam, mu=mu, row_class=rc, num_classes=3)
    assert np.isfinite(d).all() and (d[0:2, 1] == 0).all() and d[2, 3] == 0 and (d >= 0).all()


def test_group_lasso_singleton_groups_solve_the_quadratic_problem(oracle):
    # with groups of one entry h = mu*sum|X_ij| + (lam/2)||X||^2; on the feasible set sum X = 1,
    # so the minimiser is the one of the quadratic problem alone
    m, n, lam, mu = 6, 7, 0.7, 0.3
    C, p, q = _rand_problem(m, n, 21)
    rho = 0.2
    a = oracle.solve(C, p, q, rho=rho, reg_kind=oracle.REG_QUADRATIC, lam=lam, max_iters=40000)
    b = oracle.solve(C, p, q, rho=rho, reg_kind=oracle.REG_GROUP_LASSO, lam=lam, mu=mu,
                     row_class=np.arange(m, dtype=np.int32), num_classes=m, max_iters=40000)
    assert np.abs(a.X - b.X).max() < 1e-9


def _conj_sup(w, lam, mu):
    """sup_x <w,x> - mu||x|| - (lam/2)||x||^2 by numerical maximisation."""
    f = lambda x: -(w @ x - mu * np.linalg.norm(x) - 0.5 * lam * (x @ x))
    return -min(sopt.minimize(f, x0, method="Nelder-Mead", options=dict(xatol=1e-10, fatol=1e-14, maxiter=20000)).fun
                for x0 in (w, 0.1 * w, np.zeros_like(w) + 1e-3))


def test_gap_conjugate_terms_match_numerical_supremum(oracle):
    # one group (one class, one column): the h* term of the gap must equal the numerical sup
    rng = np.random.default_rng(31)
    m = 4
    for lam, mu in [(0.9, 0.0), (0.9, 0.4), (0.5, 2.5)]:
        C = rng.uniform(0.1, 1.0, size=(m, 1)).astype(np.float32)
        phi = rng.uniform(0.2, 1.5, size=m)
        varphi = np.array([0.3])
        rho = 0.7
        W = np.maximum((phi[:, None] + varphi[None, :]) / rho - C, 0.0)[:, 0]
        X = np.abs(rng.normal(size=(m, 1)))
        p, q = X.sum(1), X.sum(0)
        kind = oracle.REG_QUADRATIC if mu == 0.0 else oracle.REG_GROUP_LASSO
        g = oracle.objective_gap(C, X, p, q, phi, varphi, rho, reg_kind=kind, lam=lam, mu=mu,
                                 row_class=np.zeros(m, dtype=np.int32), num_classes=1)
        assert abs(g.h_conj - _conj_sup(W, lam, mu)) < 1e-8
        assert abs(g.cost - float((C.astype(np.float64) * X).sum())) < 1e-14
        assert abs(g.h - (mu * np.linalg.norm(X) + 0.5 * lam * (X ** 2).sum())) < 1e-14
        assert abs(g.dual_linear - (p @ phi + q @ varphi) / rho) < 1e-14
        assert abs(g.gap - (g.cost + g.h - g.dual_linear + g.h_conj)) < 1e-14


@pytest.mark.parametrize("lam", [0.5, 0.0])
def test_group_lasso_solution_is_certified_by_the_gap(oracle, lam):
    # weak duality: gap >= 0 for a dual-feasible pair and gap = 0 only at the optimum
    m, n, ncls, mu = 12, 10, 3, 0.05
    C, p, q = _rand_problem(m, n, 41)
    rc = np.sort(np.random.default_rng(42).integers(0, ncls, m)).astype(np.int32)
    rho = 0.1
    res = oracle.solve(C, p, q, rho=rho, reg_kind=oracle.REG_GROUP_LASSO, lam=lam, mu=mu, row_class=rc,
                       num_classes=ncls, max_iters=100000)
    g = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho, reg_kind=oracle.REG_GROUP_LASSO,
                             lam=lam, mu=mu, row_class=rc, num_classes=ncls)
    assert max(res.res_row[-1], res.res_col[-1]) < 1e-9
    assert res.X.min() >= 0.0
    assert abs(g.gap) < 1e-9 and g.dual_res < 1e-9
    # compare with a general-purpose constrained minimiser on the same (tiny) problem
    if lam > 0:
        A = np.zeros((m + n, m * n))
        for i in range(m):
            A[i, i * n:(i + 1) * n] = 1.0
        for j in range(n):
            A[m + j, j::n] = 1.0

        def obj(x):
            X = x.reshape(m, n)
            gl = sum(np.sqrt((X[rc == c] ** 2).sum(0) + 1e-16).sum() for c in range(ncls))
            return float((C * X).sum() + mu * gl + 0.5 * lam * (X ** 2).sum())

        out = sopt.minimize(obj, np.outer(p, q).ravel(), method="SLSQP", bounds=[(0, None)] * (m * n),
                            constraints=[dict(type="eq", fun=lambda x: A[:-1] @ x - np.concatenate([p, q])[:-1])],
                            options=dict(maxiter=500, ftol=1e-14))
        assert g.objective <= out.fun + 1e-7  # the oracle's plan is at least as good
        assert abs(g.objective - out.fun) < 1e-4


# ---------------------------------------------------------------------------------------------
# the O(m+n) recursion printed as eq. (6) reproduces the explicit three-update iteration
# ---------------------------------------------------------------------------------------------
def _np_prox(kind, rho, lam, mu, rc, ncls):
    if kind == 0:
        return lambda V: V
    if kind == 1:
        return lambda V: V / (1 + rho * lam)

    def gl(V):
        out = np.zeros_like(V)
        for c in range(ncls):
            rows = rc == c
            nrm = np.sqrt((V[rows] ** 2).sum(0))
            sc = np.where(nrm > 0, np.maximum(1 - rho * mu / np.where(nrm > 0, nrm, 1.0), 0.0), 0.0) / (1 + rho * lam)
            out[rows] = V[rows] * sc[None, :]
        return out

    return gl


def _eq6_iterates(C, p, q, rho, prox, K):
    """Eq. (5)/(8) for X with the vector recursion of eq. (6), f = 1_m, e = 1_n."""
    m, n = C.shape
    C = C.astype(np.float64)
    phi = np.full(m, (1 + m / (m + n)) / (3 * (m + n)))
    varphi = np.full(n, (1 + n / (m + n)) / (3 * (m + n)))
    X = np.zeros((m, n))
    a = n * phi + varphi.sum() - p  # a_0 = Y_0 1 - p
    b = m * varphi + phi.sum() - q
    theta = a.sum() / (m + n)
    for _ in range(K):
        X = prox(np.maximum(X + phi[:, None] + varphi[None, :] - rho * C, 0.0))
        r, s = X.sum(1) - p, X.sum(0) - q
        eta = r.sum() / (m + n)
        phi = (a - 2 * r + (2 * eta - theta)) / n
        varphi = (b - 2 * s + (2 * eta - theta)) / m
        a, b, theta = a - r, b - s, theta - eta
    return X, phi, varphi, a, b, theta


@pytest.mark.parametrize("kind", [0, 1, 2])
@pytest.mark.parametrize("m,n", [(9, 13), (16, 16)])
def test_eq6_vector_recursion_equals_explicit_iteration(oracle, kind, m, n):
    C, p, q = _rand_problem(m, n, 50 + kind)
    rc = np.random.default_rng(5).integers(0, 3, m).astype(np.int32)
    rho, lam, mu = 2.0 / (m + n), 0.3, 0.02
    K = 300
    X6, phi6, varphi6, a6, b6, theta6 = _eq6_iterates(C, p, q, rho, _np_prox(kind, rho, lam, mu, rc, 3), K)
    res = oracle.solve(C, p, q, rho=rho, reg_kind=kind, lam=lam, mu=mu, row_class=rc, num_classes=3,
                       max_iters=K, return_Y=True)
    assert np.abs(res.X - X6).max() < 1e-13
    assert np.abs(res.phi - phi6).max() < 1e-13 and np.abs(res.varphi - varphi6).max() < 1e-13
    # eq. (5): Y_k - X_k = phi_k 1^T + 1 varphi_k^T ; and a_k = Y_k 1 - p, b_k = Y_k^T 1 - q
    assert np.abs(res.Y - res.X - res.phi[:, None] - res.varphi[None, :]).max() < 1e-13
    assert np.abs(res.Y.sum(1) - p - a6).max() < 1e-12 and np.abs(res.Y.sum(0) - q - b6).max() < 1e-12
    assert abs(theta6 - a6.sum() / (m + n)) < 1e-13
    # the residual trace is the one of the iterate just produced; and 1^T r = 1^T s
    assert abs(res.res_row[-1] - np.linalg.norm(X6.sum(1) - p)) < 1e-14
    assert abs(res.res_col[-1] - np.linalg.norm(X6.sum(0) - q)) < 1e-14
    assert abs((X6.sum(1) - p).sum() - (X6.sum(0) - q).sum()) < 1e-14


# ---------------------------------------------------------------------------------------------
# initialization (Initialization paragraph and Appendix B)
# ---------------------------------------------------------------------------------------------
def test_initial_vectors_match_hand_computed_values(oracle):
    # tests/golden/init_constants.txt: exact rationals worked out by hand from the printed formula
    with open(os.path.join(GOLDEN, "init_constants.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert rows
    for m, n, pn, pd, vn, vd in rows:
        phi0, varphi0 = oracle.initial_vectors(int(m), int(n))
        assert phi0.shape == (int(m),) and varphi0.shape == (int(n),)
        assert abs(phi0[0] - int(pn) / int(pd)) < 1e-18 and abs(varphi0[0] - int(vn) / int(vd)) < 1e-18


def test_cold_start_stays_at_zero_for_the_predicted_number_of_iterations(oracle):
    # Appendix B: from X_0 = p q^T, phi_0 = varphi_0 = 0 and rho = 2/(m+n) the first iterates are
    # X_k = 0 with phi_k, varphi_k growing linearly in k.  Carrying eq. (6) through by hand gives
    #   phi_k = (k+1)(p - 1/(m+n))/n,  varphi_k = (k+1)(q - 1/(m+n))/m
    # (the appendix prints "+ 1/(m+n)"; with that sign eq. (6) is not satisfied), hence X_k = 0
    # exactly while k <= min_ij rho C_ij / (p_i/n + q_j/m - 1/(mn)).
    m, n = 30, 50
    rng = np.random.default_rng(1)
    C = rng.uniform(0.5, 1.0, size=(m, n)).astype(np.float32)
    C /= C.max()
    p = rng.uniform(0.5, 1.5, m)
    q = rng.uniform(0.5, 1.5, n)
    p, q = p / p.sum(), q / q.sum()
    rho = 2.0 / (m + n)
    w = p[:, None] / n + q[None, :] / m - 1.0 / (m * n)
    N = int(np.floor((rho * C.astype(np.float64) / w)[w > 0].min()))
    assert N >= 5
    X0 = np.outer(p, q)
    for k in (1, 2, N):
        res = oracle.solve(C, p, q, rho=rho, max_iters=k, X0=X0, phi0=np.zeros(m), varphi0=np.zeros(n))
        assert not res.X.any()
        assert np.abs(res.phi - (k + 1) * (p - 1.0 / (m + n)) / n).max() < 1e-15
        assert np.abs(res.varphi - (k + 1) * (q - 1.0 / (m + n)) / m).max() < 1e-15
    res = oracle.solve(C, p, q, rho=rho, max_iters=N + 1, X0=X0, phi0=np.zeros(m), varphi0=np.zeros(n))
    assert res.X.any()
    # the warm start of the Initialization paragraph skips that phase: phi_0 + varphi_0 = 1/(m+n)
    # = rho/2, so the first iterate is X_1 = rho [1/2 - C]_+ in closed form
    C2 = rng.uniform(0.0, 1.0, size=(m, n)).astype(np.float32)
    warm = oracle.solve(C2, p, q, rho=rho, max_iters=1)
    assert np.abs(warm.X - rho * np.maximum(0.5 - C2.astype(np.float64), 0.0)).max() < 1e-16
    assert warm.X.any()


# ---------------------------------------------------------------------------------------------
# invariants that hold for every regularizer
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [0, 1, 2])
def test_feasibility_nonnegativity_and_residual_decay(oracle, kind):
    import drot_inputs

    P = drot_inputs.random_problem(40, 56, seed=7, reg_kind=kind, lam=0.2, mu=0.02, num_classes=4)
    kw = dict(reg_kind=kind, lam=P.lam, mu=P.mu, row_class=P.row_class, num_classes=P.num_classes)
    a = oracle.solve(P.C, P.p, P.q, max_iters=500, **kw)
    b = oracle.solve(P.C, P.p, P.q, max_iters=4000, **kw)
    assert a.X.min() >= 0 and b.X.min() >= 0
    assert max(b.res_row[-1], b.res_col[-1]) < 0.2 * max(a.res_row[-1], a.res_col[-1])
    g = oracle.objective_gap(P.C, b.X, P.p, P.q, b.phi, b.varphi, float(P.rho), **kw)
    ga = oracle.objective_gap(P.C, a.X, P.p, P.q, a.phi, a.varphi, float(P.rho), **kw)
    assert abs(g.gap) < abs(ga.gap) + 1e-12


def test_stopping_rule_takes_first_passing_check(oracle):
    C, p, q = _rand_problem(20, 20, 9)
    full = oracle.solve(C, p, q, max_iters=5000)
    tol = 1e-4
    res = oracle.solve(C, p, q, max_iters=5000, tol=tol, check_every=10)
    r = np.maximum(full.res_row, full.res_col)
    expected = next(k for k in range(10, 5001, 10) if r[k - 1] <= tol)
    assert res.iters == expected
    assert max(res.res_row[-1], res.res_col[-1]) <= tol


@pytest.mark.parametrize("kind", [0, 1])
def test_gap_stopping_rule_takes_the_first_check_that_passes_both_tests(oracle, kind):
    # Section 3 "Stopping criteria" / Appendix C: with a gap tolerance a check passes when the residual
    # test does and |gap| <= gap_tol |objective|, dual residual <= gap_tol, the gap being evaluated at
    # every gap_every-th check only.  The expected stop is rebuilt from separate fixed-length runs and
    # the (separately pinned) evaluation of the gap at their iterates.
    C, p, q = _rand_problem(18, 22, 11)
    kw = dict(reg_kind=kind, lam=0.5 if kind else 0.0)
    tol, gap_tol, every, gap_every = 2e-3, 5e-3, 10, 3
    rho = oracle.default_stepsize(18, 22)
    res = oracle.solve(C, p, q, max_iters=20000, tol=tol, check_every=every, gap_every=gap_every, gap_tol=gap_tol, **kw)
    plain = oracle.solve(C, p, q, max_iters=20000, tol=tol, check_every=every, **kw)
    expected = None
    for k in range(every * gap_every, 20001, every * gap_every):
        it = oracle.solve(C, p, q, max_iters=k, **kw)
        t = oracle.objective_gap(C, it.X, p, q, it.phi, it.varphi, rho, **kw)
        if (max(it.res_row[-1], it.res_col[-1]) <= tol and abs(t.gap) <= gap_tol * abs(t.objective)
                and t.dual_res <= gap_tol):
            expected = k
            break
    assert expected is not None and res.iters == expected
    assert res.iters > plain.iters  # (the gap test is the binding one here)
    # the trace holds every evaluation up to the stop, at the multiples of every * gap_every
    assert list(res.gap_trace[:, 0]) == list(range(every * gap_every, expected + 1, every * gap_every))
    last = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho, **kw)
    assert res.gap_trace[-1, 1] == last.objective and res.gap_trace[-1, 2] == last.gap and res.gap_trace[-1, 3] == last.dual_res


def test_point_cloud_cost_matches_numpy_and_scipy(oracle):
    from scipy.spatial.distance import cdist

    rng = np.random.default_rng(77)
    xs = rng.normal(size=(13, 5)).astype(np.float32)
    xt = rng.normal(0.5, 2.0, size=(9, 5)).astype(np.float32)
    ref = cdist(xs.astype(np.float64), xt.astype(np.float64), metric="sqeuclidean")
    C = oracle.sqdist_cost(xs, xt, 0.25)
    assert C.dtype == np.float32 and C.shape == (13, 9)
    assert np.abs(C - 0.25 * ref).max() <= 1e-6 * (0.25 * ref).max()
    assert (oracle.sqdist_cost(xs, xs, 1.0).diagonal() == 0).all()


# ---------------------------------------------------------------------------------------------
# entrywise members of the class of Section 2: weighted l1 and constrained OT
# ---------------------------------------------------------------------------------------------
def _marginal_constraints(m, n):
    A_eq = np.zeros((m + n, m * n))
    for i in range(m):
        A_eq[i, i * n:(i + 1) * n] = 1.0
    for j in range(n):
        A_eq[m + j, j::n] = 1.0
    return A_eq


def test_weighted_l1_prox_is_the_scalar_minimiser(oracle):
    # argmin_x rho*w*|x| + (x - v)^2/2 for v >= 0, by a bounded scalar minimiser
    rng = np.random.default_rng(21)
    V = np.abs(rng.normal(size=(6, 5)))
    W = rng.uniform(0.0, 2.0, size=(6, 5)).astype(np.float32)
    rho = 0.7
    out = oracle.prox_entrywise(V, rho, weights=W)
    hit_zero = 0
    for v, w, x in zip(V.ravel(), W.ravel().astype(np.float64), out.ravel()):
        ref = sopt.minimize_scalar(lambda z: rho * w * abs(z) + 0.5 * (z - v) ** 2, bounds=(-5.0, 5.0), method="bounded",
                                   options=dict(xatol=1e-12)).x
        assert abs(x - ref) < 1e-6
        assert x == max(v - rho * w, 0.0)
        hit_zero += int(x == 0.0)
    assert 0 < hit_zero < V.size
    # forbidden entries are projected to zero, the rest is untouched
    S = rng.uniform(size=V.shape) < 0.3
    out = oracle.prox_entrywise(V, rho, forbidden=S)
    assert not out[S].any() and np.array_equal(out[~S], V[~S])


@pytest.mark.parametrize("lam", [0.0, 0.6])
def test_entrywise_terms_compose_with_the_group_lasso_prox(oracle, lam):
    # prox of rho*(<W,X> + indicator{X_S = 0} + mu*sum_g ||X_g|| + lam/2 ||X||^2) at a nonnegative
    # point, computed as entrywise step then group step, against a numerical minimiser per group
    rng = np.random.default_rng(22)
    m, n, ncls = 6, 4, 2
    row_class = np.array([0, 1, 0, 1, 1, 0], dtype=np.int32)
    V = np.abs(rng.normal(size=(m, n)))
    W = rng.uniform(0.0, 0.8, size=(m, n)).astype(np.float32)
    S = rng.uniform(size=(m, n)) < 0.25
    rho, mu = 0.5, 0.7
    out = oracle.prox_h(oracle.prox_entrywise(V, rho, weights=W, forbidden=S), rho, reg_kind=oracle.REG_GROUP_LASSO,
                        lam=lam, mu=mu, row_class=row_class, num_classes=ncls)
    assert not out[S].any() and out.min() >= 0.0
    for c in range(ncls):
        rows = np.where(row_class == c)[0]
        for j in range(n):
            free = ~S[rows, j]
            v, w, x = V[rows, j][free], W[rows, j][free].astype(np.float64), out[rows, j][free]
            if v.size == 0:
                continue

            def f(z):
                return (w @ np.abs(z)) + mu * np.linalg.norm(z) + 0.5 * lam * (z @ z) + ((z - v) @ (z - v)) / (2 * rho)

            best = min(sopt.minimize(f, z0, method="Nelder-Mead", options=dict(xatol=1e-10, fatol=1e-14, maxiter=40000)).fun
                       for z0 in (v, 0.5 * v, 1e-3 * np.ones_like(v)))
            assert f(x) <= best + 1e-9


@pytest.mark.parametrize("m,n,seed", [(6, 9, 5), (10, 10, 6)])
def test_weighted_l1_solution_equals_lp_with_shifted_cost(oracle, m, n, seed):
    # on X >= 0 the l1 term is linear: min <C,X> + <W,X> over the transport polytope
    C, p, q = _rand_problem(m, n, seed)
    W = np.random.default_rng(seed + 50).uniform(0.0, 0.7, size=(m, n)).astype(np.float32)
    A_eq = _marginal_constraints(m, n)
    lp = sopt.linprog((C.astype(np.float64) + W.astype(np.float64)).ravel(), A_eq=A_eq[:-1],
                      b_eq=np.concatenate([p, q])[:-1], bounds=(0, None), method="highs")
    assert lp.status == 0
    rho = oracle.default_stepsize(m, n)
    res = oracle.solve(C, p, q, max_iters=60000, weights=W)
    g = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho, weights=W)
    assert abs(g.objective - lp.fun) < 1e-9
    assert abs(g.h - float((W.astype(np.float64) * res.X).sum())) < 1e-12
    assert abs(g.gap) < 1e-9 and g.dual_res < 1e-9
    # the plain problem with the same C has a different optimum: the weights matter here
    lp0 = sopt.linprog(C.astype(np.float64).ravel(), A_eq=A_eq[:-1], b_eq=np.concatenate([p, q])[:-1], bounds=(0, None),
                       method="highs")
    assert lp0.fun < lp.fun - 1e-3


@pytest.mark.parametrize("n", [4, 5, 6])
def test_constrained_optimum_equals_best_allowed_permutation(oracle, n):
    # uniform marginals: the optimum over plans that vanish on S is a permutation avoiding S
    C, p, q = _rand_problem(n, n, 300 + n, uniform=True)
    best_perm = min(itertools.permutations(range(n)), key=lambda s: sum(float(C[i, s[i]]) for i in range(n)))
    S = np.zeros((n, n), dtype=bool)
    for i in range(0, n, 2):
        S[i, best_perm[i]] = True  # forbid half of the unconstrained optimum
    allowed = [s for s in itertools.permutations(range(n)) if not any(S[i, s[i]] for i in range(n))]
    best = min(sum(float(C[i, s[i]]) for i in range(n)) for s in allowed) / n
    rho = oracle.default_stepsize(n, n)
    res = oracle.solve(C, p, q, max_iters=40000, forbidden=S)
    g = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho, forbidden=S)
    assert not res.X[S].any()
    assert abs(g.objective - best) < 1e-9 and abs(g.gap) < 1e-9 and g.dual_res < 1e-9
    assert max(res.res_row[-1], res.res_col[-1]) < 1e-9


@pytest.mark.parametrize("lam", [0.0, 0.05])
def test_constrained_solution_equals_constrained_program(oracle, lam):
    # general marginals: LP (lam = 0) resp. QP (lam > 0, SLSQP) with the entries of S fixed at zero
    m, n = 7, 6
    C, p, q = _rand_problem(m, n, 77)
    S = np.random.default_rng(78).uniform(size=(m, n)) < 0.3
    S[np.arange(m), np.arange(m) % n] = False  # keep the problem feasible with room to spare
    A_eq = _marginal_constraints(m, n)
    b_eq = np.concatenate([p, q])
    bounds = [(0, 0) if s else (0, None) for s in S.ravel()]
    c64 = C.astype(np.float64).ravel()
    lp = sopt.linprog(c64, A_eq=A_eq[:-1], b_eq=b_eq[:-1], bounds=bounds, method="highs")
    assert lp.status == 0
    rho = oracle.default_stepsize(m, n)
    kind = oracle.REG_QUADRATIC if lam > 0 else oracle.REG_NONE
    res = oracle.solve(C, p, q, reg_kind=kind, lam=lam, max_iters=80000, forbidden=S)
    g = oracle.objective_gap(C, res.X, p, q, res.phi, res.varphi, rho, reg_kind=kind, lam=lam, forbidden=S)
    assert not res.X[S].any() and max(res.res_row[-1], res.res_col[-1]) < 1e-9
    if lam == 0.0:
        assert abs(g.objective - lp.fun) < 1e-9
    else:
        qp = sopt.minimize(lambda x: c64 @ x + 0.5 * lam * (x @ x), lp.x, jac=lambda x: c64 + lam * x, method="SLSQP",
                           bounds=bounds, constraints=[dict(type="eq", fun=lambda x: A_eq[:-1] @ x - b_eq[:-1],
                                                            jac=lambda x: A_eq[:-1])],
                           options=dict(ftol=1e-14, maxiter=500))
        assert qp.success
        assert abs(g.objective - qp.fun) < 1e-7
        assert np.abs(res.X.ravel() - qp.x).max() < 1e-5
    assert abs(g.gap) < 1e-8
