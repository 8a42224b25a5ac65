"""GPU parity tests: the HIP solver (through the C ABI) against the fp64 CPU oracle.

Run on the MI355X machine with `python -u -m pytest tests -m gpu -x -v --timeout 600 --timeout-method thread`.
Each case prints what it is about to run (and flushes) before touching the GPU.
"""
import sys

import numpy as np
import pytest
import torch

import drot_inputs
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-parity] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def drot():
    import paper_2305_18483_amd as drot_mod

    drot_mod.load_library()  # raises if the HIP library is missing: no fallback
    assert torch.cuda.is_available()
    return drot_mod


_CONFIGS = {}


def _config(k):
    """The k-th benchmark configuration, generated once per test session (cfg4 takes a while)."""
    if k not in _CONFIGS:
        _say(f"generating configuration {k}")
        _CONFIGS[k] = drot_inputs.config(k)
    return _CONFIGS[k]


def _stats():
    st = pu.LAST_STATS
    return (f"support mismatches {st.get('support_mismatches')} of {st.get('nonzeros')} nonzeros "
            f"(largest such entry / scale {st.get('largest_mismatched_entry', 0.0):.1e}), relative error on entries "
            f">= 1e-2 max {st.get('rel_err_big_entries', 0.0):.1e}, Frobenius {st.get('frob', 0.0):.1e}")


def _run_case(drot, oracle, P, K, label, solver=None, **kw):
    _say(f"{label}: {P.name} m={P.m} n={P.n} reg={P.reg_kind} K={K}")
    solver = solver or drot.Solver(P.m, P.n)
    gres, Xg, phig, varphig = pu.gpu_solve(solver, P, K, **kw)
    assert gres.code == drot.DROT_OK and gres.iters == K
    _say(f"{label}: GPU done, oracle running")
    ores = pu.oracle_solve(oracle, P, K, stepsize=kw.get("stepsize") or None)
    ratio = pu.assert_parity(oracle, P, gres, Xg, phig, varphig, ores, stepsize=kw.get("stepsize") or None, label=label)
    _say(f"{label}: plan error / scale = {ratio:.2e}; {_stats()}")
    return gres, Xg, ores


def _checks_of(P, X, phi, varphi):
    """fp64 evaluation of a returned triple by the plain-torch module that shares nothing with either solver."""
    import drot_checks

    dev = X.device
    rc = None if P.row_class is None else torch.from_numpy(P.row_class).to(dev)
    return drot_checks.fp64_terms(torch.from_numpy(P.C).to(dev), X, torch.from_numpy(P.p).to(dev),
                                  torch.from_numpy(P.q).to(dev), phi, varphi, float(P.rho), reg_kind=P.reg_kind,
                                  lam=float(np.float32(P.lam)), mu=float(np.float32(P.mu)), row_class=rc,
                                  num_classes=P.num_classes)


# ---------------------------------------------------------------------------------------------
# the five benchmark configurations
# ---------------------------------------------------------------------------------------------
def test_cfg1_unregularized_100_fixed_2000(drot, oracle):
    _run_case(drot, oracle, _config(1), 2000, "cfg1")


def test_cfg2_quadratic_1000_fixed_3000(drot, oracle):
    _run_case(drot, oracle, _config(2), 3000, "cfg2")


def _to_tolerance_against_the_oracle(drot, oracle, P, solver, tol, check_every, max_iters, label):
    """Both sides iterate to the residual `tol`, testing every check_every iterations.  The stop checks may
    differ by one interval (a borderline test can flip with fp32 rounding); the plans are compared element
    by element at the earlier of the two stops, the later side re-run for exactly that many iterations."""
    _say(f"{label}: to {tol:g}, GPU")
    gres, Xg, phig, varphig = pu.gpu_solve(solver, P, max_iters, tol=tol)
    assert gres.code == drot.DROT_OK and gres.converged and gres.iters % check_every == 0
    _say(f"{label}: GPU stopped after {gres.iters}; oracle running")
    ores = pu.oracle_solve(oracle, P, max_iters, tol=tol, check_every=check_every)
    _say(f"{label}: oracle stopped after {ores.iters}")
    assert abs(gres.iters - ores.iters) <= check_every, (gres.iters, ores.iters)
    r, s_ = pu.residuals(P, Xg)
    assert max(r, s_) <= tol + 1e-7
    stop_g = gres.iters
    K = min(gres.iters, ores.iters)
    if gres.iters > K:
        gres, Xg, phig, varphig = pu.gpu_solve(solver, P, K)
    if ores.iters > K:
        ores = pu.oracle_solve(oracle, P, K)
    ratio = pu.assert_parity(oracle, P, gres, Xg, phig, varphig, ores, label=label)
    _say(f"{label}: at iteration {K}: plan error / scale = {ratio:.2e}; {_stats()}")
    return stop_g, ores


def test_cfg2_quadratic_1000_to_tolerance(drot, oracle):
    # the run the configuration names: to a marginal residual of 1e-5, both sides, compared element by
    # element where they stop (and the same at 1e-4, which takes a tenth of the iterations)
    P = _config(2)
    solver = drot.Solver(P.m, P.n, check_every=100)
    _to_tolerance_against_the_oracle(drot, oracle, P, solver, 1e-4, 100, 200000, "cfg2 to 1e-4")
    stop, _ = _to_tolerance_against_the_oracle(drot, oracle, P, solver, 1e-5, 100, 400000, "cfg2 to 1e-5")
    # Optimality of the returned point, scaled so that nothing small is divided by.  A fixed point of the
    # sweep satisfies rho*lambda*X = [phi + varphi - rho*C]_+ entry by entry (Section 3, quadratic
    # regularization: X = [Y - rho C]_+ / (1 + rho*lambda), with Y - X = phi 1^T + 1 varphi^T); one sweep
    # away from it, X_K and X_{K+1} = [X_K + t]_+ / (1 + rho*lambda) with t = phi_K + varphi_K - rho C give
    # |rho*lambda*X_K - [t]_+| <= (1 + rho*lambda) |X_K - X_{K+1}| in every entry (case by case on the signs
    # of t and X_K + t).  So the defect is bounded by the last change of the plan, plus the fp32 rounding of
    # t (terms of size rho).  (The textbook form X = [u + v - C]_+ / lambda is this identity divided by
    # rho*lambda = 1e-5: it magnifies the rounding of t a hundred thousand times and holds only in the limit.)
    import drot_checks

    gres, Xg, phig, varphig = pu.gpu_solve(solver, P, 400000, tol=1e-5)
    assert gres.iters == stop
    dev = torch.device("cuda:0")
    C, X_K = torch.from_numpy(P.C).to(dev), torch.from_numpy(Xg).to(dev)
    lam, rho = float(np.float32(P.lam)), float(P.rho)
    defect = drot_checks.fixed_point_defect(C, X_K, torch.from_numpy(phig).to(dev), torch.from_numpy(varphig).to(dev), rho, lam)
    solver.set_continue(True)
    _, X_next, _, _ = pu.gpu_solve(solver, P, 1, X_out=X_K.clone())
    solver.set_continue(False)
    change = float(np.abs(X_next.astype(np.float64) - Xg.astype(np.float64)).max())
    rounding = 8 * 2.0 ** -24 * rho * 3.0  # phi_i, varphi_j and rho*C_ij are each below 3*rho here
    _say(f"cfg2 at 1e-5: fixed-point defect {defect:.3e}, last change of the plan {change:.3e}, plan scale {Xg.max():.3e}")
    assert defect <= (1.0 + rho * lam) * change + rounding
    t = _checks_of(P, X_K, torch.from_numpy(phig).to(dev), torch.from_numpy(varphig).to(dev))
    assert t.min_entry >= 0.0 and max(t.r_row, t.r_col) <= 1e-5 + 1e-7
    assert abs(gres.objective - t.objective) <= 1e-5 * abs(t.objective)
    assert abs(gres.gap - t.gap) <= 2e-5 * max(abs(t.cost), abs(t.dual_linear), abs(t.h_conj))


def test_cfg3_unregularized_10000_reduced_K(drot, oracle):
    # full size, the launch configuration the benchmark times: the dense first sweeps
    _run_case(drot, oracle, _config(3), 30, "cfg3")


def test_cfg4_quadratic_20000_reduced_K(drot, oracle):
    _run_case(drot, oracle, _config(4), 12, "cfg4")


@pytest.mark.parametrize("cfg,K", [(3, 1000), (4, 500)])
def test_full_size_fixed_iterations_against_the_oracle(drot, oracle, cfg, K):
    # the fixed-iteration runs the configurations name (1000 resp. 500 iterations), element by element
    # against the fp64 iteration, in the launch configuration the benchmark times: by then the solver has
    # long moved to the lean screened sweep (line flags, its own renewals of the bounds).  The oracle
    # needs one to two minutes for these.
    P = _config(cfg)
    solver = drot.Solver(P.m, P.n)
    solver.set_profile(True)
    gres, Xg, ores = _run_case(drot, oracle, P, K, f"cfg{cfg}, {K} iterations", solver=solver)
    kinds = [k for _, k in solver.profile_sweeps()]
    solver.set_profile(False)
    assert kinds.count(7) >= 20, kinds
    # fp64 properties of the returned plan that hold at any size
    X = torch.from_numpy(Xg).to("cuda:0").double()
    r = float((X.sum(dim=1) - torch.from_numpy(P.p).to("cuda:0").double()).norm())
    s_ = float((X.sum(dim=0) - torch.from_numpy(P.q).to("cuda:0").double()).norm())
    assert float(X.min()) >= 0.0
    assert abs(r - gres.r_row) <= 1e-6 and abs(s_ - gres.r_col) <= 1e-6, (r, gres.r_row, s_, gres.r_col)


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_full_size_runs_to_tolerance_hold_up_in_fp64(drot, cfg):
    # the time-to-tolerance runs the benchmark reports (tens of thousands of iterations at cfg4, hundreds
    # of renewals of the screening bounds): what they return is checked by fp64 code that shares nothing
    # with the library -- nonnegativity, both residual norms, objective, duality gap (Appendix C)
    P = _config(cfg)
    dev = torch.device("cuda:0")
    solver = drot.Solver(P.m, P.n, check_every=100)
    _say(f"cfg{cfg} to a residual of 1e-4")
    C, p, q, rc = pu.to_dev(P)
    res = solver.solve(C, p, q, reg_kind=P.reg_kind, lam=P.lam, mu=P.mu, row_class=rc, num_classes=P.num_classes,
                       max_iters=100000, tol=1e-4)
    phi, varphi = solver.duals(P.m, P.n, dev)
    torch.cuda.synchronize()
    assert res.code == drot.DROT_OK and res.converged and res.iters % 100 == 0
    t = _checks_of(P, res.X, phi, varphi)
    _say(f"cfg{cfg}: {res.iters} iterations; fp64: min {t.min_entry:.1e}, residuals {t.r_row:.3e}/{t.r_col:.3e}, "
         f"objective {t.objective:.8f} (reported {res.objective:.8f}), gap {t.gap:.4e} (reported {res.gap:.4e}), "
         f"dual residual {t.dual_res:.3e} (reported {res.dual_res:.3e}), {t.nnz} nonzeros")
    assert t.min_entry >= 0.0
    assert max(t.r_row, t.r_col) <= 1e-4 + 1e-7
    assert abs(t.r_row - res.r_row) <= 1e-6 and abs(t.r_col - res.r_col) <= 1e-6
    assert abs(res.objective - t.objective) <= 1e-5 * abs(t.objective)
    gap_scale = max(abs(t.cost), abs(t.dual_linear), abs(t.h_conj))
    assert abs(res.gap - t.gap) <= 2e-5 * gap_scale
    assert abs(res.dual_res - t.dual_res) <= 2e-5 * max(t.dual_res, gap_scale)


def test_beyond_the_benchmark_size(drot):
    # 1.4e9 entries (twice the benchmark's rows, ragged, padded working copies): the indices of every
    # array stay in range, the screened sweeps give the bits of the unscreened ones, and the residuals
    # the library reports are those of the returned plan in fp64.  Inputs are made on the device.
    m, n = 40000, 35007
    gen = torch.Generator(device="cuda:0").manual_seed(77)
    xs = torch.randn((m, 3), generator=gen, device="cuda:0")
    xt = 0.3 + 1.2 * torch.randn((n, 3), generator=gen, device="cuda:0")
    C = torch.cdist(xs, xt).pow_(2)
    C /= C.max()
    p = torch.full((m,), 1.0 / m, device="cuda:0")
    q = torch.full((n,), 1.0 / n, device="cuda:0")
    solver = drot.Solver(m, n, compute_gap=False)
    _say(f"large problem {m}x{n}")
    outs = []
    for mode in (0, -1):
        solver.set_screening(mode)
        X = torch.empty_like(C)
        res = solver.solve(C, p, q, reg_kind=1, lam=1e-3, max_iters=260, X_out=X)
        phi, varphi = solver.duals(m, n, C.device)
        outs.append((X, phi.clone(), varphi.clone(), res))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][2], outs[1][2])
    X, res = outs[1][0], outs[1][3]
    assert float(X.min()) >= 0.0
    r = float((X.sum(dim=1, dtype=torch.float64) - p.double()).norm())
    s_ = float((X.sum(dim=0, dtype=torch.float64) - q.double()).norm())
    assert abs(r - res.r_row) <= 1e-6 and abs(s_ - res.r_col) <= 1e-6, (r, res.r_row, s_, res.r_col)


def test_cfg5_group_lasso_5000_fixed_1000(drot, oracle):
    # the configuration's own run: 1000 iterations at full size
    _run_case(drot, oracle, _config(5), 1000, "cfg5")


def test_cfg5_recipe_1000_fixed_1000(drot, oracle):
    _run_case(drot, oracle, drot_inputs.config(5, size=1000), 1000, "cfg5 small")


# ---------------------------------------------------------------------------------------------
# ragged shapes, several tiles, tails; all three regularizers
# ---------------------------------------------------------------------------------------------
SHAPES = [(1, 1), (1, 700), (700, 1), (5, 3), (64, 256), (65, 257), (333, 517), (257, 1023), (1300, 900),
          (2050, 1030)]


@pytest.mark.parametrize("m,n", SHAPES)
@pytest.mark.parametrize("kind", [0, 1, 2])
def test_ragged_shapes(drot, oracle, m, n, kind):
    P = drot_inputs.random_problem(m, n, seed=1000 + 3 * m + n, reg_kind=kind, lam=0.5 if kind else 0.0,
                                   mu=0.05 if kind == 2 else 0.0, num_classes=min(7, m))
    _run_case(drot, oracle, P, 150, f"ragged {m}x{n} kind={kind}")


def test_group_lasso_unsorted_labels(drot, oracle):
    P = drot_inputs.random_problem(300, 413, seed=77, reg_kind=2, lam=0.1, mu=0.08, num_classes=5,
                                   sorted_classes=False)
    assert (np.diff(P.row_class) < 0).any()
    _run_case(drot, oracle, P, 300, "group lasso, unsorted labels")


def test_two_pass_group_lasso_is_bit_reproducible(drot):
    # the group norms of the general path are added up in a fixed order (rows of a class in chunks, then the
    # chunks): two runs give the same bits, on unsorted labels and on a class too long for the resident kernel
    cases = [drot_inputs.random_problem(700, 900, seed=79, reg_kind=2, lam=0.1, mu=0.08, num_classes=6, sorted_classes=False),
             _two_class_problem(1500, 333, 1100, seed=80)]
    for P in cases:
        solver = drot.Solver(P.m, P.n)
        _say(f"two-pass group lasso, run twice, {P.m}x{P.n}")
        runs = [pu.gpu_solve(solver, P, 150)[1:] for _ in range(2)]
        other = drot.Solver(P.m, P.n)
        runs.append(pu.gpu_solve(other, P, 150)[1:])
        for r in runs[1:]:
            for a, b in zip(runs[0], r):
                assert np.array_equal(a, b)


def test_group_lasso_without_quadratic_term(drot, oracle):
    P = drot_inputs.random_problem(200, 320, seed=78, reg_kind=2, lam=0.0, mu=0.05, num_classes=4)
    _run_case(drot, oracle, P, 300, "group lasso, lambda=0")


def test_explicit_stepsize(drot, oracle):
    P = drot_inputs.random_problem(120, 90, seed=5, reg_kind=1, lam=0.3)
    _run_case(drot, oracle, P, 400, "explicit stepsize", stepsize=0.02)


# ---------------------------------------------------------------------------------------------
# stopping rule, edge cases, reuse, streams, determinism, error paths
# ---------------------------------------------------------------------------------------------
def test_stops_at_first_passing_check(drot, oracle):
    P = drot_inputs.random_problem(90, 110, seed=9)
    solver = drot.Solver(P.m, P.n, check_every=10)
    _to_tolerance_against_the_oracle(drot, oracle, P, solver, 1e-4, 10, 50000, "stopping rule")
    # out of iterations before the tolerance: a status, not an error
    gres2, _, _, _ = pu.gpu_solve(solver, P, 20, tol=1e-9)
    assert gres2.code == drot.DROT_MAX_ITERS and not gres2.converged and gres2.iters == 20


def test_zero_iterations_returns_x0(drot):
    P = drot_inputs.random_problem(33, 47, seed=3)
    solver = drot.Solver(P.m, P.n)
    X = torch.full((P.m, P.n), 7.0, device="cuda:0")
    gres, Xg, _, _ = pu.gpu_solve(solver, P, 0, X_out=X)
    assert gres.iters == 0 and not Xg.any()


def test_handle_reuse_across_sizes_and_bitwise_determinism(drot, oracle):
    solver = drot.Solver(600, 800)
    big = drot_inputs.random_problem(600, 800, seed=11, reg_kind=1, lam=0.2)
    small = drot_inputs.random_problem(130, 77, seed=12)
    _say("handle reuse")
    _, Xa, _, _ = pu.gpu_solve(solver, big, 100)
    _run_case(drot, oracle, small, 100, "reuse small after big", solver=solver)
    _, Xb, _, _ = pu.gpu_solve(solver, big, 100)
    assert np.array_equal(Xa, Xb)  # fixed reduction order: bit-identical reruns
    with pytest.raises(drot.DrotError):
        pu.gpu_solve(solver, drot_inputs.random_problem(601, 10, seed=1), 1)  # larger than the handle


def test_runs_on_a_side_stream(drot, oracle):
    P = drot_inputs.random_problem(210, 190, seed=21, reg_kind=1, lam=0.4)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        _run_case(drot, oracle, P, 120, "side stream", stream=s)


def test_invalid_arguments_are_rejected(drot):
    P = drot_inputs.random_problem(10, 12, seed=2)
    solver = drot.Solver(P.m, P.n)
    C, p, q, _ = pu.to_dev(P)
    with pytest.raises(drot.DrotError):
        solver.solve(C, p, q, max_iters=-1)
    with pytest.raises(drot.DrotError):
        solver.solve(C, p, q, reg_kind=7)
    with pytest.raises(drot.DrotError):
        solver.solve(C, p, q, reg_kind=drot.DROT_REG_QUADRATIC, lam=-1.0)
    with pytest.raises(drot.DrotError):
        solver.solve(C, p, q, reg_kind=drot.DROT_REG_GROUP_LASSO, mu=0.1, num_classes=2)  # no labels
    with pytest.raises(drot.DrotError):
        solver.set_check_every(0)
    with pytest.raises(drot.DrotError):
        drot.Solver(0, 5)


def test_continuation_is_bit_identical_to_one_long_solve(drot):
    P = drot_inputs.random_problem(310, 530, seed=31, reg_kind=1, lam=0.2)
    solver = drot.Solver(P.m, P.n)
    _say("continuation")
    _, X_long, phi_long, _ = pu.gpu_solve(solver, P, 90)
    X = torch.empty((P.m, P.n), device="cuda:0")
    pu.gpu_solve(solver, P, 37, X_out=X)
    solver.set_continue(True)
    res, X_two, phi_two, _ = pu.gpu_solve(solver, P, 53, X_out=X)
    solver.set_continue(False)
    assert res.iters == 53
    assert np.array_equal(X_long, X_two) and np.array_equal(phi_long, phi_two)
    # profile mode reports a positive mean sweep time and does not change the result
    solver.set_profile(True)
    _, X_prof, _, _ = pu.gpu_solve(solver, P, 90)
    ms, cnt = solver.profile()
    solver.set_profile(False)
    assert cnt == 90 and ms > 0.0 and np.array_equal(X_prof, X_long)


def _two_class_problem(m, n, first_len, seed, lam=0.05, mu=0.05):
    P = drot_inputs.random_problem(m, n, seed=seed, reg_kind=2, lam=lam, mu=mu, num_classes=2)
    P.row_class = np.concatenate([np.zeros(first_len, np.int32), np.ones(m - first_len, np.int32)])
    return P


@pytest.mark.parametrize("m,first_len,label", [(1200, 900, "one class of 900 rows (16 rows per lane)"),
                                               (1500, 1100, "one class of 1100 rows (two-pass fallback)"),
                                               (700, 130, "classes of 130 and 570 rows")])
def test_group_lasso_class_sizes(drot, oracle, m, first_len, label):
    _run_case(drot, oracle, _two_class_problem(m, 333, first_len, seed=90 + m), 120, f"group lasso, {label}")


def test_group_lasso_both_paths_agree_with_the_oracle(drot, oracle):
    # sorted labels: the group-resident kernel by default, the two-pass path when forced
    P = drot_inputs.config(5, size=600)
    solver = drot.Solver(P.m, P.n)
    _run_case(drot, oracle, P, 200, "group lasso, group-resident path", solver=solver)
    solver.set_group_two_pass(True)
    _run_case(drot, oracle, P, 200, "group lasso, forced two-pass path", solver=solver)


def test_group_lasso_label_out_of_range_is_rejected(drot):
    P = drot_inputs.random_problem(40, 50, seed=8, reg_kind=2, lam=0.1, mu=0.1, num_classes=3)
    P.row_class = P.row_class.copy()
    P.row_class[7] = 3
    solver = drot.Solver(P.m, P.n)
    with pytest.raises(drot.DrotError):
        pu.gpu_solve(solver, P, 5)


@pytest.mark.parametrize("xoff,coff", [(1, 1), (2, 0), (3, 1), (0, 3)])
@pytest.mark.parametrize("m,n", [(70, 517), (131, 1022)])
def test_unaligned_base_pointers(drot, oracle, m, n, xoff, coff):
    # X_out and C handed over as views that start 4, 8 or 12 bytes past a 16-byte boundary
    P = drot_inputs.random_problem(m, n, seed=500 + 7 * xoff + coff, reg_kind=1, lam=0.3)
    _say(f"unaligned bases: X +{4 * xoff} B, C +{4 * coff} B, {m}x{n}")
    dev = torch.device("cuda:0")
    Cbuf = torch.zeros(m * n + 8, device=dev)
    Xbuf = torch.full((m * n + 8,), 3.0, device=dev)
    C = Cbuf[coff:coff + m * n].view(m, n)
    C.copy_(torch.from_numpy(P.C))
    X = Xbuf[xoff:xoff + m * n].view(m, n)
    assert X.data_ptr() % 16 == 4 * xoff and C.data_ptr() % 16 == 4 * coff
    solver = drot.Solver(m, n)
    p, q = torch.from_numpy(P.p).to(dev), torch.from_numpy(P.q).to(dev)
    res = solver.solve(C, p, q, reg_kind=P.reg_kind, lam=P.lam, max_iters=150, X_out=X)
    phi, varphi = solver.duals(m, n, dev)
    torch.cuda.synchronize()
    ores = pu.oracle_solve(oracle, P, 150)
    pu.assert_parity(oracle, P, res, X.cpu().numpy(), phi.cpu().numpy(), varphi.cpu().numpy(), ores, label="unaligned")
    # nothing outside the m*n window was touched
    assert (Xbuf[:xoff] == 3.0).all() and (Xbuf[xoff + m * n:] == 3.0).all()


@pytest.mark.parametrize("m,n,kind", [(333, 517, 1), (1000, 1000, 0), (2048, 300, 1)])
def test_fused_and_separate_vector_updates_give_the_same_bits(drot, oracle, m, n, kind):
    # small problems fold the eq. (6) update into the next sweep; both ways must agree exactly,
    # whatever the spacing of the residual checks
    P = drot_inputs.random_problem(m, n, seed=600 + m, reg_kind=kind, lam=0.2 if kind else 0.0)
    _say(f"fused vs separate update {m}x{n}")
    solver = drot.Solver(m, n)
    _, X_fused, phi_fused, varphi_fused = pu.gpu_solve(solver, P, 120)
    solver.set_fused_update(0)
    _, X_sep, phi_sep, varphi_sep = pu.gpu_solve(solver, P, 120)
    solver.set_fused_update(-1)
    assert np.array_equal(X_fused, X_sep) and np.array_equal(phi_fused, phi_sep) and np.array_equal(varphi_fused, varphi_sep)
    solver.set_check_every(7)
    res, X_chk, phi_chk, _ = pu.gpu_solve(solver, P, 120, tol=1e-12)  # checks every 7 iterations, never passes
    assert res.iters == 120 and np.array_equal(X_chk, X_fused) and np.array_equal(phi_chk, phi_fused)
    ores = pu.oracle_solve(oracle, P, 120)
    pu.assert_parity(oracle, P, res, X_chk, phi_chk, varphi_fused, ores, check_gap=False, label="fused")


@pytest.mark.parametrize("m,n,classes", [(333, 517, 3), (1500, 1000, 2), (1203, 2047, 5), (700, 90, 1)])
def test_group_lasso_fused_and_separate_vector_updates_give_the_same_bits(drot, oracle, m, n, classes):
    # the same for the group-resident group-lasso sweep (1, 2, 4 or 8 rows per thread)
    P = drot_inputs.random_problem(m, n, seed=650 + m, reg_kind=2, lam=0.1, mu=0.02, num_classes=classes)
    _say(f"group lasso, fused vs separate update {m}x{n}, {classes} classes")
    solver = drot.Solver(m, n)
    _, X_fused, phi_fused, varphi_fused = pu.gpu_solve(solver, P, 90)
    solver.set_fused_update(0)
    _, X_sep, phi_sep, varphi_sep = pu.gpu_solve(solver, P, 90)
    solver.set_fused_update(-1)
    assert np.array_equal(X_fused, X_sep) and np.array_equal(phi_fused, phi_sep) and np.array_equal(varphi_fused, varphi_sep)
    solver.set_check_every(7)
    res, X_chk, phi_chk, _ = pu.gpu_solve(solver, P, 90, tol=1e-12)
    assert res.iters == 90 and np.array_equal(X_chk, X_fused) and np.array_equal(phi_chk, phi_fused)
    # continuation in two halves lands on the same bits
    solver.set_check_every(100)
    X = torch.empty((P.m, P.n), device="cuda:0")
    pu.gpu_solve(solver, P, 41, X_out=X)
    solver.set_continue(True)
    _, X_two, phi_two, _ = pu.gpu_solve(solver, P, 49, X_out=X)
    solver.set_continue(False)
    assert np.array_equal(X_two, X_fused) and np.array_equal(phi_two, phi_fused)
    ores = pu.oracle_solve(oracle, P, 90)
    pu.assert_parity(oracle, P, res, X_chk, phi_chk, varphi_fused, ores, check_gap=False, label="fused group lasso")


@pytest.mark.parametrize("m,n", [(1, 1), (1, 256), (128, 1), (16, 256), (17, 33), (33, 200), (64, 255), (65, 130),
                                 (100, 100), (128, 256)])
@pytest.mark.parametrize("kind", [0, 1])
def test_resident_kernel_for_tiny_problems(drot, oracle, m, n, kind):
    # at most 128 x 256: one workgroup runs all the iterations between two residual checks in one
    # launch; same tolerance against the fp64 iteration, and the general path agrees with it
    P = drot_inputs.random_problem(m, n, seed=900 + 7 * m + n, reg_kind=kind, lam=0.4 if kind else 0.0)
    solver = drot.Solver(m, n, check_every=13)
    _say(f"resident {m}x{n} kind={kind}")
    K = 200
    tol = 1e-12 if m * n > 1 else 0.0  # checks every 13 iterations, never passes (1 x 1 is solved exactly)
    res, X_res, phi_res, varphi_res = pu.gpu_solve(solver, P, K, tol=tol)
    assert res.iters == K
    ores = pu.oracle_solve(oracle, P, K)
    pu.assert_parity(oracle, P, res, X_res, phi_res, varphi_res, ores, label="resident")
    solver.set_resident(0)
    res_gen, X_gen, phi_gen, varphi_gen = pu.gpu_solve(solver, P, K, tol=tol)
    solver.set_resident(-1)
    pu.assert_parity(oracle, P, res_gen, X_gen, phi_gen, varphi_gen, ores, label="general path, tiny problem")
    # continuation: 77 + 123 iterations land where 200 do (resident stretches are deterministic)
    X = torch.empty((m, n), device="cuda:0")
    pu.gpu_solve(solver, P, 77, X_out=X)
    solver.set_continue(True)
    _, X_two, phi_two, _ = pu.gpu_solve(solver, P, 123, X_out=X)
    solver.set_continue(False)
    _, X_one, phi_one, _ = pu.gpu_solve(solver, P, K)
    assert np.array_equal(X_two, X_one) and np.array_equal(phi_two, phi_one)


def test_resident_kernel_stops_at_the_same_check_as_the_oracle(drot, oracle):
    P = _config(1)
    solver = drot.Solver(P.m, P.n, check_every=10)
    _to_tolerance_against_the_oracle(drot, oracle, P, solver, 1e-5, 10, 100000, "resident, stopping rule at cfg1")


@pytest.mark.parametrize("K,check_every", [(150, 100), (151, 100), (37, 7)])
@pytest.mark.parametrize("kind", [0, 1])
def test_even_odd_cost_skipping(drot, oracle, K, check_every, kind):
    # C is read every second sweep (the first sweep of a pair stores X - rho*C); the result must
    # still match the fp64 iteration within the same tolerance, for odd and even iteration counts
    P = drot_inputs.random_problem(700, 1300, seed=700 + K, reg_kind=kind, lam=0.3 if kind else 0.0)
    solver = drot.Solver(P.m, P.n, check_every=check_every)
    solver.set_fused_update(0)  # the scheme applies to the unfused sweep
    solver.set_skip_cost(1)
    _say(f"even/odd K={K} check_every={check_every} kind={kind}")
    gres, Xg, phig, varphig = pu.gpu_solve(solver, P, K, tol=1e-12)  # residual checks active, never pass
    assert gres.iters == K
    ores = pu.oracle_solve(oracle, P, K)
    ratio = pu.assert_parity(oracle, P, gres, Xg, phig, varphig, ores, label="even/odd")
    _say(f"even/odd: plan error / scale = {ratio:.2e}")


def test_plain_scheme_full_size(drot, oracle):
    # 10000 x 10000 with every sweep on 32-row tiles reading all of C (the defaults at this size, the
    # zero-segment skipping and the screened sweeps, are what the cfg3 and cfg4 cases above cover)
    P = _config(3)
    solver = drot.Solver(P.m, P.n)
    solver.set_skip_cost(0)
    solver.set_skip_unchanged(0)
    _say("plain scheme at 10000 x 10000, K=25")
    gres, Xg, phig, varphig = pu.gpu_solve(solver, P, 25)
    ores = pu.oracle_solve(oracle, P, 25)
    pu.assert_parity(oracle, P, gres, Xg, phig, varphig, ores, label="plain cfg3")


@pytest.mark.parametrize("kind", [0, 1])
def test_sweep_schemes_beyond_the_fused_path(drot, oracle, kind):
    # 2300 rows are more than the fused small-problem path takes.  Default: plain sweeps on 128-row
    # tiles that neither read nor write back all-zero row segments; mode 1 of skip_cost: the even/odd
    # scheme; skip_unchanged 0: plain sweeps on 32-row tiles touching everything.  All three match
    # the fp64 iteration (they differ in rounding and summation order only).
    P = drot_inputs.random_problem(2300, 2500, seed=720 + kind, reg_kind=kind, lam=0.3 if kind else 0.0)
    solver = drot.Solver(P.m, P.n)
    _say(f"sweep schemes kind={kind}")
    ores = pu.oracle_solve(oracle, P, 120)
    res, X, phi, varphi = pu.gpu_solve(solver, P, 120)
    pu.assert_parity(oracle, P, res, X, phi, varphi, ores, label="zero segments skipped (default)")
    zero_segments = [X[:, j:j + 256].max(axis=1) == 0 for j in range(0, P.n, 256)]
    assert float(np.mean(zero_segments)) > 0.1  # the case really exercises the skipping
    solver.set_skip_cost(1)
    res, X, phi, varphi = pu.gpu_solve(solver, P, 120)
    pu.assert_parity(oracle, P, res, X, phi, varphi, ores, label="even/odd")
    solver.set_skip_cost(0)
    solver.set_skip_unchanged(0)
    res, X, phi, varphi = pu.gpu_solve(solver, P, 120)
    pu.assert_parity(oracle, P, res, X, phi, varphi, ores, label="plain, everything read and written")
    with pytest.raises(drot.DrotError):
        solver.set_skip_cost(2)
    with pytest.raises(drot.DrotError):
        solver.set_skip_unchanged(2)


@pytest.mark.parametrize("kind,m,n", [(0, 2300, 2500), (1, 2100, 3000), (0, 2049, 257), (1, 4000, 1500)])
def test_screening_changes_no_bit(drot, oracle, kind, m, n):
    # leaving out the reads of C that the bound certifies useless must give the very iterates of the
    # unscreened sweeps (same tiles, same summation order), over several refresh periods, across
    # residual checks, and with forbidden pairs (C = +inf) in the picture
    base = drot_inputs.random_problem(m, n, seed=1500 + m, reg_kind=kind, lam=0.05 if kind else 0.0)
    P = drot_inputs.with_entrywise_terms(base, seed=1501, forbid_frac=0.2 if kind else 0.0)
    solver = drot.Solver(m, n, check_every=37)
    _say(f"screening, bitwise, {m}x{n} kind={kind}")
    K = 300
    solver.set_screening(0)
    res_plain, X_plain, phi_plain, varphi_plain = pu.gpu_solve(solver, P, K, tol=1e-12)
    solver.set_screening(1)  # (automatic mode starts at 11.5 million entries)
    solver.set_profile(True)
    res, X, phi, varphi = pu.gpu_solve(solver, P, K, tol=1e-12)
    kinds = [kind_ for _, kind_ in solver.profile_sweeps()]
    solver.set_profile(False)
    assert 5 in kinds and 6 in kinds  # screened and refresh sweeps both ran
    assert np.array_equal(X, X_plain) and np.array_equal(phi, phi_plain) and np.array_equal(varphi, varphi_plain)
    ores = pu.oracle_solve(oracle, P, K)
    pu.assert_parity(oracle, P, res, X, phi, varphi, ores, label="screened")


def test_continuing_after_an_early_stop_screens_with_valid_bounds(drot):
    # A solve that converges at a check has one more stretch of sweeps queued behind the stop flag, which
    # do nothing -- a refresh of the screening bounds among them.  A continued solve must not take that
    # refresh for done: its iterates are those of the unscreened sweeps, bit for bit.
    P = drot_inputs.random_problem(2300, 2500, seed=1500 + 2300, reg_kind=1, lam=0.05)
    _say("continuation after convergence, screened against unscreened")
    outs = []
    for mode in (0, 1):
        solver = drot.Solver(P.m, P.n, check_every=25)
        solver.set_skip_cost(0)
        solver.set_screening(mode)
        # (host-ordered refreshes fall on sweeps 2, 10, 26, 58, 122, 250: the one at 122 sits in the stretch
        # queued behind a stop at iteration 100)
        probe, _, _, _ = pu.gpu_solve(solver, P, 100)
        tol = float(np.float32(max(probe.r_row, probe.r_col) * 1.0005))
        X = torch.empty((P.m, P.n), device="cuda:0")
        res, _, _, _ = pu.gpu_solve(solver, P, 5000, tol=tol, X_out=X)
        assert res.converged and res.iters <= 100, (res.iters, tol)
        stop = res.iters
        solver.set_continue(True)
        solver.set_profile(True)
        res2, X2, phi2, varphi2 = pu.gpu_solve(solver, P, 180, tol=1e-12, X_out=X)
        kinds = [k for _, k in solver.profile_sweeps()]
        solver.set_profile(False)
        assert res2.iters == 180
        if mode == 1:
            assert 5 in kinds or 7 in kinds, kinds  # the continued call does screen
        outs.append((stop, X2, phi2, varphi2))
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1:], outs[1][1:]):
        assert np.array_equal(a, b)


def test_zero_iterations_on_a_reused_padded_handle_reports_x0(drot):
    # n % 32 != 0: the library iterates on a padded copy of X; a solve with zero iterations on a handle
    # that still holds an earlier plan there must report X_0 = 0, not that plan
    P = drot_inputs.random_problem(300, 333, seed=61, reg_kind=1, lam=0.2)
    solver = drot.Solver(P.m, P.n)
    pu.gpu_solve(solver, P, 50)
    res, X0, _, _ = pu.gpu_solve(solver, P, 0)
    assert res.iters == 0 and not X0.any()
    assert res.objective == 0.0


def test_screening_across_calls_and_starts(drot, oracle):
    # the bounds outlive a call: a continued solve goes on screening with them, and lands on the
    # bits of one long unscreened solve; a warm start begins a new epoch; l1 weights just shift C
    base = drot_inputs.random_problem(2110, 2600, seed=1700, d=6, reg_kind=1, lam=0.02)
    P = drot_inputs.with_entrywise_terms(base, seed=1701, weight_scale=0.3)
    solver = drot.Solver(P.m, P.n, check_every=20)
    _say("screening across calls")
    solver.set_screening(0)
    res_plain, X_plain, phi_plain, varphi_plain = pu.gpu_solve(solver, P, 240, tol=1e-12)
    solver.set_screening(1)
    X = torch.empty((P.m, P.n), device="cuda:0")
    pu.gpu_solve(solver, P, 100, tol=1e-12, X_out=X)
    solver.set_continue(True)
    solver.set_profile(True)
    res, X_two, phi_two, varphi_two = pu.gpu_solve(solver, P, 140, tol=1e-12, X_out=X)
    kinds = [k for _, k in solver.profile_sweeps()]
    solver.set_profile(False)
    solver.set_continue(False)
    assert kinds[0] != 6 and (5 in kinds or 7 in kinds)  # no new epoch at the start of the continued call
    assert np.array_equal(X_two, X_plain) and np.array_equal(phi_two, phi_plain) and np.array_equal(varphi_two, varphi_plain)
    ores = pu.oracle_solve(oracle, P, 240)
    pu.assert_parity(oracle, P, res_plain, X_plain, phi_plain, varphi_plain, ores, label="screening, weights")
    # warm start from that point, screened against unscreened
    C, p, q, _ = pu.to_dev(P)
    W = torch.from_numpy(P.weights).to(C.device)
    outs = []
    for mode in (0, 1):
        solver.set_screening(mode)
        Xw = torch.from_numpy(X_plain).to(C.device)
        r = solver.solve(C, p, q, reg_kind=1, lam=P.lam, max_iters=120, X_out=Xw, weights=W,
                         phi0=torch.from_numpy(phi_plain).to(C.device), varphi0=torch.from_numpy(varphi_plain).to(C.device))
        outs.append(r.X.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("m,n", [(2049, 257), (2111, 300), (4000, 1000)])
def test_screening_on_ragged_shapes(drot, m, n):
    # last tile with 1 ... 63 rows, last column segment with 1 ... 255 columns, padded working copies
    P = drot_inputs.random_problem(m, n, seed=1800 + m, d=4, reg_kind=0)
    solver = drot.Solver(m, n, check_every=15)
    _say(f"screening, ragged {m}x{n}")
    outs = []
    for mode in (0, 1):
        solver.set_screening(mode)
        _, X, phi, varphi = pu.gpu_solve(solver, P, 200, tol=1e-12)
        outs.append((X, phi, varphi))
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("mode", [-1, 7])
def test_lean_screened_sweep_changes_no_bit(drot, oracle, mode):
    # wide rows: after the first status reports a sparse plan the solver moves to the one-wave-per-tile
    # screened sweep, which keeps its own refresh schedule and line flags for X; iterates must still be
    # those of the unscreened sweeps, bit for bit.  mode 7: new bounds at least every 7th sweep, so the
    # sweep's own renewals (everything read, nothing certified) come up many times.
    P = drot_inputs.random_problem(2100, 8192 + 40, seed=1600, d=8, reg_kind=1, lam=0.01)
    solver = drot.Solver(P.m, P.n, check_every=25)
    _say(f"lean screened sweep, bitwise, screening mode {mode}")
    K = 260
    solver.set_screening(0)
    _, X_plain, phi_plain, varphi_plain = pu.gpu_solve(solver, P, K, tol=1e-12)
    solver.set_screening(mode)
    solver.set_profile(True)
    res, X, phi, varphi = pu.gpu_solve(solver, P, K, tol=1e-12)
    kinds = [k for _, k in solver.profile_sweeps()]
    reads = solver.profile_reads()
    solver.set_profile(False)
    assert kinds.count(7) > 50, kinds
    lean_reads = [r for r, k in zip(reads, kinds) if k == 7]
    assert min(lean_reads) < 0.5  # it does leave most of C unread
    renewals = sum(1 for r in lean_reads if r > 0.999)
    assert renewals >= (len(lean_reads) // 10 if mode == 7 else 0), (renewals, len(lean_reads))  # (7 sweeps, then the renewal)
    assert np.array_equal(X, X_plain) and np.array_equal(phi, phi_plain) and np.array_equal(varphi, varphi_plain)
    ores = pu.oracle_solve(oracle, P, K)
    pu.assert_parity(oracle, P, res, X, phi, varphi, ores, label="lean screened")


def test_early_looks_at_the_density_start_the_lean_sweep_before_the_first_check(drot):
    # residual checks 1000 iterations apart: the host would learn how sparse the plan is after 2000
    # iterations; the extra status readings after 16, 32 and 64 iterations (no stopping test in them)
    # let it move to the lean sweep within the first 100 or so, and no bit of the result changes
    P = drot_inputs.random_problem(2100, 8192 + 40, seed=1600, d=8, reg_kind=1, lam=0.01)
    solver = drot.Solver(P.m, P.n, check_every=1000)
    _say("early density readings")
    K = 300
    solver.set_screening(0)
    _, X_plain, phi_plain, varphi_plain = pu.gpu_solve(solver, P, K, tol=1e-12)
    solver.set_screening(1)
    solver.set_profile(True)
    res, X, phi, varphi = pu.gpu_solve(solver, P, K, tol=1e-12)
    kinds = [k for _, k in solver.profile_sweeps()]
    solver.set_profile(False)
    assert res.iters == K and 7 in kinds[:200], kinds
    assert np.array_equal(X, X_plain) and np.array_equal(phi, phi_plain) and np.array_equal(varphi, varphi_plain)


def test_lean_sweep_does_not_depend_on_the_even_odd_option(drot):
    # the density readings that let the screened sweeps use their lean kernel are taken whether or not
    # the choice of the even/odd pairs is left to the library; cut into continued calls at odd places,
    # the solve lands on the same bits
    P = drot_inputs.random_problem(2100, 8192 + 40, seed=1601, d=6, reg_kind=0)
    solver = drot.Solver(P.m, P.n, check_every=50)
    solver.set_skip_cost(0)
    _say("lean sweep with the even/odd scheme switched off")
    K = 240
    solver.set_screening(0)
    _, X_plain, phi_plain, varphi_plain = pu.gpu_solve(solver, P, K, tol=1e-12)
    solver.set_screening(1)
    solver.set_profile(True)
    _, X, phi, varphi = pu.gpu_solve(solver, P, K, tol=1e-12)
    kinds = [k for _, k in solver.profile_sweeps()]
    solver.set_profile(False)
    assert kinds.count(7) > 20, kinds
    assert np.array_equal(X, X_plain) and np.array_equal(phi, phi_plain) and np.array_equal(varphi, varphi_plain)
    Xc = torch.empty((P.m, P.n), device="cuda:0")
    pu.gpu_solve(solver, P, 97, tol=1e-12, X_out=Xc)
    solver.set_continue(True)
    pu.gpu_solve(solver, P, 11, tol=1e-12, X_out=Xc)
    _, X3, phi3, varphi3 = pu.gpu_solve(solver, P, K - 108, tol=1e-12, X_out=Xc)
    solver.set_continue(False)
    assert np.array_equal(X3, X_plain) and np.array_equal(phi3, phi_plain) and np.array_equal(varphi3, varphi_plain)


def test_dense_plans_switch_to_the_even_odd_scheme(drot, oracle):
    # a strong quadratic term keeps the plan dense: the density the reduction reports must move the
    # solver from the zero-segment-skipping sweeps to the even/odd pairs (and the result must not care)
    P = drot_inputs.random_problem(2300, 1500, seed=740, reg_kind=1, lam=3000.0)
    solver = drot.Solver(P.m, P.n, check_every=10)
    solver.set_screening(1)
    solver.set_profile(True)
    _say("dense plan, adaptive scheme")
    res, X, phi, varphi = pu.gpu_solve(solver, P, 90)
    kinds = [kind for _, kind in solver.profile_sweeps()]
    solver.set_profile(False)
    nonzero_segments = [X[:, j:j + 256].max(axis=1) > 0 for j in range(0, P.n, 256)]
    assert float(np.mean(nonzero_segments)) > 0.9  # (a tenth of the entries is enough for that)
    # first stretch: the default scheme (sweep 1 has nothing to read, sweeps 2 and 10 record the bounds)
    assert kinds[:10] == [0, 6] + [5] * 7 + [6]
    assert set(kinds[30:]) == {1, 2}, kinds     # switched after the first status came back, one stretch late
    ores = pu.oracle_solve(oracle, P, 90)
    pu.assert_parity(oracle, P, res, X, phi, varphi, ores, label="dense plan")


@pytest.mark.parametrize("m,n,kind", [(200, 512, 1), (200, 500, 0), (1000, 1024, 1), (77, 300, 0)])
def test_skipping_zero_segments_changes_no_bit(drot, m, n, kind):
    # with the same tiles (fused update off keeps a small problem on the plain 32-row sweep) leaving out the
    # loads and stores of unchanged / all-zero row segments must give the very same X, phi, varphi,
    # from the dense first iterations to the sparse ones, also across a residual check and a continuation
    P = drot_inputs.random_problem(m, n, seed=5, reg_kind=kind, lam=0.01 if kind else 0.0)
    solver = drot.Solver(m, n, check_every=7)
    solver.set_fused_update(0)
    solver.set_resident(0)
    _say(f"zero-segment skipping, bitwise, {m}x{n}")
    for K in (1, 2, 9, 10, 30, 120):
        solver.set_skip_unchanged(0)
        _, X_all, phi_all, varphi_all = pu.gpu_solve(solver, P, K, tol=1e-12)
        solver.set_skip_unchanged(1)
        _, X_skip, phi_skip, varphi_skip = pu.gpu_solve(solver, P, K, tol=1e-12)
        assert np.array_equal(X_all, X_skip) and np.array_equal(phi_all, phi_skip) and np.array_equal(varphi_all, varphi_skip), K
    X = torch.empty((m, n), device="cuda:0")
    pu.gpu_solve(solver, P, 50, X_out=X)
    solver.set_continue(True)
    _, X_two, _, _ = pu.gpu_solve(solver, P, 70, X_out=X)
    solver.set_continue(False)
    assert np.array_equal(X_two, X_skip)


@pytest.mark.parametrize("m,n,classes", [(600, 2100, 3), (1203, 2600, 5), (1800, 2100, 2)])
def test_group_lasso_skipping_zero_lines_changes_no_bit(drot, m, n, classes):
    # group-resident group lasso beyond the fused small-problem path: leaving out the loads and stores
    # of the all-zero 128-byte lines of X (known from the strip row sums) must give the very same
    # iterates, from the dense first iterations on, across a residual check, a continuation and a
    # warm start (whose sums come in another layout and must not be taken for flags)
    P = drot_inputs.random_problem(m, n, seed=1900 + m, reg_kind=2, lam=0.01, mu=0.1, num_classes=classes)
    solver = drot.Solver(m, n, check_every=9)
    _say(f"group lasso, zero-line skipping, bitwise, {m}x{n}")
    outs = {}
    for mode in (0, 1):
        solver.set_skip_unchanged(mode)
        for K in (1, 2, 10, 60):
            outs[(mode, K)] = pu.gpu_solve(solver, P, K, tol=1e-12)[1:]
        X = torch.empty((m, n), device="cuda:0")
        pu.gpu_solve(solver, P, 25, X_out=X)
        solver.set_continue(True)
        outs[(mode, "two")] = pu.gpu_solve(solver, P, 35, X_out=X)[1:]
        solver.set_continue(False)
    for key in [k for k in outs if k[0] == 0]:
        for a, b in zip(outs[key], outs[(1, key[1])]):
            assert np.array_equal(a, b), key
    for a, b in zip(outs[(1, "two")], outs[(1, 60)]):
        assert np.array_equal(a, b)
    Xz = outs[(1, 60)][0]
    zero_lines = [Xz[:, j:j + 32].max(axis=1) == 0 for j in range(0, n, 32)]
    assert float(np.mean(zero_lines)) > 0.1  # the case really exercises the skipping


@pytest.mark.parametrize("terms", ["weights", "forbidden", "both"])
@pytest.mark.parametrize("kind,m,n", [(0, 90, 120), (1, 128, 256), (0, 333, 517), (1, 700, 90), (2, 333, 517),
                                      (0, 2300, 700), (1, 2300, 700), (2, 2300, 700)])
def test_weighted_l1_and_constrained_ot(drot, oracle, kind, m, n, terms):
    # the entrywise members of the regularizer class: l1 weights (the library solves on C + W) and
    # forbidden pairs (C = +inf), alone, together and on top of the quadratic and group-lasso terms;
    # the shapes cover the resident, the fused small-problem, the even/odd and the group-resident paths
    base = drot_inputs.random_problem(m, n, seed=1100 + m + kind, reg_kind=kind, lam=0.3 if kind else 0.0,
                                      mu=0.03 if kind == 2 else 0.0, num_classes=4)
    P = drot_inputs.with_entrywise_terms(base, seed=1200 + n, weight_scale=0.5 if terms != "forbidden" else 0.0,
                                         forbid_frac=0.3 if terms != "weights" else 0.0)
    gres, Xg, ores = _run_case(drot, oracle, P, 150, f"{terms} kind={kind} {m}x{n}")
    if P.forbidden is not None:
        assert not Xg[P.forbidden].any() and not ores.X[P.forbidden].any()
        assert np.isfinite(gres.objective) and np.isfinite(gres.gap)


def test_constrained_ot_on_the_two_pass_group_lasso_path(drot, oracle):
    base = drot_inputs.random_problem(300, 413, seed=1301, reg_kind=2, lam=0.1, mu=0.05, num_classes=5, sorted_classes=False)
    P = drot_inputs.with_entrywise_terms(base, seed=1302, weight_scale=0.4, forbid_frac=0.25)
    _run_case(drot, oracle, P, 200, "entrywise terms, unsorted labels")


@pytest.mark.parametrize("kind,m,n", [(0, 150, 210), (1, 2300, 700), (2, 600, 333), (1, 90, 120)])
def test_warm_start_matches_the_oracle_from_the_same_point(drot, oracle, kind, m, n):
    # start from an arbitrary (X_0, phi_0, varphi_0): Y_0 = X_0 + phi_0 1^T + 1 varphi_0^T, eq. (5)
    P = drot_inputs.random_problem(m, n, seed=800 + kind, reg_kind=kind, lam=0.2 if kind else 0.0,
                                   mu=0.04 if kind == 2 else 0.0, num_classes=4)
    rng = np.random.default_rng(801)
    X0 = (np.outer(P.p, P.q) * rng.uniform(0.0, 2.0, size=(m, n))).astype(np.float32)
    phi0 = rng.uniform(0.0, 1.0 / (m + n), size=m).astype(np.float32)
    varphi0 = rng.uniform(0.0, 1.0 / (m + n), size=n).astype(np.float32)
    K = 100
    _say(f"warm start kind={kind} {m}x{n}")
    dev = torch.device("cuda:0")
    C, p, q, rc = pu.to_dev(P)
    X = torch.from_numpy(X0).to(dev)
    solver = drot.Solver(m, n)
    res = solver.solve(C, p, q, reg_kind=kind, lam=P.lam, mu=P.mu, row_class=rc, num_classes=P.num_classes,
                       max_iters=K, X_out=X, phi0=torch.from_numpy(phi0).to(dev), varphi0=torch.from_numpy(varphi0).to(dev))
    phi, varphi = solver.duals(m, n, dev)
    torch.cuda.synchronize()
    ores = oracle.solve(P.C, P.p, P.q, rho=float(P.rho), reg_kind=kind, lam=float(np.float32(P.lam)),
                        mu=float(np.float32(P.mu)), row_class=P.row_class, num_classes=P.num_classes, max_iters=K,
                        X0=X0, phi0=phi0, varphi0=varphi0)
    assert res.iters == K
    pu.assert_parity(oracle, P, res, X.cpu().numpy(), phi.cpu().numpy(), varphi.cpu().numpy(), ores, label="warm start")


def test_warm_start_from_a_checkpoint_continues_the_solve(drot, oracle):
    # save (X, phi, varphi) after K1 iterations, restart from them on a fresh handle for K2 more
    P = drot_inputs.random_problem(400, 560, seed=810, reg_kind=1, lam=0.2)
    K1, K2 = 80, 70
    dev = torch.device("cuda:0")
    a = drot.Solver(P.m, P.n)
    _, X_full, phi_full, _ = pu.gpu_solve(a, P, K1 + K2)
    _, X_half, phi_half, varphi_half = pu.gpu_solve(a, P, K1)
    b = drot.Solver(P.m, P.n)
    C, p, q, _ = pu.to_dev(P)
    X = torch.from_numpy(X_half).to(dev)
    res = b.solve(C, p, q, reg_kind=1, lam=P.lam, max_iters=K2, X_out=X, phi0=torch.from_numpy(phi_half).to(dev),
                  varphi0=torch.from_numpy(varphi_half).to(dev))
    torch.cuda.synchronize()
    err = np.abs(X.cpu().numpy().astype(np.float64) - X_full).max() / np.abs(X_full).max()
    _say(f"checkpoint restart: difference / scale = {err:.2e}")
    assert res.iters == K2 and err <= 1e-5


@pytest.mark.parametrize("m,n,d,kind", [(150, 210, 3, 0), (333, 517, 10, 1), (1300, 900, 32, 1), (64, 256, 1, 0),
                                        (70, 300, 17, 1)])
def test_cost_from_point_clouds(drot, oracle, m, n, d, kind):
    # cost recomputed on the matrix cores in every sweep; the oracle gets the same cost formed in fp64
    P = drot_inputs.random_problem(m, n, seed=900 + d, d=d, reg_kind=kind, lam=0.3 if kind else 0.0)
    scale = np.float32(1.0 / P.cmax)
    P.C = oracle.sqdist_cost(P.xs, P.xt, float(scale))
    assert abs(float(P.C.max()) - 1.0) < 1e-3
    K = 150
    _say(f"point-cloud cost {m}x{n} d={d} kind={kind}")
    dev = torch.device("cuda:0")
    solver = drot.Solver(m, n)
    res = solver.solve_points(torch.from_numpy(P.xs).to(dev), torch.from_numpy(P.xt).to(dev), float(scale),
                              torch.from_numpy(P.p).to(dev), torch.from_numpy(P.q).to(dev), reg_kind=kind, lam=P.lam,
                              max_iters=K)
    phi, varphi = solver.duals(m, n, dev)
    torch.cuda.synchronize()
    ores = pu.oracle_solve(oracle, P, K)
    assert res.iters == K
    ratio = pu.assert_parity(oracle, P, res, res.X.cpu().numpy(), phi.cpu().numpy(), varphi.cpu().numpy(), ores,
                             label="points")
    _say(f"point-cloud cost: plan error / scale = {ratio:.2e}")


@pytest.mark.parametrize("m,n,d,kind", [(150, 210, 3, 0), (1300, 911, 12, 1), (2100, 8232, 8, 1)])
def test_warm_start_with_the_cost_from_point_clouds(drot, oracle, m, n, d, kind):
    # drot_solve_points_warm from an arbitrary (X_0, phi_0, varphi_0) against the oracle from the same point on the
    # same cost formed in fp64; and the same bits whether or not the sweeps skip and screen
    P = drot_inputs.random_problem(m, n, seed=950 + d, d=d, reg_kind=kind, lam=0.05 if kind else 0.0)
    scale = np.float32(1.0 / P.cmax)
    P.C = oracle.sqdist_cost(P.xs, P.xt, float(scale))
    rng = np.random.default_rng(951)
    X0 = (np.outer(P.p, P.q) * rng.uniform(0.0, 2.0, size=(m, n)) * (rng.uniform(size=(m, n)) < 0.3)).astype(np.float32)
    X0[:, n // 2:n // 2 + 300] = 0.0  # (whole row segments of zeros: the first sweep leaves them unread)
    phi0 = rng.uniform(0.0, 1.0 / (m + n), size=m).astype(np.float32)
    varphi0 = rng.uniform(0.0, 1.0 / (m + n), size=n).astype(np.float32)
    K = 120
    _say(f"warm start, point-cloud cost {m}x{n} d={d} kind={kind}")
    dev = torch.device("cuda:0")
    args = [torch.from_numpy(a).to(dev) for a in (P.xs, P.xt)]
    pq = [torch.from_numpy(a).to(dev) for a in (P.p, P.q)]
    start = dict(phi0=torch.from_numpy(phi0).to(dev), varphi0=torch.from_numpy(varphi0).to(dev))
    solver = drot.Solver(m, n, check_every=20)
    X = torch.from_numpy(X0).to(dev)
    res = solver.solve_points(*args, float(scale), *pq, reg_kind=kind, lam=P.lam, max_iters=K, X_out=X, **start)
    phi, varphi = solver.duals(m, n, dev)
    torch.cuda.synchronize()
    ores = oracle.solve(P.C, P.p, P.q, rho=float(P.rho), reg_kind=kind, lam=float(np.float32(P.lam)), max_iters=K,
                        X0=X0, phi0=phi0, varphi0=varphi0)
    assert res.iters == K
    pu.assert_parity(oracle, P, res, X.cpu().numpy(), phi.cpu().numpy(), varphi.cpu().numpy(), ores, label="points, warm")
    solver.set_skip_unchanged(0)
    X2 = torch.from_numpy(X0).to(dev)
    solver.solve_points(*args, float(scale), *pq, reg_kind=kind, lam=P.lam, max_iters=K, X_out=X2, **start)
    phi2, varphi2 = solver.duals(m, n, dev)
    assert torch.equal(X, X2) and torch.equal(phi, phi2) and torch.equal(varphi, varphi2)
    with pytest.raises(drot.DrotError):  # (both potentials or neither)
        solver.solve_points(*args, float(scale), *pq, max_iters=1, X_out=X2, phi0=start["phi0"])


@pytest.mark.parametrize("m,n,d,kind", [(333, 517, 3, 0), (1300, 2100, 6, 1), (900, 2300, 2, 0)])
def test_point_cloud_sweep_skipping_zero_segments_changes_no_bit(drot, m, n, d, kind):
    # the sweep that recomputes the cost also leaves all-zero row segments of X unread and unwritten;
    # same bits as with everything moved, from the first iterations on and across a continuation
    P = drot_inputs.random_problem(m, n, seed=2100 + d, d=d, reg_kind=kind, lam=0.02 if kind else 0.0)
    scale = float(np.float32(1.0 / P.cmax))
    dev = torch.device("cuda:0")
    xs, xt = torch.from_numpy(P.xs).to(dev), torch.from_numpy(P.xt).to(dev)
    p, q = torch.from_numpy(P.p).to(dev), torch.from_numpy(P.q).to(dev)
    solver = drot.Solver(m, n, check_every=13)
    _say(f"point-cloud cost, zero-segment skipping, bitwise, {m}x{n} d={d}")
    outs = {}
    for mode in (0, 1):
        solver.set_skip_unchanged(mode)
        for K in (1, 2, 40, 150):
            r = solver.solve_points(xs, xt, scale, p, q, reg_kind=kind, lam=P.lam, max_iters=K, tol=1e-12)
            phi, varphi = solver.duals(m, n, dev)
            outs[(mode, K)] = (r.X.cpu().numpy(), phi.cpu().numpy(), varphi.cpu().numpy())
    for K in (1, 2, 40, 150):
        for a, b in zip(outs[(0, K)], outs[(1, K)]):
            assert np.array_equal(a, b), K
    X = torch.empty((m, n), device=dev)
    solver.solve_points(xs, xt, scale, p, q, reg_kind=kind, lam=P.lam, max_iters=61, tol=1e-12, X_out=X)
    solver.set_continue(True)
    r = solver.solve_points(xs, xt, scale, p, q, reg_kind=kind, lam=P.lam, max_iters=89, tol=1e-12, X_out=X)
    solver.set_continue(False)
    assert np.array_equal(r.X.cpu().numpy(), outs[(1, 150)][0])
    Xz = outs[(1, 150)][0]
    zero_segments = [Xz[:, j:j + 256].max(axis=1) == 0 for j in range(0, n, 256)]
    assert float(np.mean(zero_segments)) > 0.02  # (some segments really are skipped)


@pytest.mark.parametrize("points", [False, True])
def test_screening_bounds_hold_over_long_stretches_without_renewal(drot, points):
    # thousands of sweeps, the bounds renewed only when the schedule's cap or the device's rent-or-buy rule says so
    # (hundreds of sweeps apart): the drift of varphi since the epoch grows large against the gaps the certificate
    # lives on, and the iterates must still be those of the sweeps that certify nothing, bit for bit
    m, n, K = 2100, 8232, 3000
    P = drot_inputs.random_problem(m, n, seed=2500 + int(points), d=8, reg_kind=1, lam=0.01)
    dev = torch.device("cuda:0")
    solver = drot.Solver(m, n, check_every=100)
    _say(f"long screened run, {'point clouds' if points else 'stored cost'}, {m}x{n}, K={K}")
    scale = np.float32(1.0 / P.cmax)
    xs, xt = torch.from_numpy(P.xs).to(dev), torch.from_numpy(P.xt).to(dev)
    C, p, q, _ = pu.to_dev(P)

    def run():
        if points:
            r = solver.solve_points(xs, xt, float(scale), p, q, reg_kind=1, lam=P.lam, max_iters=K, tol=1e-12)
        else:
            r = solver.solve(C, p, q, reg_kind=1, lam=P.lam, max_iters=K, tol=1e-12)
        phi, varphi = solver.duals(m, n, dev)
        return r.X.clone(), phi, varphi

    outs = []
    for screening in (0, 1):
        solver.set_screening(screening)
        solver.set_profile(bool(screening))
        outs.append(run())
        if screening:
            kinds = [r.kind for r in solver.profile_records()]
            assert sum(k in (7, 8) for k in kinds) >= 20, kinds  # (the lean sweeps took over within the 256 sweeps profiled)
    solver.set_profile(False)
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)


@pytest.mark.parametrize("m,n,d,kind", [(2100, 8232, 8, 1), (2300, 8192, 3, 0), (1531, 9999, 6, 1)])
def test_point_cloud_screening_changes_no_bit(drot, oracle, m, n, d, kind):
    # wide rows: once a status has reported a sparse plan the point-cloud variant forms the cost only for the row
    # segments no bound covers (gathered onto the matrix cores in blocks of 16 rows); the iterates must be those of its
    # full sweeps bit for bit, over several renewals of the bounds, across residual checks and a continuation, and they
    # must match the fp64 iteration on the cost formed in fp64
    P = drot_inputs.random_problem(m, n, seed=2300 + d, d=d, reg_kind=kind, lam=0.01 if kind else 0.0)
    scale = np.float32(1.0 / P.cmax)
    dev = torch.device("cuda:0")
    xs, xt = torch.from_numpy(P.xs).to(dev), torch.from_numpy(P.xt).to(dev)
    p, q = torch.from_numpy(P.p).to(dev), torch.from_numpy(P.q).to(dev)
    solver = drot.Solver(m, n, check_every=25)
    _say(f"point-cloud cost, screening, bitwise, {m}x{n} d={d}")
    K = 260

    def run(iters, X_out=None):
        r = solver.solve_points(xs, xt, float(scale), p, q, reg_kind=kind, lam=P.lam, max_iters=iters, tol=1e-12, X_out=X_out)
        phi, varphi = solver.duals(m, n, dev)
        return r, r.X.cpu().numpy(), phi.cpu().numpy(), varphi.cpu().numpy()

    solver.set_screening(0)
    _, X_plain, phi_plain, varphi_plain = run(K)
    solver.set_screening(1)
    solver.set_profile(True)
    res, X, phi, varphi = run(K)
    rec = solver.profile_records()
    solver.set_profile(False)
    kinds = [r.kind for r in rec]
    assert kinds.count(8) >= 10 and kinds.count(9) >= 3, kinds
    formed = [r.c_fraction for r in rec if r.kind == 8]
    assert min(formed) < 0.5  # it does leave most of the cost unformed
    assert np.array_equal(X, X_plain) and np.array_equal(phi, phi_plain) and np.array_equal(varphi, varphi_plain)
    Xc = torch.empty((m, n), device=dev)
    run(97, X_out=Xc)
    solver.set_continue(True)
    run(11, X_out=Xc)
    _, X3, phi3, varphi3 = run(K - 108, X_out=Xc)
    solver.set_continue(False)
    assert np.array_equal(X3, X_plain) and np.array_equal(phi3, phi_plain) and np.array_equal(varphi3, varphi_plain)
    P.C = oracle.sqdist_cost(P.xs, P.xt, float(scale))
    ores = pu.oracle_solve(oracle, P, K)
    ratio = pu.assert_parity(oracle, P, res, X, phi, varphi, ores, label="points, screened")
    _say(f"point-cloud cost, screened: plan error / scale = {ratio:.2e}; kinds {kinds.count(8)} screened, {kinds.count(9)} recording")


def test_ot_cost_gradient_is_the_plan(drot, oracle):
    # Section "Backpropagation through regularized OT-costs": grad_C OT_h(C) = X* when the
    # solution is unique (quadratic term).  Checked against the oracle's plan at convergence and
    # against central differences of the value along a random direction.
    # (lambda is large so that the plan varies smoothly over the finite-difference step: with a weak
    # quadratic term OT_h is nearly piecewise linear in C and a central difference straddles kinks)
    P = drot_inputs.random_problem(40, 50, seed=1400, reg_kind=1, lam=50.0)
    dev = torch.device("cuda:0")
    C, p, q, _ = pu.to_dev(P)
    solver = drot.Solver(P.m, P.n, check_every=50)
    kw = dict(reg_kind=1, lam=P.lam, max_iters=200000, tol=1e-7)
    _say("ot_cost value and gradient")
    Cg = C.clone().requires_grad_(True)
    value = drot.ot_cost(solver, Cg, p, q, **kw)
    (3.0 * value).backward()
    grad = Cg.grad.cpu().numpy() / 3.0
    ores = oracle.solve(P.C, P.p, P.q, rho=float(P.rho), reg_kind=1, lam=float(np.float32(P.lam)), max_iters=200000,
                        tol=1e-9, check_every=50)
    assert np.abs(grad - ores.X).max() <= 1e-4 * ores.X.max()
    t = oracle.objective_gap(P.C, ores.X, P.p, P.q, ores.phi, ores.varphi, float(P.rho), reg_kind=1,
                             lam=float(np.float32(P.lam)))
    assert abs(float(value.detach()) - t.objective) <= 1e-5 * abs(t.objective)
    E = torch.from_numpy(np.random.default_rng(1401).uniform(-1.0, 1.0, size=(P.m, P.n)).astype(np.float32)).to(dev)
    eps = 2e-3
    up = float(drot.ot_cost(solver, C + eps * E, p, q, **kw))
    down = float(drot.ot_cost(solver, C - eps * E, p, q, **kw))
    directional = float((E.cpu().numpy().astype(np.float64) * grad).sum())
    assert abs((up - down) / (2 * eps) - directional) <= 1e-2 * abs(directional)
