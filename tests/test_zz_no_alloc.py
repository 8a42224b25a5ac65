"""drot_solve_static -- the entry point for callers that cannot allocate -- against drot_solve.

It runs out of a fixed array inside the library, enqueues everything and returns without waiting; its
X, phi, varphi and info block must be those of drot_solve on the same inputs: bit for bit where both run
the same sweeps, and within the bar of the parity tests in any case.  Two calls in a row share the
workspace, the second on a smaller problem.
"""
import sys

import numpy as np
import pytest
import torch

import drot_inputs

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-static] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def drot():
    import paper_2305_18483_amd as drot_mod

    drot_mod.load_library()
    assert torch.cuda.is_available()
    return drot_mod


def _both(drot, P, K, tol):
    dev = torch.device("cuda:0")
    C, p, q = (torch.from_numpy(a).to(dev) for a in (P.C, P.p, P.q))
    assert C.data_ptr() % 128 == 0
    solver = drot.Solver(P.m, P.n)
    ref = solver.solve(C, p, q, reg_kind=P.reg_kind, lam=P.lam, max_iters=K, tol=tol)
    phi_ref, varphi_ref = solver.duals(P.m, P.n, dev)
    X = torch.full((P.m, P.n), 7.0, device=dev)
    phi, varphi = torch.empty(P.m, device=dev), torch.empty(P.n, device=dev)
    info = torch.zeros(64, dtype=torch.uint8, device=dev)
    rc = drot.solve_static(C, p, q, X, reg_kind=P.reg_kind, lam=P.lam, max_iters=K, tol=tol, phi_out=phi,
                           varphi_out=varphi, info_out=info)
    assert rc == drot.DROT_OK
    torch.cuda.synchronize()
    got = drot.read_info(info)
    return ref, phi_ref, varphi_ref, X, phi, varphi, got


def _compare(ref, phi_ref, varphi_ref, X, phi, varphi, got, label):
    scale = float(ref.X.max())
    err = float((X - ref.X).abs().max())
    _say(f"{label}: iters {got.iters} (reference {ref.iters}), converged {got.converged}, max |X - X_ref| / scale = {err / scale:.1e}")
    assert got.iters == ref.iters and bool(got.converged) == ref.converged
    assert err <= 1e-4 * scale
    assert float((phi - phi_ref).abs().max()) <= 1e-4 * float(phi_ref.abs().max())
    assert float((varphi - varphi_ref).abs().max()) <= 1e-4 * float(varphi_ref.abs().max())
    assert abs(got.r_row - ref.r_row) <= 1e-6 and abs(got.r_col - ref.r_col) <= 1e-6
    assert abs(got.objective - ref.objective) <= 1e-5 * abs(ref.objective)
    assert abs(got.gap - ref.gap) <= 2e-5 * max(abs(ref.objective), abs(ref.gap))
    # the sweeps are the same ones here (sparse plans never take the even/odd pairs): the very same bits
    assert torch.equal(X, ref.X) and torch.equal(phi, phi_ref) and torch.equal(varphi, varphi_ref)


def test_static_entry_point_matches_drot_solve_on_two_calls_in_a_row(drot):
    # first a problem on the 64-row tiles with screening (12.3 million entries), then, in the same
    # workspace, smaller ones: the fused small-problem sweep with a tolerance that stops it early, and
    # the one-workgroup resident kernel
    big = drot_inputs.random_problem(3500, 3520, seed=5100, d=5, reg_kind=1, lam=0.02)
    small = drot_inputs.random_problem(1000, 1024, seed=5101, reg_kind=1, lam=0.3)
    tiny = drot_inputs.random_problem(100, 96, seed=5102, reg_kind=0)
    _say("3500 x 3520, 260 iterations")
    _compare(*_both(drot, big, 260, 0.0), "big")
    _say("1000 x 1024, to a residual of 1e-3")
    out = _both(drot, small, 20000, 1e-3)
    assert out[0].converged and out[0].iters < 20000
    _compare(*out, "small")
    _say("100 x 96, 500 iterations")
    _compare(*_both(drot, tiny, 500, 0.0), "tiny")
    _say("3500 x 3520 again, 130 iterations")
    _compare(*_both(drot, big, 130, 0.0), "big again")


def test_static_entry_point_rejects_what_it_cannot_hold(drot):
    dev = torch.device("cuda:0")
    m = n = 4128
    C = torch.zeros((m, n), device=dev)
    p = torch.full((m,), 1.0 / m, device=dev)
    X = torch.empty_like(C)
    with pytest.raises(drot.DrotError) as e:
        drot.solve_static(C, p, p, X, max_iters=1)
    assert e.value.code == drot.binding.DROT_ERR_TOO_LARGE and "workspace" in str(e.value)
    # rows off the 128-byte lines would need padded copies, which are allocations
    C2 = torch.zeros((64, 100), device=dev)
    p2, q2 = torch.full((64,), 1.0 / 64, device=dev), torch.full((100,), 0.01, device=dev)
    with pytest.raises(drot.DrotError) as e:
        drot.solve_static(C2, p2, q2, torch.empty_like(C2), max_iters=1)
    assert e.value.code == drot.binding.DROT_ERR_INVALID_ARG
