"""ctypes front end of the CPU oracle in drot_oracle.c -- TEST INFRASTRUCTURE, not the product.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.  It
marshals numpy arrays into the plain-C functions; all arithmetic is in the C file.  The oracle
takes the same fp32 C, p, q (and the same fp32 stepsize and weights) the GPU solver receives and
widens them to fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "drot_oracle.c")
_LIB = os.path.join(_HERE, "libdrot_oracle.so")

REG_NONE, REG_QUADRATIC, REG_GROUP_LASSO = 0, 1, 2

_c_double_p = ctypes.POINTER(ctypes.c_double)
_c_float_p = ctypes.POINTER(ctypes.c_float)
_c_int_p = ctypes.POINTER(ctypes.c_int)
_c_ubyte_p = ctypes.POINTER(ctypes.c_ubyte)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: the sums are the plain left-to-right ones)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_row_col_sums.argtypes = [_c_double_p, ctypes.c_int, ctypes.c_int, _c_double_p, _c_double_p]
        lib.oracle_row_col_sums.restype = None
        lib.oracle_project_marginals.argtypes = [_c_double_p, ctypes.c_int, ctypes.c_int, _c_double_p,
                                                 _c_double_p, _c_double_p, _c_double_p, _c_double_p]
        lib.oracle_project_marginals.restype = None
        lib.oracle_prox_h.argtypes = [_c_double_p, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                      ctypes.c_double, ctypes.c_double, _c_int_p, ctypes.c_int, _c_double_p]
        lib.oracle_prox_h.restype = None
        lib.oracle_prox_entrywise.argtypes = [_c_double_p, ctypes.c_int, ctypes.c_int, ctypes.c_double, _c_float_p,
                                              _c_ubyte_p]
        lib.oracle_prox_entrywise.restype = None
        lib.oracle_drot_solve.argtypes = [
            _c_float_p, _c_double_p, _c_double_p, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_int, ctypes.c_double, ctypes.c_double, _c_int_p, ctypes.c_int,
            _c_float_p, _c_ubyte_p,
            _c_double_p, _c_double_p, _c_double_p,
            ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            _c_double_p, _c_double_p, _c_double_p, _c_double_p, _c_double_p, _c_double_p, ctypes.c_int, _c_int_p]
        lib.oracle_drot_solve.restype = ctypes.c_int
        lib.oracle_objective_gap.argtypes = [
            _c_float_p, _c_double_p, _c_double_p, _c_double_p, _c_double_p, _c_double_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_double, ctypes.c_double,
            _c_int_p, ctypes.c_int, _c_float_p, _c_ubyte_p, _c_double_p]
        lib.oracle_objective_gap.restype = None
        lib.oracle_sqdist_cost.argtypes = [_c_float_p, _c_float_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_double, _c_float_p]
        lib.oracle_sqdist_cost.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _dp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_c_double_p)


def _ip(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_c_int_p)


def _fp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_c_float_p)


def _bp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_c_ubyte_p)


def _entrywise(weights, forbidden, shape):
    """fp32 weights and a uint8 mask, contiguous, of the cost's shape (or None)."""
    W = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
    S = None if forbidden is None else np.ascontiguousarray(np.asarray(forbidden) != 0, dtype=np.uint8)
    assert W is None or (W.shape == shape and (W >= 0).all())
    assert S is None or S.shape == shape
    return W, S


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    """Threads the oracle's parallel loops use (OpenMP's maximum for this process)."""
    return int(_load().oracle_num_threads())


def default_stepsize(m: int, n: int) -> float:
    """rho = 2/(m+n) (Stepsize selection), rounded to fp32 the way the GPU library rounds it."""
    return float(np.float32(2.0) / np.float32(m + n))


def initial_vectors(m: int, n: int):
    """phi_0, varphi_0 of the Initialization paragraph (X_0 = 0)."""
    phi0 = (1.0 + m / (m + n)) / (3.0 * (m + n))
    varphi0 = (1.0 + n / (m + n)) / (3.0 * (m + n))
    return np.full(m, phi0), np.full(n, varphi0)


def sqdist_cost(xs, xt, scale) -> np.ndarray:
    """C_ij = scale * ||xs_i - xt_j||^2 from fp32 point clouds (fp64 arithmetic, one rounding to fp32)."""
    xs = np.ascontiguousarray(xs, dtype=np.float32)
    xt = np.ascontiguousarray(xt, dtype=np.float32)
    m, d = xs.shape
    n = xt.shape[0]
    assert xt.shape[1] == d
    C = np.empty((m, n), dtype=np.float32)
    _load().oracle_sqdist_cost(xs.ctypes.data_as(_c_float_p), xt.ctypes.data_as(_c_float_p), m, n, d, float(scale),
                               C.ctypes.data_as(_c_float_p))
    return C


def project_marginals(V, p, q):
    """Closed-form projection onto {Z: Z1 = p, Z^T1 = q}; returns (Z, corr_row, corr_col)."""
    V = _f64(V)
    m, n = V.shape
    p, q = _f64(p), _f64(q)
    Z = np.empty_like(V)
    cr, cc = np.empty(m), np.empty(n)
    _load().oracle_project_marginals(_dp(V), m, n, _dp(p), _dp(q), _dp(Z), _dp(cr), _dp(cc))
    return Z, cr, cc


def prox_h(Xbar, rho, reg_kind=REG_NONE, lam=0.0, mu=0.0, row_class=None, num_classes=0):
    """prox_{rho h} of a nonnegative matrix (returns a new array)."""
    X = _f64(Xbar).copy()
    m, n = X.shape
    rc = None if row_class is None else np.ascontiguousarray(row_class, dtype=np.int32)
    scratch = np.empty(max(1, num_classes) * n)
    _load().oracle_prox_h(_dp(X), m, n, float(rho), int(reg_kind), float(lam), float(mu), _ip(rc),
                          int(num_classes), _dp(scratch))
    return X


@dataclass
class OracleResult:
    X: np.ndarray
    phi: np.ndarray
    varphi: np.ndarray
    iters: int
    res_row: np.ndarray  # ||X_k 1 - p||_2 for k = 1..iters
    res_col: np.ndarray
    Y: Optional[np.ndarray] = None
    gap_trace: Optional[np.ndarray] = None  # rows (k, objective, gap, dual residual) of the gap evaluations


def prox_entrywise(Xbar, rho, weights=None, forbidden=None):
    """Weighted-l1 soft-threshold and/or zeroing of the forbidden entries of a nonnegative matrix."""
    X = _f64(Xbar).copy()
    W, S = _entrywise(weights, forbidden, X.shape)
    _load().oracle_prox_entrywise(_dp(X), X.shape[0], X.shape[1], float(rho), _fp(W), _bp(S))
    return X


def solve(C, p, q, rho=None, reg_kind=REG_NONE, lam=0.0, mu=0.0, row_class=None, num_classes=0,
          max_iters=1000, tol=0.0, check_every=1, X0=None, phi0=None, varphi0=None,
          return_Y=False, weights=None, forbidden=None, gap_every=0, gap_tol=0.0) -> OracleResult:
    """Run the plain three-update iteration; see oracle_drot_solve in the C file."""
    C = np.ascontiguousarray(C, dtype=np.float32)
    m, n = C.shape
    W, S = _entrywise(weights, forbidden, (m, n))
    p, q = _f64(p), _f64(q)
    rho = default_stepsize(m, n) if rho is None or rho <= 0 else float(rho)
    d_phi0, d_varphi0 = initial_vectors(m, n)
    phi0 = d_phi0 if phi0 is None else _f64(phi0)
    varphi0 = d_varphi0 if varphi0 is None else _f64(varphi0)
    X0 = None if X0 is None else _f64(X0)
    rc = None
    if reg_kind == REG_GROUP_LASSO:
        rc = np.ascontiguousarray(row_class, dtype=np.int32)
        assert rc.shape == (m,) and rc.min() >= 0 and rc.max() < num_classes
    X = np.empty((m, n))
    Y = np.empty((m, n)) if return_Y else None
    phi, varphi = np.empty(m), np.empty(n)
    trace = np.zeros(2 * max(1, max_iters))
    if gap_tol > 0 and gap_every < 1:
        gap_every = 1  # (a gap tolerance needs the gap at the checks)
    gap_cap = max_iters // max(1, check_every * max(1, gap_every)) + 1 if gap_every >= 1 else 1
    gtrace = np.zeros(4 * gap_cap)
    glen = ctypes.c_int(0)
    it = _load().oracle_drot_solve(
        C.ctypes.data_as(_c_float_p), _dp(p), _dp(q), m, n, rho, int(reg_kind), float(lam), float(mu),
        _ip(rc), int(num_classes), _fp(W), _bp(S), _dp(X0), _dp(phi0), _dp(varphi0), int(max_iters), float(tol),
        int(check_every), int(gap_every), float(gap_tol), _dp(X), _dp(Y), _dp(phi), _dp(varphi), _dp(trace),
        _dp(gtrace), int(gap_cap), ctypes.byref(glen))
    if it < 0:
        raise MemoryError("oracle ran out of memory")
    tr = trace[: 2 * it].reshape(-1, 2)
    return OracleResult(X=X, phi=phi, varphi=varphi, iters=it, res_row=tr[:, 0].copy(), res_col=tr[:, 1].copy(), Y=Y,
                        gap_trace=gtrace[: 4 * glen.value].reshape(-1, 4).copy())


@dataclass
class GapTerms:
    cost: float  # <C, X>
    h: float  # h(X)
    dual_linear: float  # (p^T phi + q^T varphi)/rho
    h_conj: float  # h*(W) where finite
    gap: float
    dual_res: float

    @property
    def objective(self) -> float:
        return self.cost + self.h


def objective_gap(C, X, p, q, phi, varphi, rho, reg_kind=REG_NONE, lam=0.0, mu=0.0, row_class=None,
                  num_classes=0, weights=None, forbidden=None) -> GapTerms:
    C = np.ascontiguousarray(C, dtype=np.float32)
    m, n = C.shape
    W, S = _entrywise(weights, forbidden, (m, n))
    X, p, q, phi, varphi = _f64(X), _f64(p), _f64(q), _f64(phi), _f64(varphi)
    rc = None if row_class is None else np.ascontiguousarray(row_class, dtype=np.int32)
    out = np.zeros(6)
    _load().oracle_objective_gap(C.ctypes.data_as(_c_float_p), _dp(X), _dp(p), _dp(q), _dp(phi), _dp(varphi),
                                 m, n, float(rho), int(reg_kind), float(lam), float(mu), _ip(rc),
                                 int(num_classes), _fp(W), _bp(S), _dp(out))
    return GapTerms(*[float(v) for v in out])
