"""Thin ctypes binding of libdrot.so (C ABI declared in include/drot.h).

Argument marshalling only: every step of the solver runs inside the HIP library.  PyTorch is
used for device buffers and the stream handle.  There is no CPU fallback: if the library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdrot.so")

DROT_REG_NONE, DROT_REG_QUADRATIC, DROT_REG_GROUP_LASSO = 0, 1, 2
DROT_OK, DROT_MAX_ITERS = 0, 1
DROT_ERR_INVALID_ARG, DROT_ERR_ALLOC, DROT_ERR_HIP, DROT_ERR_NOT_INITIALIZED, DROT_ERR_TOO_LARGE = -1, -2, -3, -4, -5
DROT_STATIC_MAX_M = DROT_STATIC_MAX_N = 4096

# every symbol include/drot.h declares
EXPORTED_SYMBOLS = (
    "drot_create", "drot_destroy", "drot_set_option", "drot_set_gap_tolerance", "drot_get_checks", "drot_get_profile",
    "drot_solve", "drot_solve_points", "drot_solve_warm", "drot_solve_points_warm", "drot_solve_static", "drot_get_info", "drot_get_duals",
    "drot_strerror",
)

# drot_option
(DROT_OPT_CHECK_EVERY, DROT_OPT_COMPUTE_GAP, DROT_OPT_GAP_EVERY, DROT_OPT_CONTINUE, DROT_OPT_PROFILE,
 DROT_OPT_SKIP_UNCHANGED, DROT_OPT_SCREENING, DROT_OPT_SKIP_COST, DROT_OPT_FUSED_UPDATE, DROT_OPT_RESIDENT,
 DROT_OPT_GROUP_TWO_PASS, DROT_OPT_NONTEMPORAL) = range(12)


class drot_reg_params(ctypes.Structure):
    _fields_ = [("lambda_", ctypes.c_float), ("mu", ctypes.c_float), ("num_classes", ctypes.c_int),
                ("row_class", ctypes.c_void_p), ("weights", ctypes.c_void_p)]


class drot_info(ctypes.Structure):
    _fields_ = [("iters", ctypes.c_int), ("converged", ctypes.c_int), ("r_row", ctypes.c_float),
                ("r_col", ctypes.c_float), ("objective", ctypes.c_double), ("gap", ctypes.c_double),
                ("dual_res", ctypes.c_double)]


class drot_check(ctypes.Structure):
    _fields_ = [("iters", ctypes.c_int), ("gap_evaluated", ctypes.c_int), ("r_row", ctypes.c_float),
                ("r_col", ctypes.c_float), ("objective", ctypes.c_double), ("gap", ctypes.c_double),
                ("dual_res", ctypes.c_double)]


class drot_sweep_timing(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_float), ("kind", ctypes.c_int), ("c_fraction", ctypes.c_double),
                ("x_fraction", ctypes.c_double)]


class DrotError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} (code {code})")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libdrot.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2305_18483_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.drot_create.argtypes = [ctypes.POINTER(vp), ci, ci]
    lib.drot_destroy.argtypes = [vp]
    lib.drot_set_option.argtypes = [vp, ci, ci]
    lib.drot_set_gap_tolerance.argtypes = [vp, cf]
    lib.drot_get_checks.argtypes = [vp, ctypes.POINTER(drot_check), ci, ctypes.POINTER(ci)]
    lib.drot_get_profile.argtypes = [vp, ctypes.POINTER(drot_sweep_timing), ci, ctypes.POINTER(ci)]
    lib.drot_solve.argtypes = [vp, vp, vp, vp, ci, ci, cf, ci, ctypes.POINTER(drot_reg_params), ci, cf, vp, vp]
    lib.drot_solve_warm.argtypes = [vp, vp, vp, vp, ci, ci, cf, ci, ctypes.POINTER(drot_reg_params), ci, cf, vp, vp, vp, vp]
    lib.drot_solve_points.argtypes = [vp, vp, vp, ci, cf, vp, vp, ci, ci, cf, ci, ctypes.POINTER(drot_reg_params), ci, cf,
                                      vp, vp]
    lib.drot_solve_points_warm.argtypes = [vp, vp, vp, ci, cf, vp, vp, ci, ci, cf, ci, ctypes.POINTER(drot_reg_params), ci,
                                           cf, vp, vp, vp, vp]
    lib.drot_solve_static.argtypes = [vp, vp, vp, ci, ci, cf, ci, ctypes.POINTER(drot_reg_params), ci, cf, vp, vp, vp, vp, vp]
    lib.drot_get_info.argtypes = [vp, ctypes.POINTER(drot_info)]
    lib.drot_get_duals.argtypes = [vp, vp, vp]
    lib.drot_strerror.argtypes = [ci]
    lib.drot_strerror.restype = ctypes.c_char_p
    for name in EXPORTED_SYMBOLS:
        if name != "drot_strerror":
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().drot_strerror(int(code)).decode()


def _ptr(t: Optional[torch.Tensor], dtype, what: str):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous {dtype} tensor on the GPU")
    return ctypes.c_void_p(t.data_ptr())


@dataclass
class SolveResult:
    X: torch.Tensor
    code: int  # DROT_OK or DROT_MAX_ITERS
    iters: int
    converged: bool
    r_row: float
    r_col: float
    objective: float
    gap: float
    dual_res: float


def solve_static(C: torch.Tensor, p: torch.Tensor, q: torch.Tensor, X_out: torch.Tensor, *, stepsize: float = 0.0,
                 reg_kind: int = DROT_REG_NONE, lam: float = 0.0, max_iters: int = 1000, tol: float = 0.0,
                 phi_out: Optional[torch.Tensor] = None, varphi_out: Optional[torch.Tensor] = None,
                 info_out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> int:
    """drot_solve_static: enqueues the solve on the stream and returns at once, allocating nothing.  info_out: a
    device tensor of at least ctypes.sizeof(drot_info) bytes (uint8) that receives the drot_info block.  Returns
    the code of the call (DROT_OK: enqueued); raises DrotError on a negative one."""
    lib = load_library()
    m, n = C.shape
    params = drot_reg_params(float(lam), 0.0, 0, None, None)
    stream = stream if stream is not None else torch.cuda.current_stream(C.device)
    if info_out is not None and (not info_out.is_cuda or info_out.numel() * info_out.element_size() < ctypes.sizeof(drot_info)):
        raise ValueError("info_out must be a device buffer of at least sizeof(drot_info) bytes")
    rc = lib.drot_solve_static(_ptr(C, torch.float32, "C"), _ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"), int(m),
                               int(n), float(stepsize), int(reg_kind), ctypes.byref(params), int(max_iters), float(tol),
                               _ptr(X_out, torch.float32, "X_out"), _ptr(phi_out, torch.float32, "phi_out"),
                               _ptr(varphi_out, torch.float32, "varphi_out"),
                               None if info_out is None else ctypes.c_void_p(info_out.data_ptr()),
                               ctypes.c_void_p(stream.cuda_stream))
    if rc < 0:
        raise DrotError(rc, "drot_solve_static")
    return rc


def read_info(info_out: torch.Tensor) -> drot_info:
    """The drot_info block a drot_solve_static call left in a device buffer (synchronises with the device)."""
    raw = info_out.view(torch.uint8).cpu().numpy().tobytes()[:ctypes.sizeof(drot_info)]
    return drot_info.from_buffer_copy(raw)


class Solver:
    """Owns one drot_handle (workspace for problems up to max_m x max_n on the current device)."""

    def __init__(self, max_m: int, max_n: int, check_every: Optional[int] = None, compute_gap: Optional[bool] = None):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        rc = self._lib.drot_create(ctypes.byref(self._h), int(max_m), int(max_n))
        if rc != DROT_OK:
            self._h = ctypes.c_void_p()
            raise DrotError(rc, "drot_create")
        if check_every is not None:
            self.set_check_every(check_every)
        if compute_gap is not None:
            self.set_compute_gap(compute_gap)

    def set_option(self, option: int, value: int) -> None:
        rc = self._lib.drot_set_option(self._h, int(option), int(value))
        if rc != DROT_OK:
            raise DrotError(rc, f"drot_set_option({option}, {value})")

    # one name per option of include/drot.h
    def set_check_every(self, k: int) -> None:
        self.set_option(DROT_OPT_CHECK_EVERY, k)

    def set_compute_gap(self, enable: bool) -> None:
        self.set_option(DROT_OPT_COMPUTE_GAP, bool(enable))

    def set_gap_every(self, k: int) -> None:
        self.set_option(DROT_OPT_GAP_EVERY, k)

    def set_continue(self, enable: bool) -> None:
        self.set_option(DROT_OPT_CONTINUE, bool(enable))

    def set_profile(self, enable: bool) -> None:
        self.set_option(DROT_OPT_PROFILE, bool(enable))

    def set_skip_unchanged(self, mode: int) -> None:
        self.set_option(DROT_OPT_SKIP_UNCHANGED, mode)

    def set_screening(self, mode: int) -> None:
        self.set_option(DROT_OPT_SCREENING, mode)

    def set_skip_cost(self, mode: int) -> None:
        self.set_option(DROT_OPT_SKIP_COST, mode)

    def set_fused_update(self, mode: int) -> None:
        self.set_option(DROT_OPT_FUSED_UPDATE, mode)

    def set_resident(self, mode: int) -> None:
        self.set_option(DROT_OPT_RESIDENT, mode)

    def set_group_two_pass(self, enable: bool) -> None:
        self.set_option(DROT_OPT_GROUP_TWO_PASS, bool(enable))

    def set_nontemporal(self, mode: int) -> None:
        self.set_option(DROT_OPT_NONTEMPORAL, mode)

    def set_gap_tolerance(self, gap_tol: float) -> None:
        rc = self._lib.drot_set_gap_tolerance(self._h, float(gap_tol))
        if rc != DROT_OK:
            raise DrotError(rc, "drot_set_gap_tolerance")

    def checks(self) -> list:
        """The residual checks of the last solve (drot_get_checks), as drot_check records."""
        cnt = ctypes.c_int()
        cap = 4096
        buf = (drot_check * cap)()
        rc = self._lib.drot_get_checks(self._h, buf, cap, ctypes.byref(cnt))
        if rc != DROT_OK:
            raise DrotError(rc, "drot_get_checks")
        if cnt.value > cap:
            cap = cnt.value
            buf = (drot_check * cap)()
            self._lib.drot_get_checks(self._h, buf, cap, ctypes.byref(cnt))
        return [buf[e] for e in range(min(cnt.value, cap))]

    def profile_records(self) -> list:
        """drot_get_profile: one drot_sweep_timing per sweep the last solve timed in profile mode."""
        buf = (drot_sweep_timing * 256)()
        cnt = ctypes.c_int()
        rc = self._lib.drot_get_profile(self._h, buf, 256, ctypes.byref(cnt))
        if rc != DROT_OK:
            raise DrotError(rc, "drot_get_profile")
        return [buf[e] for e in range(min(cnt.value, 256))]

    def profile(self) -> tuple:
        """(mean sweep duration in ms, number of sweeps timed) of the last solve in profile mode."""
        rec = self.profile_records()
        return (sum(r.ms for r in rec) / len(rec) if rec else 0.0), len(rec)

    def profile_sweeps(self) -> list:
        """[(ms, kind)] of the sweeps the last solve timed in profile mode, in launch order."""
        return [(float(r.ms), int(r.kind)) for r in self.profile_records()]

    def profile_reads(self) -> list:
        """Fraction of the row segments of C that each timed sweep of the last solve read."""
        return [float(r.c_fraction) for r in self.profile_records()]

    def solve(self, C: torch.Tensor, p: torch.Tensor, q: torch.Tensor, *, stepsize: float = 0.0,
              reg_kind: int = DROT_REG_NONE, lam: float = 0.0, mu: float = 0.0,
              row_class: Optional[torch.Tensor] = None, num_classes: int = 0, max_iters: int = 1000,
              tol: float = 0.0, X_out: Optional[torch.Tensor] = None,
              stream: Optional[torch.cuda.Stream] = None, phi0: Optional[torch.Tensor] = None,
              varphi0: Optional[torch.Tensor] = None, weights: Optional[torch.Tensor] = None) -> SolveResult:
        """drot_solve (or drot_solve_warm when phi0 and varphi0 are given: X_out then holds X_0 on entry);
        raises DrotError on a negative return code.  weights: m x n device tensor of the weighted l1 term."""
        m, n = C.shape
        warm = phi0 is not None or varphi0 is not None
        if X_out is None:
            if warm:
                raise ValueError("a warm start needs X_out holding the starting plan")
            X_out = torch.empty_like(C)
        if weights is not None and tuple(weights.shape) != (m, n):
            raise ValueError("weights must have the shape of C")
        params = drot_reg_params(float(lam), float(mu), int(num_classes),
                                 None if row_class is None else row_class.data_ptr(),
                                 None if weights is None else _ptr(weights, torch.float32, "weights").value)
        if row_class is not None:
            _ptr(row_class, torch.int32, "row_class")
        stream = stream if stream is not None else torch.cuda.current_stream(C.device)
        common = (self._h, _ptr(C, torch.float32, "C"), _ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"),
                  int(m), int(n), float(stepsize), int(reg_kind), ctypes.byref(params), int(max_iters), float(tol),
                  _ptr(X_out, torch.float32, "X_out"))
        if warm:
            rc = self._lib.drot_solve_warm(*common, _ptr(phi0, torch.float32, "phi0"),
                                           _ptr(varphi0, torch.float32, "varphi0"), ctypes.c_void_p(stream.cuda_stream))
        else:
            rc = self._lib.drot_solve(*common, ctypes.c_void_p(stream.cuda_stream))
        if rc < 0:
            raise DrotError(rc, "drot_solve_warm" if warm else "drot_solve")
        info = self.info()
        return SolveResult(X=X_out, code=rc, iters=info.iters, converged=bool(info.converged), r_row=info.r_row,
                           r_col=info.r_col, objective=info.objective, gap=info.gap, dual_res=info.dual_res)

    def solve_points(self, xs: torch.Tensor, xt: torch.Tensor, cost_scale: float, p: torch.Tensor, q: torch.Tensor, *,
                     stepsize: float = 0.0, reg_kind: int = DROT_REG_NONE, lam: float = 0.0, max_iters: int = 1000,
                     tol: float = 0.0, X_out: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None, phi0: Optional[torch.Tensor] = None,
                     varphi0: Optional[torch.Tensor] = None) -> SolveResult:
        """drot_solve_points: cost recomputed from the point clouds xs (m x d), xt (n x d) in every sweep
        (drot_solve_points_warm when phi0 and varphi0 are given: X_out then holds X_0 on entry)."""
        m, d = xs.shape
        n = xt.shape[0]
        if xt.shape[1] != d:
            raise ValueError("xs and xt must have the same number of columns")
        warm = phi0 is not None or varphi0 is not None
        if X_out is None:
            if warm:
                raise ValueError("a warm start needs X_out holding the starting plan")
            X_out = torch.empty((m, n), dtype=torch.float32, device=xs.device)
        params = drot_reg_params(float(lam), 0.0, 0, None, None)
        stream = stream if stream is not None else torch.cuda.current_stream(xs.device)
        common = (self._h, _ptr(xs, torch.float32, "xs"), _ptr(xt, torch.float32, "xt"), int(d), float(cost_scale),
                  _ptr(p, torch.float32, "p"), _ptr(q, torch.float32, "q"), int(m), int(n), float(stepsize), int(reg_kind),
                  ctypes.byref(params), int(max_iters), float(tol), _ptr(X_out, torch.float32, "X_out"))
        if warm:
            rc = self._lib.drot_solve_points_warm(*common, _ptr(phi0, torch.float32, "phi0"),
                                                  _ptr(varphi0, torch.float32, "varphi0"), ctypes.c_void_p(stream.cuda_stream))
        else:
            rc = self._lib.drot_solve_points(*common, ctypes.c_void_p(stream.cuda_stream))
        if rc < 0:
            raise DrotError(rc, "drot_solve_points_warm" if warm else "drot_solve_points")
        info = self.info()
        return SolveResult(X=X_out, code=rc, iters=info.iters, converged=bool(info.converged), r_row=info.r_row,
                           r_col=info.r_col, objective=info.objective, gap=info.gap, dual_res=info.dual_res)

    def info(self) -> drot_info:
        out = drot_info()
        rc = self._lib.drot_get_info(self._h, ctypes.byref(out))
        if rc != DROT_OK:
            raise DrotError(rc, "drot_get_info")
        return out

    def duals(self, m: int, n: int, device) -> tuple:
        phi = torch.empty(m, dtype=torch.float32, device=device)
        varphi = torch.empty(n, dtype=torch.float32, device=device)
        rc = self._lib.drot_get_duals(self._h, ctypes.c_void_p(phi.data_ptr()), ctypes.c_void_p(varphi.data_ptr()))
        if rc != DROT_OK:
            raise DrotError(rc, "drot_get_duals")
        return phi, varphi

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.drot_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
