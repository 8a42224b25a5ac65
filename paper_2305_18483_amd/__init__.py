"""MI355X-native Douglas-Rachford solver for regularized discrete optimal transport.

The product is the HIP library built from csrc/ (C ABI in include/drot.h); this package is its
thin Python binding.  Nothing here computes on the CPU.
"""
from .autograd import ot_cost
from .binding import (DROT_MAX_ITERS, DROT_OK, DROT_REG_GROUP_LASSO, DROT_REG_NONE, DROT_REG_QUADRATIC, DrotError,
                      Solver, SolveResult, load_library, read_info, solve_static, strerror)

__all__ = ["ot_cost", "Solver", "SolveResult", "DrotError", "load_library", "strerror", "solve_static", "read_info", "DROT_OK", "DROT_MAX_ITERS",
           "DROT_REG_NONE", "DROT_REG_QUADRATIC", "DROT_REG_GROUP_LASSO"]
