"""Seeded synthetic inputs for the regularized-OT solver (shared by tests, bench and oracle checks).

This module only *generates data*: point clouds, squared-Euclidean cost matrices normalised to
max(C) = 1 (the normalisation the paper's stepsize rule assumes, "Stepsize selection" paragraph),
marginal weights and row labels.  It holds none of the solver's arithmetic and imports neither the
HIP binding nor the oracle; both sides receive the very same fp32 arrays produced here.

The five configurations stand in for the paper's simulated data sets (Gaussian / uniform point
clouds with a squared-distance cost, Section "Numerical experiments"): the paper never states its
random parameters, so the shapes and distributions below are a synthetic recipe of the same form.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

REG_NONE = 0
REG_QUADRATIC = 1
REG_GROUP_LASSO = 2


@dataclass
class Problem:
    """One OT instance: everything a solver (GPU or oracle) needs, as fp32/int32 host arrays."""

    name: str
    C: np.ndarray  # (m, n) float32, row-major, max(C) == 1
    p: np.ndarray  # (m,) float32, sums to 1
    q: np.ndarray  # (n,) float32, sums to 1
    reg_kind: int = REG_NONE
    lam: float = 0.0  # weight of (lam/2)||X||_F^2
    mu: float = 0.0  # weight of the group-lasso term
    row_class: Optional[np.ndarray] = None  # (m,) int32 labels in [0, num_classes)
    num_classes: int = 0
    fixed_iters: int = 0  # K of the fixed-iteration run the configuration names
    tol: float = 0.0  # residual the configuration iterates to (0 = none named)
    xs: Optional[np.ndarray] = None  # (m, d) float32 source points
    xt: Optional[np.ndarray] = None  # (n, d) float32 target points
    cmax: float = 1.0  # the max squared distance C was divided by
    weights: Optional[np.ndarray] = None  # (m, n) float32 >= 0: weights of an added l1 term, or None
    forbidden: Optional[np.ndarray] = None  # (m, n) bool: pairs that must carry no mass (constrained OT), or None
    meta: dict = field(default_factory=dict)

    @property
    def m(self) -> int:
        return int(self.C.shape[0])

    @property
    def n(self) -> int:
        return int(self.C.shape[1])

    @property
    def rho(self) -> np.float32:
        """Default stepsize 2/(m+n), evaluated in fp32 exactly as the library evaluates it."""
        return np.float32(2.0) / np.float32(self.m + self.n)


def sqdist_cost(xs: np.ndarray, xt: np.ndarray, block: int = 4096):
    """C_ij = ||xs_i - xt_j||^2 / max_ij(.) in fp64, cast once to fp32. Returns (C, cmax)."""
    xs = np.asarray(xs, dtype=np.float64)
    xt = np.asarray(xt, dtype=np.float64)
    m, n = xs.shape[0], xt.shape[0]
    xs2 = np.einsum("id,id->i", xs, xs)
    xt2 = np.einsum("jd,jd->j", xt, xt)
    C = np.empty((m, n), dtype=np.float32)
    # first pass: the maximum, block by block (keeps the fp64 temporary small at 20000 x 20000)
    cmax = 0.0
    for i0 in range(0, m, block):
        i1 = min(i0 + block, m)
        D = xs2[i0:i1, None] + xt2[None, :] - 2.0 * (xs[i0:i1] @ xt.T)
        np.maximum(D, 0.0, out=D)
        cmax = max(cmax, float(D.max()))
    if cmax <= 0.0:
        cmax = 1.0
    for i0 in range(0, m, block):
        i1 = min(i0 + block, m)
        D = xs2[i0:i1, None] + xt2[None, :] - 2.0 * (xs[i0:i1] @ xt.T)
        np.maximum(D, 0.0, out=D)
        D /= cmax
        C[i0:i1] = D.astype(np.float32)
    return C, cmax


def uniform_weights(k: int) -> np.ndarray:
    return np.full(k, 1.0 / k, dtype=np.float64).astype(np.float32)


def random_weights(k: int, seed: int) -> np.ndarray:
    """iid Uniform(0.5, 1.5) weights normalised to sum 1."""
    w = np.random.default_rng(seed).uniform(0.5, 1.5, size=k)
    return (w / w.sum()).astype(np.float32)


def point_cloud_problem(name, xs, xt, p, q, **kw) -> Problem:
    C, cmax = sqdist_cost(xs, xt)
    return Problem(name=name, C=C, p=p, q=q, xs=np.asarray(xs, np.float32),
                   xt=np.asarray(xt, np.float32), cmax=cmax, **kw)


def config(k: int, size: Optional[int] = None) -> Problem:
    """Benchmark configuration k = 1..5 (the k-th entry of the configuration list, counted from one);
    `size` overrides m = n (same recipe, smaller)."""
    if k == 1:
        n = size or 100
        xs = np.random.default_rng(101).uniform(0.0, 1.0, size=(n, 2))
        xt = np.random.default_rng(102).uniform(0.0, 1.0, size=(n, 2))
        return point_cloud_problem("cfg1_unreg_100", xs, xt, uniform_weights(n), uniform_weights(n),
                                   reg_kind=REG_NONE, fixed_iters=2000)
    if k == 2:
        n = size or 1000
        xs = np.random.default_rng(201).normal(0.0, 1.0, size=(n, 10))
        xt = np.random.default_rng(202).normal(0.5, 1.0, size=(n, 10))
        return point_cloud_problem("cfg2_quad_1000", xs, xt, random_weights(n, 203), random_weights(n, 204),
                                   reg_kind=REG_QUADRATIC, lam=0.01, tol=1e-5)
    if k == 3:
        n = size or 10000
        xs = np.random.default_rng(301).uniform(0.0, 1.0, size=(n, 5))
        xt = np.random.default_rng(302).uniform(0.0, 1.0, size=(n, 5))
        return point_cloud_problem("cfg3_unreg_10000", xs, xt, uniform_weights(n), uniform_weights(n),
                                   reg_kind=REG_NONE, fixed_iters=1000, tol=1e-4)
    if k == 4:
        n = size or 20000
        xs = np.random.default_rng(401).normal(0.0, 1.0, size=(n, 32))
        xt = np.random.default_rng(402).normal(0.0, np.sqrt(2.0), size=(n, 32))
        return point_cloud_problem("cfg4_quad_20000", xs, xt, random_weights(n, 403), random_weights(n, 404),
                                   reg_kind=REG_QUADRATIC, lam=0.001, fixed_iters=500, tol=1e-4)
    if k == 5:
        n = size or 5000
        return domain_adaptation_problem(n_classes=10, per_class=n // 10, d=64, seed_src=501, seed_tgt=502,
                                         mu=0.1, lam=0.01, name="cfg5_grouplasso_5000")
    raise ValueError(f"no configuration {k}")


def domain_adaptation_problem(n_classes, per_class, d, seed_src, seed_tgt, mu, lam, name,
                              per_class_tgt: Optional[int] = None) -> Problem:
    """Labelled source / unlabelled target clouds shaped like the paper's domain-adaptation task.

    Source: n_classes Gaussians in R^d, means ~ N(0, 4I), unit covariance, rows sorted by class.
    Target: the same means, pushed through a per-class near-identity rotation (Q factor of
    I + 0.1 G_c) and shifted by one shared offset ~ N(0, I).  Groups are (source class, target column).
    """
    per_class_tgt = per_class_tgt or per_class
    rs = np.random.default_rng(seed_src)
    rt = np.random.default_rng(seed_tgt)
    means = rs.normal(0.0, 2.0, size=(n_classes, d))
    xs = np.concatenate([means[c] + rs.normal(0.0, 1.0, size=(per_class, d)) for c in range(n_classes)])
    offset = rt.normal(0.0, 1.0, size=d)
    parts = []
    for c in range(n_classes):
        Q, _ = np.linalg.qr(np.eye(d) + 0.1 * rt.normal(0.0, 1.0, size=(d, d)))
        z = means[c] + rt.normal(0.0, 1.0, size=(per_class_tgt, d))
        parts.append(z @ Q.T + offset)
    xt = np.concatenate(parts)
    m, n = xs.shape[0], xt.shape[0]
    row_class = np.repeat(np.arange(n_classes, dtype=np.int32), per_class)
    return point_cloud_problem(name, xs, xt, uniform_weights(m), uniform_weights(n),
                               reg_kind=REG_GROUP_LASSO, lam=lam, mu=mu, row_class=row_class,
                               num_classes=n_classes, fixed_iters=1000, tol=1e-4)


def random_problem(m: int, n: int, seed: int, d: int = 3, reg_kind: int = REG_NONE, lam: float = 0.0,
                   mu: float = 0.0, num_classes: int = 0, uniform: bool = False,
                   sorted_classes: bool = True) -> Problem:
    """Small general instance (m != n allowed, ragged sizes) for parity and edge-case tests."""
    rng = np.random.default_rng(seed)
    xs = rng.normal(0.0, 1.0, size=(m, d))
    xt = rng.normal(0.3, 1.2, size=(n, d))
    p = uniform_weights(m) if uniform else random_weights(m, seed + 1)
    q = uniform_weights(n) if uniform else random_weights(n, seed + 2)
    row_class = None
    if reg_kind == REG_GROUP_LASSO:
        num_classes = max(1, num_classes)
        row_class = rng.integers(0, num_classes, size=m).astype(np.int32)
        if sorted_classes:
            row_class = np.sort(row_class)
    return point_cloud_problem(f"rand_{m}x{n}_s{seed}", xs, xt, p, q, reg_kind=reg_kind, lam=lam, mu=mu,
                               row_class=row_class, num_classes=num_classes)


def with_entrywise_terms(P: Problem, seed: int, weight_scale: float = 0.0, forbid_frac: float = 0.0) -> Problem:
    """Copy of P with random l1 weights in [0, weight_scale) and/or a random set of forbidden pairs.

    Pairs with (i + j) % 3 == 0 are never forbidden, so every row and column keeps allowed partners.
    """
    rng = np.random.default_rng(seed)
    m, n = P.m, P.n
    W = rng.uniform(0.0, weight_scale, size=(m, n)).astype(np.float32) if weight_scale > 0 else None
    S = None
    if forbid_frac > 0:
        S = rng.uniform(size=(m, n)) < forbid_frac
        ii, jj = np.meshgrid(np.arange(m), np.arange(n), indexing="ij")
        S &= (ii + jj) % 3 != 0
    return dataclasses.replace(P, name=P.name + "_entrywise", weights=W, forbidden=S)
