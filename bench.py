#!/usr/bin/env python3
"""Benchmark of the Douglas-Rachford OT solver on one MI355X.

A step is one iteration of the method: the sweep over the m x n plan (prox of nonnegativity, cost
and regularizer fused with the row/column sums), the O(m+n) vector update, and the periodic
residual test where one is scheduled.  Default workload: the quadratically regularized
20000 x 20000 configuration (C and X 1.6 GB each, resident in HBM before timing starts).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--size N]

prints one JSON line.  `value` is K iterations timed after a cold start of W iterations.  The solver
is deterministic, so the same W + K iterations are then run once more in profile mode (HIP events on
the launch stream around every sweep; the kernels count what they read): `roofline` describes the
dominant sweep kernel of exactly the timed iterations.  The leg `steady_state` does the same with a
fixed warm-up of 200 and 500 timed iterations, whatever --steps/--warmup say: a cold start is dense
for its first dozens of iterations and sparse afterwards, and the two regimes run different kernels.

Further legs: the same 500 iterations with the screening off, with the even/odd scheme of the paper's
GPU appendix, and with every byte moved (12 bytes per element: the dense streaming rate of the sweep
kernel); the cost recomputed from the point clouds; time to a residual of 1e-4 and to a relative
duality gap of 1e-3, each checked in fp64 by code that shares nothing with the library; sizes n and
n - 1 side by side (alignment); the CPU oracle on a bounded sample, on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
MFMA_F32_PEAK_TFLOPS = 157.3
SEG_COLS = 256             # columns of a row segment, the unit of the zero-segment skipping
STEADY_WARMUP, STEADY_STEPS = 200, 500
ALIGN_STEPS = 2000  # (one copy of X out of the padded working copy per call: 1 % of 600 iterations at n = 10239, 0.3 % of 2000)
KERNEL_NAMES = {
    0: "sweep_kernel (reads X and C, stores X)",
    1: "sweep_kernel, first of a pair (reads X and C, stores X - rho*C)",
    2: "sweep_kernel, second of a pair (reads X - rho*C, stores X)",
    3: "resident_kernel (X and C stay in registers; the time is per iteration)",
    4: "sweep_kernel on 64-row tiles (reads C; reads and stores only the nonzero row segments of X)",
    5: "screened_sweep_kernel (reads C only where a bound does not certify zeros; nonzero row segments of X)",
    6: "screened_sweep_kernel, refresh (reads all of C, records the bounds)",
    7: "screened_lean_kernel (one wave per 64 x 256 tile; reads C only where a bound does not certify zeros)"}
# counter-measured HBM traffic per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of
# known size), written by profiles/ for one fixed, deterministic run; attached only to that very run
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_steady_state.json")


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=STEADY_STEPS)
    ap.add_argument("--warmup", type=int, default=STEADY_WARMUP,
                    help="untimed cold-start iterations (the support of the plan settles within the first 100 or so)")
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1..5 (default 4: 20000 x 20000)")
    ap.add_argument("--size", type=int, default=0, help="override m = n (same recipe)")
    ap.add_argument("--tol", type=float, default=1e-4, help="residual of the time-to-tolerance leg")
    ap.add_argument("--gap-tol", type=float, default=1e-3, help="relative duality gap of the time-to-gap leg")
    ap.add_argument("--tol-max-iters", type=int, default=400000)
    ap.add_argument("--check-every", type=int, default=100)
    ap.add_argument("--nontemporal", type=int, default=-1, help="-1: library default, 0/1: force off/on")
    ap.add_argument("--skip-cost", type=int, default=-1,
                    help="even/odd scheme (C read every second sweep): -1 library default, 0 never, 1 wherever it applies")
    ap.add_argument("--skip-unchanged", type=int, default=-1, help="zero-segment skipping: -1/1 on, 0 off")
    ap.add_argument("--only", default="", help="comma-separated legs to run besides the main measurement "
                    "(steady,variants,points,tol,gap,alignment,cpu); default: all")
    ap.add_argument("--cpu-iters", type=int, default=0, help="oracle iterations to time (0: sized for ~20 s)")
    ap.add_argument("--calibrate", action="store_true",
                    help="only run a device copy of 1 GiB five times (to scale the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    legs = set(args.only.split(",")) if args.only else {"steady", "variants", "points", "tol", "gap", "alignment", "cpu"}

    import numpy as np
    import torch

    if args.calibrate:
        # a plain elementwise kernel of known size: reads 1 GiB, writes 1 GiB per launch
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(5):
            torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch.add(a, 1.0, out=b), 2^28 floats: 1 GiB read and 1 GiB written per launch, 5 launches"}))
        return 0

    import drot_checks
    import drot_inputs
    import paper_2305_18483_amd as drot

    drot.load_library()  # raises if the HIP library has not been built: there is no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")

    t0 = time.time()
    P = drot_inputs.config(args.config, size=args.size or None)
    m, n = P.m, P.n
    nseg = (n + SEG_COLS - 1) // SEG_COLS
    log(f"workload {P.name}: m={m} n={n} reg_kind={P.reg_kind} lambda={P.lam} mu={P.mu} (generated in {time.time() - t0:.1f} s)")
    C = torch.from_numpy(P.C).to(dev)
    p = torch.from_numpy(P.p).to(dev)
    q = torch.from_numpy(P.q).to(dev)
    rc = None if P.row_class is None else torch.from_numpy(P.row_class).to(dev)
    X = torch.empty_like(C)
    kw = dict(reg_kind=P.reg_kind, lam=P.lam, mu=P.mu, row_class=rc, num_classes=P.num_classes, X_out=X)
    solver = drot.Solver(m, n, check_every=args.check_every, compute_gap=False)

    def defaults():
        solver.set_nontemporal(args.nontemporal)
        solver.set_skip_cost(args.skip_cost)
        solver.set_skip_unchanged(args.skip_unchanged)
        solver.set_screening(-1)
        solver.set_continue(False)

    defaults()
    torch.cuda.synchronize()

    def nonzero_line_fraction():
        """Fraction of the 128-byte lines (32 columns of one row) of X that hold a nonzero."""
        nz = total = 0
        for j0 in range(0, n, 32):
            nz += int((X[:, j0:j0 + 32] != 0).any(dim=1).sum().item())
            total += m
        return nz / total

    def sweep_bytes(rec, x_before, line_frac, skipping=None):
        """Algorithmic bytes of one profiled sweep: what it must move for the plan at hand.

        C on the fraction of its row segments the kernel read (counted by the kernel); X read on the row
        segments that held a nonzero before the sweep and written on those that did or do now (counted
        by the vector updates; the lean kernel moves 128-byte lines instead of row segments: priced from
        the plan the run ends with); per row segment the old and new sums, the bound, the line flags;
        the column sums per tile row.
        """
        kind, c, x_after = rec.kind, rec.c_fraction, rec.x_fraction
        mn = float(m) * n
        if skipping is None:
            skipping = args.skip_unchanged != 0
        if kind in (0, 1, 3):
            if kind == 0 and P.reg_kind == 2 and skipping:
                # group-resident group lasso: all of C; of X the nonzero 128-byte lines; two sums per line
                return (4.0 + 8.0 * line_frac) * mn + 8.0 * m * ((n + 31) // 32) + 4.0 * n * max(1, P.num_classes)
            return 12.0 * mn
        if kind == 2:
            return 8.0 * mn
        xb = x_after if x_before is None or x_before < 0 else x_before
        xw = max(xb, x_after)
        if kind == 7:
            # per row segment: the three parts of the bound (4 + 4 + 1 B) and the line flags read; the new sum and
            # flags written only where the bound did not certify zeros (the rest is unchanged in memory)
            return 4.0 * c * mn + 8.0 * line_frac * mn + (10.0 + 5.0 * c) * m * nseg + 4.0 * n * ((m + 255) // 256)
        per_segment = 8.0 if kind == 4 else 17.0  # (old and new sum; screened: also the three parts of the bound)
        return 4.0 * c * mn + 4.0 * (xb + xw) * mn + per_segment * m * nseg + 4.0 * n * ((m + 63) // 64)

    def measure(W, K, label):
        """Cold start of W iterations, K timed; then the same W + K once more in profile mode."""
        defaults()
        solver.solve(C, p, q, max_iters=W, **kw)
        solver.set_continue(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        res = solver.solve(C, p, q, max_iters=K, **kw)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        assert res.iters == K
        checksum = (float(X.sum(dtype=torch.float64)), float(X.max()), int((X != 0).sum()))
        # the same iterations again, profiled (the first 256 of the K)
        solver.set_continue(False)
        solver.solve(C, p, q, max_iters=W, **kw)
        solver.set_continue(True)
        solver.set_profile(True)
        solver.solve(C, p, q, max_iters=K, **kw)
        recs = solver.profile_records()
        solver.set_profile(False)
        solver.set_continue(False)
        again = (float(X.sum(dtype=torch.float64)), float(X.max()), int((X != 0).sum()))
        assert again == checksum, f"the profiled rerun did not reproduce the timed run: {again} vs {checksum}"
        line_frac = nonzero_line_fraction() if (any(r.kind == 7 for r in recs) or P.reg_kind == 2) else 0.0
        per_kind = {}
        x_before = None
        for r in recs:
            b = sweep_bytes(r, x_before, line_frac)
            e = per_kind.setdefault(r.kind, {"ms": 0.0, "bytes": 0.0, "n": 0, "c": 0.0, "x": 0.0})
            e["ms"] += r.ms
            e["bytes"] += b
            e["n"] += 1
            e["c"] += r.c_fraction
            e["x"] += max(r.x_fraction, 0.0)
            x_before = r.x_fraction
        entries = {}
        for kind, e in per_kind.items():
            gbs = e["bytes"] / (e["ms"] * 1e-3) / 1e9
            entries[kind] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "kernel": KERNEL_NAMES[kind]
                             if not (kind == 0 and P.reg_kind == 2) else "gl_slab_kernel / group-lasso sweep",
                             "kernel_ms": round(e["ms"] / e["n"], 5), "launches_timed": e["n"],
                             "algorithmic_bytes": e["bytes"] / e["n"],
                             "c_row_segments_read_fraction": round(e["c"] / e["n"], 5),
                             "nonzero_row_segment_fraction": round(e["x"] / e["n"], 5)}
            if kind in (4, 5, 6, 7):
                entries[kind]["dense_model_gbs"] = round(12.0 * m * n / (e["ms"] / e["n"] * 1e-3) / 1e9, 1)
        dominant = max(per_kind, key=lambda k: per_kind[k]["ms"])
        roof = dict(entries[dominant])
        roof["other_kernels"] = [entries[k] for k in sorted(entries) if k != dominant]
        roof["bytes_model"] = ("per launch: 4 B x the row segments of C read (counted by the kernel) + X read on the row segments "
                               "nonzero before and written on those nonzero before or after (counted by the vector updates; lean "
                               "kernel: the nonzero 128-byte lines of the final plan) + 8-17 B per row segment (sums, bounds, line "
                               "flags; lean kernel: 10 B read, 5 B written where no bound certified zeros) + column sums; dense sweeps 12 (8 without C) B per element; dense_model_gbs prices the "
                               "launch at 12 B per element")
        if line_frac:
            roof["nonzero_line_fraction"] = round(line_frac, 6)
        sweep_ms = sum(e["ms"] for e in per_kind.values()) / max(1, len(recs))
        total_bytes = sum(e["bytes"] for e in per_kind.values()) / max(1, len(recs))
        ms_per_step = elapsed / K * 1e3
        out = {"value": round(K / elapsed, 2), "unit": "iterations/s", "warmup": W, "steps": K,
               "ms_per_step": round(ms_per_step, 5), "roofline": roof,
               "iteration_breakdown_ms": {"sweep_kernel_mean": round(sweep_ms, 5),
                                          "vector_update_and_launch_gaps": round(max(ms_per_step - sweep_ms, 0.0), 5),
                                          "sweeps_profiled": len(recs)},
               "algorithmic_bytes_per_iteration": total_bytes,
               "hbm_gbs_whole_iteration": round(total_bytes / (ms_per_step * 1e-3) / 1e9, 1),
               "dense_model_gbs_whole_iteration": round(12.0 * m * n / (ms_per_step * 1e-3) / 1e9, 1)}
        # counter-measured traffic: only for the very run the counters were taken on
        if os.path.exists(TRAFFIC_FILE):
            tr = json.load(open(TRAFFIC_FILE))
            if tr.get("workload") == P.name and tr.get("warmup") == W and tr.get("steps") == K:
                key = {7: "screened_lean_kernel", 5: "screened_sweep_kernel", 4: "sweep_kernel_tall"}.get(dominant)
                if key in tr.get("bytes_per_launch", {}):
                    roof["traffic"] = tr["bytes_per_launch"][key]
                    roof["traffic_source"] = tr.get("source")
        log(f"{label}: {K} iterations after {W} in {elapsed:.4f} s -> {K / elapsed:.1f} it/s, {ms_per_step:.4f} ms/iteration "
            f"(sweeps {sweep_ms:.4f} ms); dominant [{roof['kernel']}]: {roof['kernel_ms']:.4f} ms x {roof['launches_timed']} "
            f"-> {roof['achieved']:.0f} GB/s algorithmic ({roof['frac']:.1%} of {HBM_PEAK_GBS:.0f})")
        for e in roof["other_kernels"]:
            log(f"    also [{e['kernel']}]: {e['kernel_ms']:.4f} ms x {e['launches_timed']} -> {e['achieved']:.0f} GB/s ({e['frac']:.1%})")
        return out

    # ---- the timed region the command line asks for ---------------------------------------------------
    K, W = args.steps, args.warmup
    main_leg = measure(W, K, "timed region")
    steady = None
    if (W, K) == (STEADY_WARMUP, STEADY_STEPS):
        steady = main_leg
    elif "steady" in legs and P.m * P.n >= 1 << 22:
        steady = measure(STEADY_WARMUP, STEADY_STEPS, "steady state")

    # ---- the same steady-state iterations with the screening off, in pairs, with every byte moved -------
    def variant(label, **options):
        defaults()
        solver.solve(C, p, q, max_iters=STEADY_WARMUP, **kw)
        for name, value in options.items():
            getattr(solver, f"set_{name}")(value)
        solver.set_continue(True)
        solver.solve(C, p, q, max_iters=2, **kw)  # (settle the scheme's first-sweep special cases)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        solver.solve(C, p, q, max_iters=STEADY_STEPS, **kw)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        solver.set_profile(True)
        solver.solve(C, p, q, max_iters=256, **kw)
        recs = solver.profile_records()
        solver.set_profile(False)
        line_frac = nonzero_line_fraction() if P.reg_kind == 2 else 0.0
        kernels, x_before = {}, None
        for r in recs:
            e = kernels.setdefault(r.kind, {"ms": 0.0, "bytes": 0.0, "n": 0})
            e["ms"] += r.ms
            e["bytes"] += sweep_bytes(r, x_before, line_frac, options.get("skip_unchanged", args.skip_unchanged) != 0)
            e["n"] += 1
            x_before = r.x_fraction
        ks = []
        for kind in sorted(kernels):
            e = kernels[kind]
            gbs = e["bytes"] / (e["ms"] * 1e-3) / 1e9
            name = "gl_slab_kernel / group-lasso sweep" if (kind == 0 and P.reg_kind == 2) else KERNEL_NAMES[kind]
            ks.append({"kernel": name, "kernel_ms": round(e["ms"] / e["n"], 5), "launches_timed": e["n"],
                       "algorithmic_bytes": e["bytes"] / e["n"], "achieved": round(gbs, 1), "unit": "GB/s",
                       "frac": round(gbs / HBM_PEAK_GBS, 4), "bound": "hbm", "peak": HBM_PEAK_GBS, "traffic": None})
        log(f"{label}: {STEADY_STEPS / dt:.1f} it/s, {dt / STEADY_STEPS * 1e3:.4f} ms/iteration; " +
            "; ".join(f"{e['kernel_ms']:.4f} ms = {e['achieved']:.0f} GB/s ({e['frac']:.1%})" for e in ks))
        defaults()
        return {"value": round(STEADY_STEPS / dt, 2), "unit": "iterations/s", "ms_per_step": round(dt / STEADY_STEPS * 1e3, 5),
                "kernels": ks}

    unscreened_leg = even_odd_leg = dense_leg = None
    if "variants" in legs and steady is not None:
        if P.reg_kind != 2:
            unscreened_leg = variant("zero segments skipped, all of C read", screening=0)
            even_odd_leg = variant("even/odd scheme (20 B/element and pair)", skip_cost=1)
            dense_leg = variant("every byte moved (12 B/element)", skip_cost=0, skip_unchanged=0)
        else:
            dense_leg = variant("every byte moved (12 B/element)", skip_unchanged=0)

    # ---- the same iterations with the cost recomputed from the point clouds --------------------------
    points_leg = None
    if "points" in legs and P.reg_kind != 2 and P.xs is not None:
        xs, xt = torch.from_numpy(P.xs).to(dev), torch.from_numpy(P.xt).to(dev)
        cs = float(np.float32(1.0 / P.cmax))
        pkw = dict(reg_kind=P.reg_kind, lam=P.lam, X_out=X)
        defaults()
        solver.solve_points(xs, xt, cs, p, q, max_iters=STEADY_WARMUP, **pkw)
        solver.set_continue(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        solver.solve_points(xs, xt, cs, p, q, max_iters=STEADY_STEPS, **pkw)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        solver.set_profile(True)
        solver.solve_points(xs, xt, cs, p, q, max_iters=256, **pkw)
        recs = solver.profile_records()
        solver.set_profile(False)
        solver.set_continue(False)
        d = int(P.xs.shape[1])
        kernels = []
        for kind, name in ((8, "lean_points_kernel (cost formed on the matrix cores only for the row segments no bound covers)"),
                           (9, "sweep_points_kernel, recording the bounds (all costs formed: 2 d flops per element)"),
                           (0, "sweep_points_kernel (all costs formed: 2 d flops per element)")):
            sel = [r for r in recs if r.kind == kind]
            if not sel:
                continue
            ms = sum(r.ms for r in sel) / len(sel)
            e = {"kernel": name, "kernel_ms": round(ms, 5), "launches_timed": len(sel)}
            if kind == 8:
                formed = sum(r.c_fraction for r in sel) / len(sel)
                # per row segment: the old row sum and the three parts of the bound read (13 B), the new sum written where the
                # cost was formed; the strip's column sums; X on its nonzero row segments (read and written); the costs are
                # not traffic; flops: blocks of 16 rows x 256 columns
                xnz = sum(max(r.x_fraction, 0.0) for r in sel) / len(sel)
                nbytes = (13.0 + 4.0 * formed) * m * nseg + 4.0 * n * ((m + 255) // 256) + 8.0 * xnz * m * n
                gbs = nbytes / (ms * 1e-3) / 1e9
                e.update({"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "algorithmic_bytes": nbytes,
                          "row_segments_with_cost_formed_fraction": round(formed, 5),
                          "nonzero_row_segment_fraction": round(xnz, 5),
                          "useful_tflops": round(2.0 * d * formed * m * n / (ms * 1e-3) / 1e12, 2)})
            else:
                tflops = 2.0 * d * m * n / (ms * 1e-3) / 1e12
                e.update({"bound": "mfma", "achieved": round(tflops, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                          "frac": round(tflops / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None})
            kernels.append(e)
        points_leg = {"value": round(STEADY_STEPS / dt, 2), "unit": "iterations/s", "ms_per_step": round(dt / STEADY_STEPS * 1e3, 5),
                      "d": d, "kernels": kernels}
        log(f"cost from point clouds (d={d}): {STEADY_STEPS / dt:.1f} it/s, {dt / STEADY_STEPS * 1e3:.4f} ms/iteration; " +
            "; ".join(f"[{e['kernel'].split(' ')[0]}] {e['kernel_ms']:.4f} ms x {e['launches_timed']} = {e['achieved']} {e['unit']} "
                      f"({e['frac']:.1%})" + (f", cost formed on {e['row_segments_with_cost_formed_fraction']:.2%} of the row segments"
                                              if "row_segments_with_cost_formed_fraction" in e else "") for e in kernels))

    # ---- time to tolerance / to a duality gap (cold start), verified in fp64 by independent code -------
    def to_tolerance(label, gap_tol):
        defaults()
        solver.set_compute_gap(True)
        solver.set_gap_tolerance(gap_tol)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = solver.solve(C, p, q, max_iters=args.tol_max_iters, tol=args.tol, **kw)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        solver.set_gap_tolerance(0.0)
        solver.set_compute_gap(False)
        phi, varphi = solver.duals(m, n, dev)
        t = drot_checks.fp64_terms(C, X, p, q, phi, varphi, float(P.rho), reg_kind=P.reg_kind, lam=float(np.float32(P.lam)),
                                   mu=float(np.float32(P.mu)), row_class=rc, num_classes=P.num_classes)
        leg = {"tol": args.tol, "gap_tol": gap_tol or None, "seconds": round(dt, 4), "iters": r.iters,
               "converged": bool(r.converged), "r_row": r.r_row, "r_col": r.r_col, "objective": r.objective, "gap": r.gap,
               "dual_res": r.dual_res, "check_every": args.check_every,
               "fp64_check": {"min_entry": t.min_entry, "r_row": t.r_row, "r_col": t.r_col, "objective": t.objective,
                              "gap": t.gap, "dual_res": t.dual_res, "nonzeros": t.nnz,
                              "by": "drot_checks.py (plain torch fp64; shares no code with the library or the oracle)"}}
        log(f"{label}: {dt:.3f} s, {r.iters} iterations, converged={r.converged}, residuals {r.r_row:.2e}/{r.r_col:.2e}, "
            f"objective {r.objective:.6f}, gap {r.gap:.3e}; fp64: min {t.min_entry:.1e}, residuals {t.r_row:.2e}/{t.r_col:.2e}, "
            f"objective {t.objective:.6f}, gap {t.gap:.3e}")
        return leg

    tol_leg = to_tolerance(f"time to a residual of {args.tol:g}", 0.0) if "tol" in legs else None
    gap_leg = to_tolerance(f"time to a residual of {args.tol:g} and a gap of {args.gap_tol:g} x objective", args.gap_tol) \
        if "gap" in legs else None

    # ---- sizes n and n - 1 side by side (rows on and off the 128-byte lines) -----------------------------
    alignment_leg = None
    if "alignment" in legs and args.config == 4 and not args.size:
        del X, C
        torch.cuda.empty_cache()
        alignment_leg = alignment(torch, drot, dev)
        C = X = None

    # ---- CPU oracle on the host cores of this machine, bounded sample of the same workload ---------------
    cpu = None
    if "cpu" in legs:
        from oracle import drot_oracle

        drot_oracle.build()
        X = C = None
        torch.cuda.empty_cache()
        okw = dict(rho=float(P.rho), reg_kind=P.reg_kind, lam=float(np.float32(P.lam)), mu=float(np.float32(P.mu)),
                   row_class=P.row_class, num_classes=P.num_classes)
        iters = args.cpu_iters
        if not iters:  # a first call to size the sample for about 20 s (its first iteration pays the page faults)
            t0 = time.perf_counter()
            drot_oracle.solve(P.C, P.p, P.q, max_iters=4, **okw)
            per_iter = (time.perf_counter() - t0) / 4
            iters = max(2, min(20000, int(20.0 / per_iter)))
        t0 = time.perf_counter()
        drot_oracle.solve(P.C, P.p, P.q, max_iters=iters, **okw)
        dt = time.perf_counter() - t0
        cpu = {"value": round(iters / dt, 4), "unit": "iterations/s", "cores": drot_oracle.num_threads(),
               "kind": "oracle", "sample": f"{iters} iterations of the same {m}x{n} problem (fp64, explicit X, Y, Z)",
               "seconds": round(dt, 2)}
        log(f"oracle: {iters} iterations in {dt:.1f} s on {cpu['cores']} threads -> {cpu['value']} it/s")

    out = {
        "metric": "DR iterations/sec at m=n=20000 fp32" if (args.config == 4 and not args.size)
        else f"DR iterations/sec at {m}x{n} fp32",
        "value": main_leg["value"], "unit": "iterations/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": main_leg["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": P.name, "m": m, "n": n, "reg_kind": int(P.reg_kind), "lambda": P.lam, "mu": P.mu,
                   "stepsize": float(P.rho), "check_every": args.check_every},
        "algorithmic_bytes_per_iteration": main_leg["algorithmic_bytes_per_iteration"],
        "hbm_gbs_whole_iteration": main_leg["hbm_gbs_whole_iteration"],
        "dense_model_gbs_whole_iteration": main_leg["dense_model_gbs_whole_iteration"],
        "iteration_breakdown_ms": main_leg["iteration_breakdown_ms"],
        "roofline": main_leg["roofline"],
        "steady_state": steady if steady is not main_leg else "the timed region above (same warm-up and steps)",
        "time_to_tol": tol_leg, "time_to_gap": gap_leg, "unscreened": unscreened_leg, "even_odd_scheme": even_odd_leg,
        "every_byte_moved": dense_leg, "cost_from_points": points_leg, "alignment": alignment_leg, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


def alignment(torch, drot, dev):
    """Iterations per second at n and n - 1 (the paper's Table 3 sizes): rows on and off the 128-byte lines,
    with every byte moved and with the library's defaults.  Synthetic clouds made on the device."""
    rows = []
    for n in (4096, 8192, 10240):
        pair = {}
        for size in (n, n - 1):
            # (the same clouds less their last points: the density of the plan, which the default path's speed
            # depends on, stays the same)
            gen = torch.Generator(device=dev).manual_seed(4000 + n)
            xs = torch.randn((n, 8), generator=gen, device=dev)[:size].contiguous()
            xt = (0.3 + 1.2 * torch.randn((n, 8), generator=gen, device=dev))[:size].contiguous()
            C = torch.cdist(xs, xt).pow_(2)
            C /= C.max()
            p = torch.full((size,), 1.0 / size, device=dev)
            q = torch.full((size,), 1.0 / size, device=dev)
            X = torch.empty_like(C)
            solver = drot.Solver(size, size, compute_gap=False)
            for scheme in ("every_byte_moved", "default"):
                if scheme == "every_byte_moved":
                    solver.set_skip_cost(0)
                    solver.set_skip_unchanged(0)
                else:
                    solver.set_skip_cost(-1)
                    solver.set_skip_unchanged(-1)
                best = 0.0
                for _ in range(5):  # (the best of five: the smallest of these runs are a few tens of milliseconds long)
                    solver.set_continue(False)
                    solver.solve(C, p, q, reg_kind=1, lam=1e-3, max_iters=200, X_out=X)
                    solver.set_continue(True)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    solver.solve(C, p, q, reg_kind=1, lam=1e-3, max_iters=ALIGN_STEPS, X_out=X)
                    torch.cuda.synchronize()
                    best = max(best, ALIGN_STEPS / (time.perf_counter() - t0))
                pair[(size, scheme)] = best
            solver.close()
            del C, X
            torch.cuda.empty_cache()
        for scheme in ("every_byte_moved", "default"):
            a, b = pair[(n, scheme)], pair[(n - 1, scheme)]
            rows.append({"n": n, "scheme": scheme, "its_per_s_n": round(a, 1), "its_per_s_n_minus_1": round(b, 1),
                         "slowdown_percent": round((a / b - 1.0) * 100.0, 2)})
            log(f"alignment {n} vs {n - 1} [{scheme}]: {a:.0f} vs {b:.0f} it/s ({(a / b - 1.0) * 100.0:+.2f} %)")
    return {"note": f"{ALIGN_STEPS} iterations continuing a 200-iteration cold start (best of five), each call copying X out of "
                    "the padded working copy when n % 32 != 0", "rows": rows}


if __name__ == "__main__":
    sys.exit(main())
