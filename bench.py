#!/usr/bin/env python3
"""Benchmark of the Douglas-Rachford OT solver on one MI355X.

A step is one iteration of the method: the sweep over the m x n plan (prox of nonnegativity, cost
and regularizer fused with the row/column sums), the O(m+n) vector update, and the periodic
residual test where one is scheduled.  Default workload: the quadratically regularized
20000 x 20000 configuration (C and X 1.6 GB each, resident in HBM before timing starts).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--size N]

prints one JSON line: iterations/s, the HBM roofline of the dominant sweep kernel (algorithmic bytes
per launch over the kernel time from HIP events recorded on the launch stream), the time to a
marginal residual of 1e-4, and the CPU oracle timed on a bounded sample on this machine's host cores.

The default sweep at this size neither reads nor writes back row segments of X that are zero and
stay zero.  Transport plans are sparse, so after the first few dozen iterations the sweep streams C
(4 bytes per element) plus the few nonzero segments of X (8 bytes per element of those); its
algorithmic bytes are counted that way, from the fraction of nonzero row segments in the plan the
timed run ends with.  Two further legs time the same iterations with the even/odd scheme of the
paper's GPU appendix (20 bytes per element and pair) and with every byte moved (12 bytes per
element): that last one is the dense streaming rate of the sweep kernel.
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
BYTES_PER_ELEMENT = {0: 12.0, 1: 12.0, 2: 8.0, 3: 12.0}  # by kind of sweep: read X, read C, write X; kind 2 reads no C;
# kind 3 (resident kernel) is priced at the same 12 although nothing leaves the registers; kind 4 (zero segments
# skipped) is priced from the plan's density, see sparse_sweep_bytes

# HBM traffic of one sweep launch in bytes, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs scaled by a
# copy kernel of known size (see profiles/); None until measured for a workload.
MEASURED_TRAFFIC_BYTES = {  # (workload, kind of sweep); profiles/sweep_kernel_cfg4_20000.md
    ("cfg4_quad_20000", 0): 4.8565e9, ("cfg4_quad_20000", 1): 4.8565e9, ("cfg4_quad_20000", 2): 3.2565e9,
    ("cfg4_quad_20000", 4): 1.6957e9, ("cfg4_quad_20000", 7): 9.271e7}
SEG_COLS = 256  # columns of a row segment, the unit of the zero-segment skipping


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=200,
                    help="untimed cold-start iterations (the support of the plan settles within the first 100 or so)")
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1..5 (default 4: 20000 x 20000)")
    ap.add_argument("--size", type=int, default=0, help="override m = n (same recipe)")
    ap.add_argument("--tol", type=float, default=1e-4, help="residual of the time-to-tolerance leg")
    ap.add_argument("--tol-max-iters", type=int, default=40000)
    ap.add_argument("--check-every", type=int, default=100)
    ap.add_argument("--nontemporal", type=int, default=-1, help="-1: library default, 0/1: force off/on")
    ap.add_argument("--skip-cost", type=int, default=-1,
                    help="even/odd scheme (C read every second sweep): -1 library default, 0 never, 1 wherever it applies")
    ap.add_argument("--skip-unchanged", type=int, default=-1, help="zero-segment skipping: -1/1 on, 0 off")
    ap.add_argument("--points", action="store_true", help="on-the-fly cost from the point clouds (drot_solve_points)")
    ap.add_argument("--skip-tol", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--cpu-iters", type=int, default=0, help="oracle iterations to time (0: sized for ~20 s)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

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
    log(f"workload {P.name}: m={m} n={n} reg_kind={P.reg_kind} lambda={P.lam} mu={P.mu} (generated in {time.time() - t0:.1f} s)")
    C = torch.from_numpy(P.C).to(dev)
    p = torch.from_numpy(P.p).to(dev)
    q = torch.from_numpy(P.q).to(dev)
    rc = None if P.row_class is None else torch.from_numpy(P.row_class).to(dev)
    X = torch.empty_like(C)
    kw = dict(reg_kind=P.reg_kind, lam=P.lam, mu=P.mu, row_class=rc, num_classes=P.num_classes, X_out=X)
    solver = drot.Solver(m, n, check_every=args.check_every, compute_gap=False)
    solver.set_nontemporal(args.nontemporal)
    solver.set_skip_cost(args.skip_cost)
    solver.set_skip_unchanged(args.skip_unchanged)
    torch.cuda.synchronize()

    # ---- warm-up (cold start), then exactly K steady-state iterations continuing from it --------------
    K, W = args.steps, args.warmup
    solver.solve(C, p, q, max_iters=W, **kw)
    solver.set_continue(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res = solver.solve(C, p, q, max_iters=K, **kw)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert res.iters == K
    ms_per_step = elapsed / K * 1e3
    log(f"{K} iterations in {elapsed:.3f} s -> {K / elapsed:.1f} it/s, {ms_per_step:.4f} ms/iteration")

    # ---- sweep kernel durations from HIP events on the launch stream (profile mode, separate solve) ----
    c_read = {}  # kind of sweep -> mean fraction of the row segments of C it read (screened kinds: counted by the kernel)

    def sweep_profile():
        solver.set_profile(True)
        solver.solve(C, p, q, max_iters=min(K, 256), **kw)
        per_kind, reads = {}, {}
        for (ms, kind), frac in zip(solver.profile_sweeps(), solver.profile_reads()):
            per_kind.setdefault(kind, []).append(ms)
            reads.setdefault(kind, []).append(frac)
        solver.set_profile(False)
        c_read.update({kind: sum(v) / len(v) for kind, v in reads.items()})
        return {kind: (sum(v) / len(v), len(v)) for kind, v in per_kind.items()}

    def nonzero_segment_fraction():
        """Fraction of row segments (256 columns of one row) of X that hold a nonzero."""
        nz = 0
        for j0 in range(0, n, SEG_COLS):
            nz += int((X[:, j0:j0 + SEG_COLS] != 0).any(dim=1).sum().item())
        return nz / (m * ((n + SEG_COLS - 1) // SEG_COLS))

    def nonzero_line_fraction():
        """Fraction of the 128-byte lines (32 columns of one row, counted from the segment's start) of X that hold a nonzero."""
        nz = total = 0
        for j0 in range(0, n, 32):
            nz += int((X[:, j0:j0 + 32] != 0).any(dim=1).sum().item())
            total += m
        return nz / total

    def sparse_sweep_bytes(frac, c_frac=1.0, screened=False, tile_rows=64, per_segment=8.0):
        # C on the fraction c_frac of its row segments; X read and written back only on the fraction
        # frac of its entries that lie in nonzero row segments (lean kernel: in nonzero 128-byte
        # lines) -- an upper bound, a piece is charged as a whole; per row segment the old and the
        # new row sum and the bound M of the screening (lean kernel: the new sum, the bound and two
        # bytes of line flags, which stand in for the old sum);
        # the column sums per 64-row tile (per four of them in the lean kernel)
        nseg = (n + SEG_COLS - 1) // SEG_COLS
        return (4.0 * c_frac * m * n + 8.0 * frac * m * n + per_segment * m * nseg +
                4.0 * n * ((m + tile_rows - 1) // tile_rows))

    line_frac = {}

    def bytes_of(kind, frac):
        if kind == 7:
            if "v" not in line_frac:
                line_frac["v"] = nonzero_line_fraction()
            return sparse_sweep_bytes(line_frac["v"], c_read.get(kind, 1.0), True, 256, 10.0)
        if kind in (4, 5, 6):
            return sparse_sweep_bytes(frac, c_read.get(kind, 1.0), kind != 4, 64, 12.0 if kind != 4 else 8.0)
        if kind == 0 and P.reg_kind == 2 and args.skip_unchanged != 0:
            # group-resident group lasso: all of C; of X the 128-byte lines (32 columns of a row) that hold
            # a nonzero; per line the old and the new sum; the column sums per class
            if "v" not in line_frac:
                line_frac["v"] = nonzero_line_fraction()
            return (4.0 + 8.0 * line_frac["v"]) * m * n + 8.0 * m * ((n + 31) // 32) + 4.0 * n * max(1, P.num_classes)
        return BYTES_PER_ELEMENT[kind] * m * n

    def kernel_entry(kind, ms, launches, nbytes=None):
        nbytes = bytes_of(kind, nonzero_segment_fraction()) if nbytes is None else nbytes
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get((P.name, kind)),
                "kernel": kernel_names[kind], "kernel_ms": round(ms, 5), "launches_timed": launches,
                "algorithmic_bytes": nbytes}

    kernel_names = {0: "gl_slab_kernel" if P.reg_kind == 2 else "sweep_kernel (reads X and C, stores X)",
                    1: "sweep_kernel, first of a pair (reads X and C, stores X - rho*C)",
                    2: "sweep_kernel, second of a pair (reads X - rho*C, stores X)",
                    3: "resident_kernel (X and C stay in registers; the time is per iteration)",
                    4: "sweep_kernel on 64-row tiles (reads C; reads and stores only the nonzero row segments of X)",
                    5: "screened_sweep_kernel (reads C only where a bound does not certify zeros; nonzero row segments of X)",
                    6: "screened_sweep_kernel, refresh (reads all of C, records the bounds)",
                    7: "screened_lean_kernel (one wave per 64 x 256 tile; reads C only where a bound does not certify zeros)"}
    prof = sweep_profile()
    frac_nz = nonzero_segment_fraction()
    kind_bytes = {k: bytes_of(k, frac_nz) for k in prof}
    dominant = max(prof, key=lambda kind: prof[kind][0] * prof[kind][1])
    roofline = kernel_entry(dominant, *prof[dominant], nbytes=kind_bytes[dominant])
    bytes_per_iteration = sum(kind_bytes[k] * cnt for k, (_, cnt) in prof.items()) / sum(c for _, c in prof.values())
    log(f"dominant sweep kernel [{roofline['kernel']}]: {roofline['kernel_ms']:.4f} ms mean over {roofline['launches_timed']} launches "
        f"-> {roofline['achieved']:.0f} GB/s algorithmic ({roofline['frac']:.1%} of {HBM_PEAK_GBS:.0f} GB/s)")
    if dominant == 0 and P.reg_kind == 2 and "v" in line_frac:
        roofline["bytes_model"] = ("4 B per element (C) + 8 B x the entries of X in nonzero 128-byte lines (counted on the final plan) "
                                   "+ 8 B per line (old and new sums) + column sums; the working set fits the 256 MB memory-side cache")
        roofline["nonzero_line_fraction"] = round(line_frac["v"], 6)
        roofline["dense_model_gbs"] = round(12.0 * m * n / (roofline["kernel_ms"] * 1e-3) / 1e9, 1)
        log(f"nonzero 128-byte lines of X: {line_frac['v']:.3%}; priced at 12 B/element the sweep would read {roofline['dense_model_gbs']:.0f} GB/s")
    if dominant in (4, 5, 6, 7):
        roofline["bytes_model"] = ("4 B x the row segments of C read (counted by the kernel) + 8 B x the entries of X in nonzero row segments "
                                   "(lean kernel: in nonzero 128-byte lines; counted on the final plan) + 8-12 B per row segment (old and new "
                                   "sums, bound, line flags) + column sums; dense_model_* prices the same launch at 12 B per element")
        roofline["nonzero_row_segment_fraction"] = round(frac_nz, 5)
        if "v" in line_frac:
            roofline["nonzero_line_fraction"] = round(line_frac["v"], 6)
        roofline["c_row_segments_read_fraction"] = round(c_read.get(dominant, 1.0), 5)
        roofline["other_kernels"] = [kernel_entry(k, *prof[k], nbytes=kind_bytes[k]) for k in sorted(prof) if k != dominant]
        roofline["dense_model_bytes"] = 12.0 * m * n
        roofline["dense_model_gbs"] = round(12.0 * m * n / (roofline["kernel_ms"] * 1e-3) / 1e9, 1)
        # (above 1: the sweep does not move the bytes the dense model charges; the leg every_byte_moved
        # below is the same solver made to move them all, with its own roofline)
        roofline["dense_model_frac"] = round(roofline["dense_model_gbs"] / HBM_PEAK_GBS, 3)
        log(f"nonzero row segments of X: {frac_nz:.3%}" + (f" (128-byte lines: {line_frac['v']:.4%})" if "v" in line_frac else "") +
            f"; row segments of C read: {c_read.get(dominant, 1.0):.3%}; "
            f"the same sweep priced at 12 B/element would read {roofline['dense_model_gbs']:.0f} GB/s")
        for e in roofline["other_kernels"]:
            log(f"  also [{e['kernel']}]: {e['kernel_ms']:.4f} ms over {e['launches_timed']} launches -> {e['achieved']:.0f} GB/s ({e['frac']:.1%})")

    def timed_leg(label, nbytes=None):
        """K more iterations from the current state with the solver's current settings, then a profile."""
        solver.set_continue(True)
        solver.solve(C, p, q, max_iters=2, **kw)  # (settle the scheme's first-sweep special cases)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        solver.solve(C, p, q, max_iters=K, **kw)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        lprof = sweep_profile()
        solver.set_continue(False)
        leg = {"value": round(K / dt, 2), "unit": "iterations/s", "ms_per_step": round(dt / K * 1e3, 5),
               "kernels": [kernel_entry(k, *lprof[k], nbytes=nbytes) for k in sorted(lprof)]}
        log(f"{label}: {K / dt:.1f} it/s, {dt / K * 1e3:.4f} ms/iteration; " +
            "; ".join(f"{e['kernel_ms']:.4f} ms = {e['achieved']:.0f} GB/s ({e['frac']:.1%})" for e in leg["kernels"]))
        return leg

    # ---- the same K iterations with the even/odd scheme, and with every byte moved ----------------------
    even_odd_leg = dense_leg = None
    unscreened_leg = None
    if dominant in (5, 6, 7):
        solver.set_screening(0)
        unscreened_leg = timed_leg("zero segments skipped, all of C read")
        solver.set_screening(-1)
    if dominant in (4, 5, 6, 7):
        solver.set_skip_cost(1)
        even_odd_leg = timed_leg("even/odd scheme (20 B/element and pair)")
        solver.set_skip_cost(0)
        solver.set_skip_unchanged(0)
        dense_leg = timed_leg("every byte moved (12 B/element)")
        solver.set_skip_cost(args.skip_cost)
        solver.set_skip_unchanged(args.skip_unchanged)
    if dominant == 0 and P.reg_kind == 2 and args.skip_unchanged != 0:
        solver.set_skip_unchanged(0)
        dense_leg = timed_leg("every byte moved (12 B/element)", nbytes=12.0 * m * n)
        solver.set_skip_unchanged(args.skip_unchanged)
    solver.set_continue(False)

    # ---- the same K iterations with the cost recomputed from the point clouds ------------------------
    points_leg = None
    if P.reg_kind != 2 and P.xs is not None and (args.points or not args.skip_tol):
        xs, xt = torch.from_numpy(P.xs).to(dev), torch.from_numpy(P.xt).to(dev)
        cs = float(np.float32(1.0 / P.cmax))
        pkw = dict(reg_kind=P.reg_kind, lam=P.lam, X_out=X)
        solver.solve_points(xs, xt, cs, p, q, max_iters=W, **pkw)
        solver.set_continue(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        solver.solve_points(xs, xt, cs, p, q, max_iters=K, **pkw)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        solver.set_profile(True)
        solver.solve_points(xs, xt, cs, p, q, max_iters=min(K, 256), **pkw)
        pms, _ = solver.profile()
        solver.set_profile(False)
        solver.set_continue(False)
        # bytes: X read and written on its nonzero row segments only (with the zero-segment skipping
        # on; every element otherwise), the old and new row sums, the column sums; the contraction is
        # 2d flops per element on the fp32 matrix cores whatever the plan looks like
        fnz = nonzero_segment_fraction() if args.skip_unchanged != 0 else 1.0
        pbytes = 8.0 * fnz * m * n + 8.0 * m * ((n + SEG_COLS - 1) // SEG_COLS) + 4.0 * n * ((m + 31) // 32)
        points_leg = {"value": round(K / dt, 2), "unit": "iterations/s", "ms_per_step": round(dt / K * 1e3, 5),
                      "d": int(P.xs.shape[1]), "algorithmic_bytes_per_iteration": pbytes,
                      "nonzero_row_segment_fraction": round(fnz, 5),
                      "kernel_ms": round(pms, 5), "kernel_hbm_gbs": round(pbytes / (pms * 1e-3) / 1e9, 1),
                      "kernel_tflops": round(2.0 * P.xs.shape[1] * m * n / (pms * 1e-3) / 1e12, 2)}
        log(f"cost from point clouds (d={points_leg['d']}): {K / dt:.1f} it/s, {dt / K * 1e3:.4f} ms/iteration; sweep "
            f"{pms:.4f} ms = {points_leg['kernel_tflops']} TFLOP/s fp32 MFMA, {points_leg['kernel_hbm_gbs']:.0f} GB/s of HBM "
            f"(X on its {fnz:.1%} nonzero row segments)")

    # ---- time to tolerance (cold start, residual test every check_every iterations) -------------------
    tol_leg = None
    if not args.skip_tol:
        solver.set_compute_gap(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = solver.solve(C, p, q, max_iters=args.tol_max_iters, tol=args.tol, **kw)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        tol_leg = {"tol": args.tol, "seconds": round(dt, 4), "iters": r.iters, "converged": bool(r.converged),
                   "r_row": r.r_row, "r_col": r.r_col, "objective": r.objective, "gap": r.gap,
                   "dual_res": r.dual_res, "check_every": args.check_every}
        log(f"time to {args.tol:g}: {dt:.3f} s, {r.iters} iterations, converged={r.converged}, "
            f"residuals {r.r_row:.2e}/{r.r_col:.2e}, objective {r.objective:.6f}, gap {r.gap:.3e}")
        solver.set_compute_gap(False)

    # ---- CPU oracle on the host cores of this machine, bounded sample of the same workload ---------------
    cpu = None
    if not args.skip_cpu:
        from oracle import drot_oracle

        drot_oracle.build()
        del X
        torch.cuda.empty_cache()
        okw = dict(rho=float(P.rho), reg_kind=P.reg_kind, lam=float(np.float32(P.lam)), mu=float(np.float32(P.mu)),
                   row_class=P.row_class, num_classes=P.num_classes)
        iters = args.cpu_iters
        if not iters:  # a first call to size the sample for about 20 s (its first iteration pays the page faults)
            t0 = time.perf_counter()
            drot_oracle.solve(P.C, P.p, P.q, max_iters=4, **okw)
            per_iter = (time.perf_counter() - t0) / 4
            iters = max(2, min(20000, int(25.0 / per_iter)))
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
        "value": round(K / elapsed, 2), "unit": "iterations/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": P.name, "m": m, "n": n, "reg_kind": int(P.reg_kind), "lambda": P.lam, "mu": P.mu,
                   "stepsize": float(P.rho), "check_every": args.check_every},
        "algorithmic_bytes_per_iteration": bytes_per_iteration,
        # (the dense model's 12 B per element over the iteration time: what a solver that moves every
        # byte would have to sustain to keep up; far above the 8000 GB/s peak when the sweeps skip work)
        "dense_model_gbs_whole_iteration": round(12.0 * m * n / (ms_per_step * 1e-3) / 1e9, 1),
        "hbm_gbs_whole_iteration": round(bytes_per_iteration / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline, "time_to_tol": tol_leg, "unscreened": unscreened_leg, "even_odd_scheme": even_odd_leg,
        "every_byte_moved": dense_leg,
        "cost_from_points": points_leg, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
