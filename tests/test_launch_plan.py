"""The launch planner (csrc/drot_plan.h) without a GPU: which kernel runs which sweep.

The product library enqueues exactly what this logic decides.  Here it is compiled with the host
compiler (libdrot_plan.so) and driven with scripted statuses: every path, every switch between paths
(zero-segment skipping <-> even/odd pairs, 8-wave screened <-> lean), continued calls, the early looks
at the density, a stop at a check with work queued behind it.
"""
import ctypes
import os

import numpy as np
import pytest

RESIDENT, PRO32, PLAIN32, TALL64, SCREENED8, LEAN, POINTS, SLAB, TWOPASS, POINTS_LEAN = range(10)
NO_UPDATE, SEPARATE, MERGED_SLAB, MERGED_TILES = range(4)
COLS = ("sweep", "mode", "first", "prev_sums", "lines_in", "refresh", "pro", "tilesum", "update", "ra", "kind", "flags")
FRESH_CARRY = (0, -1000000, -1, 8, 0, 0, 0, 0)


@pytest.fixture(scope="module")
def planlib():
    from paper_2305_18483_amd import build

    if not os.path.exists(build.PLAN_LIB_PATH) or os.path.getmtime(build.PLAN_LIB_PATH) < max(
            os.path.getmtime(build.PLAN_SOURCE), os.path.getmtime(os.path.join(os.path.dirname(build.PLAN_SOURCE), "drot_plan.h"))):
        build.build_plan()
    lib = ctypes.CDLL(build.PLAN_LIB_PATH)
    lib.drot_plan_trace.restype = ctypes.c_int
    lib.drot_plan_labels.restype = ctypes.c_int
    return lib


class Trace:
    def __init__(self, rows, statics, carry, iters):
        self.rows, self.statics, self.carry, self.iters = rows, statics, carry, iters

    def col(self, name):
        return [int(r[COLS.index(name)]) for r in self.rows]


def trace(lib, m, n, max_iters, reg_kind=0, from_points=0, warm=0, resume=0, weights=0, c_on_lines=1, x_on_lines=1,
          slab_k=0, nruns=0, feedback=1, checking=1, check_every=100, resident=-1, fused_update=-1, skip_cost=-1,
          skip_unchanged=-1, screening=-1, nontemporal=-1, force_two_pass=0, gap_every=0, densities=(), stop_at_status=-1,
          carry=FRESH_CARRY):
    problem = (ctypes.c_int * 14)(m, n, reg_kind, from_points, warm, resume, weights, c_on_lines, x_on_lines, slab_k, nruns,
                                  feedback, checking, max_iters)
    options = (ctypes.c_int * 9)(check_every, resident, fused_update, skip_cost, skip_unchanged, screening, nontemporal,
                                 force_two_pass, gap_every)
    carry_io = (ctypes.c_longlong * 8)(*carry)
    dens = (ctypes.c_double * max(1, len(densities)))(*densities)
    cap = max_iters + 8
    rows = (ctypes.c_int * (12 * cap))()
    statics = (ctypes.c_int * 10)()
    iters = ctypes.c_int()
    nrows = lib.drot_plan_trace(problem, options, carry_io, dens, len(densities), stop_at_status, rows, cap, statics,
                                ctypes.byref(iters))
    assert nrows >= 0
    arr = np.array(rows[:12 * nrows], dtype=np.int64).reshape(nrows, 12)
    names = ("nseg", "ntr", "resident", "pad_c", "pad_x", "small", "fused", "may_screen", "adaptive", "nt")
    return Trace(arr, dict(zip(names, statics)), tuple(carry_io), iters.value)


def test_the_five_configurations_take_their_paths(planlib):
    t = trace(planlib, 100, 100, 2000, checking=0)
    assert t.statics["resident"] and t.col("sweep") == [RESIDENT] and len(t.rows) == 1  # one launch for all 2000
    t = trace(planlib, 100, 100, 250, checking=1, check_every=100)
    assert t.col("sweep") == [RESIDENT] * 3  # a launch per stretch between checks
    t = trace(planlib, 1000, 1000, 300, reg_kind=1)
    assert t.statics["small"] and t.statics["fused"] and not t.statics["adaptive"] and not t.statics["nt"]
    assert t.col("sweep")[0] == PLAIN32 and set(t.col("sweep")[1:]) <= {PRO32, PLAIN32}
    # one launch per iteration: the update runs separately only at the end of a stretch
    assert [i for i, u in enumerate(t.col("update")) if u == SEPARATE] == [99, 199, 299]
    assert t.col("sweep")[100] == PLAIN32 and t.col("sweep")[101] == PRO32  # after a materialised state: plain again
    t = trace(planlib, 20000, 20000, 40, reg_kind=1, checking=0)
    assert t.statics["may_screen"] and t.statics["adaptive"] and t.statics["nt"] and not t.statics["small"]
    t = trace(planlib, 5000, 5000, 30, reg_kind=2, slab_k=4, nruns=10)
    assert set(t.col("sweep")) == {SLAB} and set(t.col("update")) == {MERGED_SLAB} and not t.statics["small"]
    t = trace(planlib, 5000, 5000, 5, reg_kind=2, slab_k=0, nruns=5000)
    assert set(t.col("sweep")) == {TWOPASS} and set(t.col("update")) == {SEPARATE}


def test_padded_copies_when_rows_are_off_the_128_byte_lines(planlib):
    assert not trace(planlib, 300, 512, 1).statics["pad_c"] and not trace(planlib, 300, 512, 1).statics["pad_x"]
    s = trace(planlib, 300, 500, 1).statics
    assert s["pad_c"] and s["pad_x"]
    s = trace(planlib, 300, 512, 1, c_on_lines=0).statics
    assert s["pad_c"] and not s["pad_x"]
    s = trace(planlib, 300, 512, 1, x_on_lines=0).statics
    assert not s["pad_c"] and s["pad_x"]
    assert trace(planlib, 300, 512, 1, weights=1).statics["pad_c"]          # C + W needs a working copy
    s = trace(planlib, 300, 500, 1, from_points=1).statics
    assert not s["pad_c"] and s["pad_x"]                                     # no stored cost to pad
    s = trace(planlib, 100, 100, 1, x_on_lines=0, c_on_lines=0).statics
    assert s["resident"] and not s["pad_c"] and not s["pad_x"]               # the resident kernel takes any pitch


def test_cold_start_of_a_large_sparse_problem_moves_to_the_lean_sweep(planlib):
    # statuses: the looks after 16, 32, 64 ... iterations report 90 %, 60 %, 20 %, 5 % nonzero row segments
    t = trace(planlib, 20000, 20000, 300, reg_kind=1, checking=1, densities=(0.9, 0.6, 0.2, 0.05))
    kinds = t.col("kind")
    # sweep 1 has nothing to read; sweep 2 records the bounds, then after 8, 16, 32 sweeps again
    assert kinds[:12] == [0, 6] + [5] * 7 + [6, 5, 5]
    assert kinds[25] == 6 and kinds[57] == 6
    flags = t.col("flags")
    ends = [i + 1 for i, f in enumerate(flags) if f & 1]
    assert ends[:6] == [16, 32, 64, 96, 100, 128]
    assert [bool(flags[e - 1] & 2) for e in ends[:6]] == [True, True, True, True, False, True]
    # the third status (after 64: 20 %) is read while the stretch to 96 is queued: lean from sweep 97 on
    first_lean = kinds.index(7)
    assert first_lean == 96 and set(kinds[96:]) == {7}
    assert t.col("lines_in")[96] == 0 and set(t.col("lines_in")[97:]) == {1}  # flags are valid from one lean sweep to the next
    assert set(t.col("update")[1:]) == {MERGED_TILES} and t.col("update")[0] == SEPARATE
    # column partials: 625 rows for the 32-row tiles, 313 in groups of four for the 64-row tiles, 79 for the lean sweep
    assert t.col("ra")[0] == 625 * 16 + 1 and t.col("ra")[5] == 313 * 16 + 4 and t.col("ra")[100] == 79 * 16 + 1
    # never the even/odd pairs here: the dense readings came from early looks
    assert set(t.col("mode")) == {0}


def test_gap_pass_goes_lean_once_bounds_and_flags_describe_the_plan(planlib):
    # stretch ends of the cold start above: no bounds after the first sweeps of a call; row-segment sums serve as
    # flags after the 8-wave sweeps, the line flags after lean sweeps; never on paths that do not screen
    t = trace(planlib, 20000, 20000, 300, reg_kind=1, checking=1, check_every=100, densities=(0.9, 0.6, 0.2, 0.02))
    flags = t.col("flags")
    ends = {i + 1: f for i, f in enumerate(flags) if f & 1}
    assert all(f & 8 for f in ends.values())  # (bounds exist from sweep 2 on)
    assert not ends[16] & 16 and not ends[96] & 16 and ends[100] & 16 and ends[300] & 16
    t = trace(planlib, 1000, 1000, 200, reg_kind=1, checking=1, check_every=100)
    assert not any(f & 8 for f in t.col("flags"))
    t = trace(planlib, 20000, 20000, 200, reg_kind=1, checking=1, check_every=100, from_points=1)
    assert not any(f & 8 for f in t.col("flags"))
    t = trace(planlib, 5000, 5000, 200, reg_kind=2, slab_k=4, nruns=10, checking=1, check_every=100)
    assert not any(f & 8 for f in t.col("flags"))
    # even/odd pairs: the sums of a plain sweep at the stretch end still describe X, the bounds are those of the
    # last refresh
    t = trace(planlib, 20000, 20000, 64, reg_kind=1, checking=0, skip_unchanged=0)
    assert not any(f & 8 for f in t.col("flags"))  # (nothing recorded bounds)


def test_dense_plans_switch_to_the_even_odd_pairs_and_back(planlib):
    t = trace(planlib, 2300, 1500, 90, reg_kind=1, checking=0, check_every=10, screening=1, densities=(0.95,))
    kinds = t.col("kind")
    assert kinds[:10] == [0, 6] + [5] * 7 + [6]
    # early looks (16, 32, ...) never start the pairs; the status of the stretch ending at 10 does, read during 10..16
    assert set(kinds[16:]) == {1, 2} and kinds[10:16] == [5] * 6
    modes = t.col("mode")
    for end in [i + 1 for i, f in enumerate(t.col("flags")) if f & 1]:
        assert modes[end - 1] in (0, 2)  # X is plain at every stretch end
    # and back below 50 %
    t = trace(planlib, 2300, 1500, 80, reg_kind=1, checking=1, check_every=10, screening=0, resume=1,
              carry=(1, 900000, -1, 8, 1, 256, 0, 100), densities=(0.9, 0.4))
    kinds = t.col("kind")
    assert set(kinds[:30]) == {1, 2} and set(kinds[30:]) == {4}
    assert t.col("prev_sums")[30] == 1  # a mode-2 sweep leaves plain X and its sums


def test_odd_stretches_of_pairs_start_with_a_plain_sweep(planlib):
    t = trace(planlib, 700, 1300, 37, reg_kind=1, checking=1, check_every=7, fused_update=0, skip_cost=1)
    assert t.col("mode")[:7] == [0, 1, 2, 1, 2, 1, 2] and t.col("first")[0] == 1
    t = trace(planlib, 700, 1300, 8, reg_kind=1, checking=0, fused_update=0, skip_cost=1)
    assert t.col("mode") == [1, 2] * 4


def test_a_continued_call_goes_on_where_the_last_one_stopped(planlib):
    kw = dict(reg_kind=1, checking=1, check_every=50, densities=(0.9, 0.5, 0.1, 0.05, 0.05, 0.05))
    one = trace(planlib, 20000, 20000, 260, **kw)
    first = trace(planlib, 20000, 20000, 150, **kw)
    assert first.carry[4] == 1 and first.carry[6] == 1 and first.carry[7] == 150 and first.carry[2] >= 0
    second = trace(planlib, 20000, 20000, 110, resume=1, carry=first.carry, reg_kind=1, checking=1, check_every=50,
                   densities=(0.05,))
    # no new epoch, no dense first sweep: lean from its first sweep, line flags valid
    assert second.col("kind")[0] == 7 and second.col("lines_in")[0] == 1 and second.col("first")[0] == 0
    assert one.col("kind")[150:] == second.col("kind")
    # without continuation state (another option set, say) nothing is taken for granted
    cold = trace(planlib, 20000, 20000, 10, resume=1, carry=(0, 50000, -1, 8, 0, 0, 0, 150), reg_kind=1)
    assert cold.col("prev_sums")[0] == 0 and cold.col("kind")[0] == 6


def test_a_stop_at_a_check_forgets_what_the_sweeps_queued_behind_it_would_have_left(planlib):
    # check_every 25, the check at iteration 100 passes; the stretch 101..125 is already queued, and the
    # host-ordered refresh at sweep 122 lies in it: it never runs, so the continued call must not count on it
    t = trace(planlib, 2300, 2500, 5000, reg_kind=1, checking=1, check_every=25, skip_cost=0, screening=1, feedback=1,
              densities=(0.5,), stop_at_status=6)  # statuses: 16, 25, 32, 50, 64, 75, 96?, ...
    ends = [i + 1 for i, f in enumerate(t.col("flags")) if f & 1]
    stop_iter = ends[6]
    assert t.iters == stop_iter and len(t.rows) == ends[7]  # one more stretch was queued
    assert t.carry[2] == -1 and t.carry[3] == 8 and t.carry[4] == 0 and t.carry[6] == 0 and t.carry[7] == stop_iter
    cont = trace(planlib, 2300, 2500, 40, reg_kind=1, checking=1, check_every=25, skip_cost=0, screening=1, resume=1,
                 carry=t.carry, densities=(0.5,))
    assert cont.col("kind")[0] == 6 and cont.col("prev_sums")[0] == 0  # new bounds first, everything read


def test_without_feedback_the_schedule_is_fixed(planlib):
    # (what an entry point that never reads the status block during the solve runs)
    t = trace(planlib, 4096, 4096, 300, reg_kind=1, checking=1, feedback=0, densities=(0.01,))
    assert not t.statics["adaptive"] and t.statics["may_screen"]
    kinds = t.col("kind")
    assert 7 not in kinds and set(t.col("mode")) == {0}
    assert not any(f & 2 for f in t.col("flags"))  # no early looks
    assert [i + 1 for i, f in enumerate(t.col("flags")) if f & 1] == [100, 200, 300]
    assert [i + 1 for i, k in enumerate(kinds) if k == 6] == [2, 10, 26, 58, 122, 250]


def test_gap_checks_ride_on_the_residual_checks(planlib):
    t = trace(planlib, 1000, 1000, 1000, reg_kind=1, checking=1, check_every=100, gap_every=3)
    ends = [(i + 1, bool(f & 4)) for i, f in enumerate(t.col("flags")) if f & 1]
    assert [e for e, g in ends if g] == [300, 600, 900] and len(ends) == 10
    # a gap trace without a tolerance still cuts the solve into stretches
    t = trace(planlib, 1000, 1000, 250, reg_kind=1, checking=0, check_every=100, gap_every=1)
    assert [(i + 1, bool(f & 4)) for i, f in enumerate(t.col("flags")) if f & 1] == [(100, True), (200, True), (250, False)]


def test_point_clouds_and_warm_starts(planlib):
    t = trace(planlib, 3000, 3000, 5, from_points=1, reg_kind=1, checking=0)
    assert set(t.col("sweep")) == {POINTS} and t.col("prev_sums") == [0, 1, 1, 1, 1] and set(t.col("update")) == {MERGED_TILES}
    t = trace(planlib, 3000, 3000, 5, from_points=1, reg_kind=1, checking=0, skip_unchanged=0)
    assert set(t.col("prev_sums")) == {0}
    t = trace(planlib, 2300, 2500, 4, warm=1, reg_kind=1, checking=0, screening=1)
    # the warm start's sums of X_0 serve as flags for the first sweep, which is no "first" sweep (X_0 is read)
    assert t.col("first") == [0, 0, 0, 0] and t.col("prev_sums")[0] == 1 and t.col("kind")[0] == 6
    t = trace(planlib, 5000, 5000, 3, warm=1, reg_kind=2, slab_k=4, nruns=10, checking=0)
    assert t.col("prev_sums") == [0, 1, 1]  # (those sums are per 256 columns, the slab kernel's flags per 32)
    # a warm start with the cost from point clouds: X_0 is read where its sums say so, and the sweep records bounds
    t = trace(planlib, 3000, 3000, 4, from_points=1, warm=1, reg_kind=1, checking=0, screening=1)
    assert set(t.col("sweep")) == {POINTS} and t.col("first") == [0, 0, 0, 0] and t.col("prev_sums") == [1, 1, 1, 1]
    assert t.col("refresh") == [1, 1, 1, 1] and set(t.col("kind")) == {9}


def test_label_analysis(planlib):
    def labels(arr, classes, max_runs=1000, force=0):
        a = np.ascontiguousarray(arr, dtype=np.int32)
        nruns = ctypes.c_int()
        k = planlib.drot_plan_labels(a.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), len(a), classes, max_runs, force,
                                     ctypes.byref(nruns))
        return k, nruns.value

    assert labels(np.repeat(np.arange(10), 500), 10) == (4, 10)       # 500 rows: 4 per row lane
    assert labels(np.repeat(np.arange(3), 128), 3) == (1, 3)
    assert labels(np.repeat(np.arange(2), 1024), 2) == (8, 2)
    assert labels(np.repeat(np.arange(2), 1025), 2) == (0, 2)         # too long for the registers
    assert labels([0, 0, 1, 1, 0], 2) == (0, 3)                       # a class in two runs
    assert labels(np.repeat(np.arange(10), 500), 10, force=1) == (0, 10)
    assert labels(np.repeat(np.arange(10), 5), 10, max_runs=9) == (0, 10)
    assert labels([0, 1, 2, 3], 3)[0] == -1 and labels([0, -1], 3)[0] == -1
    assert labels([2, 2, 2], 5) == (1, 1)                             # unused classes are fine


def test_class_chunks_of_the_two_pass_group_lasso_path(planlib):
    rng = np.random.default_rng(7)
    for m, classes in ((1, 1), (50, 3), (1000, 7), (333, 40)):
        labels = np.ascontiguousarray(rng.integers(0, classes, size=m), dtype=np.int32)
        if classes > 2:
            labels[labels == 1] = 0  # an empty class
        perm = np.zeros(m, dtype=np.int32)
        cap = m // 16 + classes + 1
        chunk_start = np.zeros(cap + 1, dtype=np.int32)
        class_first = np.zeros(classes + 1, dtype=np.int32)
        ip = ctypes.POINTER(ctypes.c_int)
        nchunks = planlib.drot_plan_chunks(labels.ctypes.data_as(ip), m, classes, perm.ctypes.data_as(ip),
                                           chunk_start.ctypes.data_as(ip), cap, class_first.ctypes.data_as(ip))
        assert nchunks >= 1 and class_first[0] == 0 and class_first[classes] == nchunks and chunk_start[nchunks] == m
        assert sorted(perm.tolist()) == list(range(m))          # a permutation of the rows
        for c in range(classes):
            rows = []
            for k in range(class_first[c], class_first[c + 1]):
                chunk = perm[chunk_start[k]:chunk_start[k + 1]].tolist()
                assert 1 <= len(chunk) <= 16
                rows += chunk
            assert rows == np.flatnonzero(labels == c).tolist()  # every row of the class once, in ascending order


def test_point_cloud_variant_screens_once_the_plan_is_sparse(planlib):
    t = trace(planlib, 20000, 20000, 200, from_points=1, reg_kind=1, checking=0, densities=(0.9, 0.6, 0.2, 0.05))
    kinds = t.col("kind")
    assert kinds[0] == 0 and set(kinds[1:96]) == {9}        # full sweeps, all but the first recording the bounds
    # lean from sweep 97 (the status after 64 iterations is read while the stretch to 96 is queued), on the bounds
    # of sweep 96; they are renewed by one full sweep after 8 sweeps, then after 16, 32, ...
    assert kinds[96:103] == [8] * 7 and kinds[103] == 9 and kinds[104:119] == [8] * 15 and kinds[119] == 9
    assert t.col("sweep")[96] == POINTS_LEAN and t.col("sweep")[103] == POINTS
    # column sums: eight 32-row tiles of the full sweep are added first, as the strips of the screened sweep store them
    assert t.col("ra")[5] == 625 * 16 + 8 and t.col("ra")[100] == 79 * 16 + 1 and t.col("ra")[0] == 625 * 16 + 8
    # one launch for the vector update: the sweeps store the totals of their tiles (the screened one of its strips)
    assert set(t.col("update")) == {MERGED_TILES} and set(t.col("tilesum")) == {1}
    # small problems, or with the screening off: the full sweep only, column sums ungrouped
    t = trace(planlib, 3000, 3000, 40, from_points=1, reg_kind=1, checking=0, densities=(0.05,))
    assert set(t.col("kind")) == {0} and set(t.col("ra")) == {94 * 16 + 8}
    t = trace(planlib, 20000, 20000, 120, from_points=1, reg_kind=1, checking=0, screening=0, densities=(0.05,))
    assert set(t.col("kind")) == {0}
    # a continued call goes on with the bounds it finds
    first = trace(planlib, 20000, 20000, 100, from_points=1, reg_kind=1, checking=0, densities=(0.9, 0.6, 0.2, 0.05))
    cont = trace(planlib, 20000, 20000, 20, from_points=1, reg_kind=1, checking=0, resume=1, carry=first.carry, densities=(0.05,))
    assert cont.col("kind")[0] == 8
