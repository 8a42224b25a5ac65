// Host-only wrapper of the launch planner (drot_plan.h) for tests that run without a GPU.
//
// drot_plan_trace() replays the host loop of a solve -- stretches, sweeps, statuses read one stretch
// late -- with the densities and the stop a test scripts in place of what a GPU would report, and
// writes down what the planner decided for every sweep.  Built with a plain C++ compiler into
// libdrot_plan.so; the product library includes the same header and does not use this file.
#include <cstring>

#include "drot_plan.h"

using namespace drot_plan;

extern "C" {

// problem[14]: m, n, reg_kind, from_points, warm, resume, has_weights, c_on_lines, x_on_lines, slab_k,
//              nruns, feedback, checking, max_iters
// options[9]:  check_every, resident, fused_update, skip_cost, skip_unchanged, screening, nontemporal,
//              force_two_pass, gap_every
// carry[8] (in and out): dense_plan, plan_density * 1e6, epoch_gen, refresh_period, sums_valid, sums_strip,
//              lines_valid, iters_done
// densities[nstatus]: what the k-th status of the call reports (fraction of nonzero row segments);
//              statuses past the end repeat the last one.  stop_at_status >= 0: that status reports convergence.
// rows [capacity][12]: sweep, mode, first, prev_sums, lines_in, refresh, pro, tilesum, update, ra_ntr * 16 + ra_cgroup,
//              profile_kind, flags (1: last sweep of a stretch, 2: that stretch is a probe, 4: its status carries the gap,
//              8: a gap evaluated there may take the lean pass, 16: with the lean sweep's line flags)
// statics[10]: nseg, ntr, resident, pad_c, pad_x, small, fused, may_screen, adaptive, nt
// Returns the number of sweeps (launches) planned, or -1 if capacity was too small.
int drot_plan_trace(const int* problem, const int* options, long long* carry, const double* densities, int nstatus,
                    int stop_at_status, int* rows, int capacity, int* statics, int* iters_done) {
  Problem P;
  P.m = problem[0];
  P.n = problem[1];
  P.reg_kind = problem[2];
  P.from_points = problem[3] != 0;
  P.warm = problem[4] != 0;
  P.resume = problem[5] != 0;
  P.has_weights = problem[6] != 0;
  P.c_on_lines = problem[7] != 0;
  P.x_on_lines = problem[8] != 0;
  P.slab_k = problem[9];
  P.nruns = problem[10];
  P.feedback = problem[11] != 0;
  P.checking = problem[12] != 0;
  P.max_iters = problem[13];
  P.tilesum_half = (size_t)ceil_div(P.n, kSegCols) * (size_t)ceil_div(P.m, kTileRows);
  if (P.tilesum_half < 4096) P.tilesum_half = 4096;
  Options O;
  O.check_every = options[0];
  O.resident = options[1];
  O.fused_update = options[2];
  O.skip_cost = options[3];
  O.skip_unchanged = options[4];
  O.screening = options[5];
  O.nontemporal = options[6];
  O.force_two_pass = options[7];
  O.gap_every = options[8];
  Carry C;
  C.dense_plan = carry[0] != 0;
  C.plan_density = (double)carry[1] * 1e-6;
  C.epoch_gen = carry[2];
  C.refresh_period = (int)carry[3];
  C.sums_valid = carry[4] != 0;
  C.sums_strip = (int)carry[5];
  C.lines_valid = carry[6] != 0;
  C.iters_done = carry[7];

  const Static S = make_static(P, O);
  statics[0] = S.nseg;
  statics[1] = S.ntr;
  statics[2] = S.resident;
  statics[3] = S.pad_c;
  statics[4] = S.pad_x;
  statics[5] = S.small;
  statics[6] = S.fused;
  statics[7] = S.may_screen;
  statics[8] = S.adaptive;
  statics[9] = S.nt;
  State T = start_state(S, P, C);
  int nrows = 0, checks = 0;
  bool converged = false;
  bool was_probe[2] = {false, false};
  int status_iters[2] = {0, 0};
  int slot = 0, stop_iters = -1;
  while (T.k < P.max_iters && !converged) {
    const Stretch R = next_stretch(S, P, O, T);
    const int k_end = T.k + R.chunk;
    for (int c = 0; T.k < k_end; ++c) {
      const Step Q = next_sweep(S, P, O, T, R, c);
      if (nrows >= capacity) return -1;
      int* r = rows + (size_t)nrows * 12;
      r[0] = Q.sweep;
      r[1] = Q.mode;
      r[2] = Q.first;
      r[3] = Q.prev_sums;
      r[4] = Q.lines_in;
      r[5] = Q.refresh;
      r[6] = Q.pro;
      r[7] = Q.tilesum;
      r[8] = Q.update;
      r[9] = Q.ra_ntr * 16 + Q.ra_cgroup;
      r[10] = Q.profile_kind;
      const GapPass G = T.k == k_end ? gap_pass(S, P, T) : kGapDense;
      r[11] = (T.k == k_end ? 1 : 0) | (T.k == k_end && R.probe ? 2 : 0) | (T.k == k_end && R.gap ? 4 : 0) |
              (G != kGapDense ? 8 : 0) | (G == kGapLeanLines ? 16 : 0);
      ++nrows;
    }
    if (S.status_at_checks) {
      was_probe[slot] = R.probe;
      status_iters[slot] = T.k;
      if (checks == stop_at_status && stop_iters < 0) stop_iters = T.k;  // (the device raises its stop flag here)
      if (checks > 0 && P.feedback) {
        // the host reads the previous stretch's status while this one is queued
        const int prev = checks - 1;
        if (stop_at_status >= 0 && prev >= stop_at_status) converged = true;
        const double d = nstatus > 0 ? densities[prev < nstatus ? prev : nstatus - 1] : 0.0;
        on_status(S, T, d, was_probe[slot ^ 1]);
      }
      slot ^= 1;
      ++checks;
    }
  }
  const bool stopped = stop_iters >= 0;
  const int reported = stopped ? stop_iters : T.k;
  const Carry F = finish(S, P, T, stopped, reported);
  carry[0] = F.dense_plan;
  carry[1] = (long long)(F.plan_density * 1e6);
  carry[2] = F.epoch_gen;
  carry[3] = F.refresh_period;
  carry[4] = F.sums_valid;
  carry[5] = F.sums_strip;
  carry[6] = F.lines_valid;
  carry[7] = F.iters_done;
  *iters_done = reported;
  (void)status_iters;
  return nrows;
}

// Label analysis of the group-lasso path: returns slab_k (0: two-pass), -1 for a label out of range;
// *nruns receives the number of runs.
int drot_plan_labels(const int* labels, int m, int num_classes, int max_runs, int force_two_pass, int* nruns) {
  const LabelRuns L = analyze_labels(labels, m, num_classes, max_runs, force_two_pass != 0);
  if (!L.valid) return -1;
  *nruns = (int)L.start.size();
  return L.slab_k;
}

// The chunk tables of the two-pass group-lasso path: perm[m], chunk_start[nchunks + 1] (capacity
// cap_chunks + 1), class_first[num_classes + 1].  Returns the number of chunks, or -1 if they do not fit.
int drot_plan_chunks(const int* labels, int m, int num_classes, int* perm, int* chunk_start, int cap_chunks,
                     int* class_first) {
  const ClassChunks K = chunk_classes(labels, m, num_classes);
  if (K.nchunks() > cap_chunks) return -1;
  std::memcpy(perm, K.perm.data(), sizeof(int) * (size_t)m);
  std::memcpy(chunk_start, K.chunk_start.data(), sizeof(int) * K.chunk_start.size());
  std::memcpy(class_first, K.class_first.data(), sizeof(int) * K.class_first.size());
  return K.nchunks();
}

}  // extern "C"
