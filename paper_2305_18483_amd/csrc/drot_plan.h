// Launch planning for the Douglas-Rachford OT solver: which kernel runs which sweep.
//
// Pure host logic, no HIP in here: drot.hip includes this header and enqueues what it decides, and
// the same header compiles with a plain C++ compiler so that every path and every switch between
// paths can be exercised without a GPU (drot_plan_host.cpp wraps it for that).
//
// One iteration of the method is a sweep over the plan (eq. (8)) followed by the vector update of
// eq. (6).  The arithmetic of an iteration is fixed; what varies is the kernel that performs it:
//
//   Resident    tiny problems: one workgroup, X and C in registers, a whole stretch per launch
//   Pro32       small problems: 32-row tiles, the vector update of the previous iteration fused
//               into the head of the sweep (one launch per iteration)
//   Plain32     32-row tiles, every byte moved; also the first sweep of every cold start and the
//               two sweeps of an even/odd pair (mode 1 stores X - rho*C, mode 2 reads it, no C)
//   Tall64      64-row tiles; all-zero row segments of X neither read nor written back
//   Screened8   the same tiles; row segments certified to stay zero also skip their reads of C;
//               with `refresh` it reads all of C and records the bounds the certificates use
//   Lean        one wave per 64 x 256 tile, for plans known to be sparse; renews its bounds itself
//   Points      cost recomputed from point clouds on the matrix cores (32-row tiles); with `refresh` it
//               also records the screening bounds
//   PointsLean  the same cost for the rows a certificate does not cover only (256-row strips)
//   Slab        group lasso, a whole class x 32 columns resident in one workgroup
//   TwoPass     group lasso, any labels: norms first, then the scaled update
//
// The choice depends on the problem (sizes, regularizer, alignment), on the options, on what the
// previous sweeps left in memory (row-segment sums, line flags, bounds) and, where the host reads
// the status block during the solve, on the density of the plan it reports.
#ifndef DROT_PLAN_H_
#define DROT_PLAN_H_

#include <cstddef>
#include <vector>

namespace drot_plan {

// Geometry the kernels are written for (drot.hip checks these against the kernels' own constants).
constexpr int kSegCols = 256;         // columns of a row segment / of a tile
constexpr int kTileRows = 32;         // rows of the small tile
constexpr int kTallTileRows = 64;     // rows of the tile of Tall64, Screened8 and Lean
constexpr int kAlignElems = 32;       // rows must start on 128-byte lines
constexpr int kSlabCols = 32;         // columns of a group-lasso slab
constexpr int kSlabRowLanes = 128;    // row lanes of the slab kernel (K = 1, 2, 4, 8 rows per lane)
constexpr int kSlabMaxRows = 1024;    // longest class the slab kernel holds
constexpr int kResidentMaxRows = 128, kResidentCols = 256;
constexpr int kColGroup = 4;          // the lean sweep adds the column sums of four tiles before it stores
constexpr int kStripRows = 256;       // rows of a strip of the point-cloud variant's screened sweep
constexpr int kPointsColGroup = 8;    // ... which adds the column sums of its eight 32-row tiles before it stores
constexpr size_t kScreenFrom = (size_t)11 << 20;  // screening on automatic: from this many entries up
constexpr int kFirstRefreshPeriod = 8, kMaxRefreshPeriod = 1024;
constexpr int kEarlyLooksUntil = 512;  // cold starts: extra density readings over this many iterations

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

enum Regularizer { kNone = 0, kQuadratic = 1, kGroupLasso = 2 };

struct Options {
  int check_every = 100;
  int resident = -1;        // -1 automatic, 0 never
  int fused_update = -1;    // -1 automatic, 0 never
  int skip_cost = -1;       // even/odd pairs: -1 by density, 0 never, 1 wherever they apply
  int skip_unchanged = -1;  // zero-segment skipping: -1/1 on, 0 off
  int screening = -1;       // -1 from kScreenFrom entries up, 0 never, 1 always, k >= 2 always, renewed at least every k
  int nontemporal = -1;     // -1 by size, 0 never, 1 always
  int force_two_pass = 0;   // group lasso: never the slab kernel
  int gap_every = 0;        // objective / gap / dual residual at every gap_every-th residual check (0: only at the end)
};

struct Problem {
  int m = 0, n = 0;
  int reg_kind = kNone;
  bool from_points = false;   // cost recomputed from point clouds
  bool warm = false;          // caller-supplied starting point
  bool resume = false;        // continues the previous solve on the handle
  bool has_weights = false;   // weighted l1 term: the solve runs on a working copy C + W
  bool c_on_lines = true;     // base address of C is a multiple of 128
  bool x_on_lines = true;     // base address of X_out is a multiple of 128
  int slab_k = 0;             // group lasso: rows per lane of the slab kernel, 0 = two-pass path
  int nruns = 0;              // group lasso: runs of equal labels
  size_t tilesum_half = 0;    // capacity of one half of the tile-total buffer
  bool feedback = true;       // the host reads the status block during the solve
  bool checking = false;      // a tolerance was given
  int max_iters = 0;
};

// What a solve hands to the next one on the same handle (continued solves).
struct Carry {
  bool dense_plan = false;
  double plan_density = -1.0;
  long long epoch_gen = -1;      // sweep that last recorded the screening bounds
  int refresh_period = kFirstRefreshPeriod;
  bool sums_valid = false;       // the row-segment sums of the last sweep describe the X in memory
  int sums_strip = 0;            // ... in pieces of this many columns
  bool lines_valid = false;      // the same for the lean sweep's line flags
  long long iters_done = 0;
};

// Decisions that hold for the whole call.
struct Static {
  int nseg = 0, ntr = 0, ntiles = 0, ntr_tall = 0;
  int nbm = 0, nbn = 0;          // workgroups of the reduction: 64 rows resp. 64 columns each
  int ld_pad = 0;                // pitch of the padded working copies
  bool nt = false;               // non-temporal accesses
  bool resident = false;
  bool pad_c = false, pad_x = false;
  int nstrips = 0;
  bool small_slab = false, small = false, fused = false;
  bool can_pair = false, adaptive_pairs = false, may_screen = false, adaptive = false;
  bool points_screen = false;    // point-cloud variant: screened sweeps once the plan is known to be sparse
  int refresh_max = kMaxRefreshPeriod;
  int sums_strip = kSegCols;
  bool status_at_checks = false; // the stretches end with a status kernel (stopping test and / or density)
};

// Non-temporal accesses pay off once X and C together no longer fit the 256 MB memory-side cache.
// Measured crossover on MI355X: cacheable wins at 8mn = 290 MB (7.2 vs 6.1 TB/s), non-temporal at
// 393 MB (6.1 vs 5.7 TB/s).
inline bool use_nontemporal(int m, int n) { return 8.0 * (double)m * (double)n > 320.0 * 1024 * 1024; }

inline Static make_static(const Problem& P, const Options& O) {
  Static S;
  const int m = P.m, n = P.n;
  S.nseg = ceil_div(n, kSegCols);
  S.ntr = ceil_div(m, kTileRows);
  S.ntiles = S.nseg * S.ntr;
  S.ntr_tall = ceil_div(m, kTallTileRows);
  S.nbm = ceil_div(m, 64);
  S.nbn = ceil_div(n, 64);
  S.ld_pad = ceil_div(n, kAlignElems) * kAlignElems;
  S.nt = O.nontemporal < 0 ? use_nontemporal(m, n) : O.nontemporal != 0;
  S.resident = O.resident != 0 && P.reg_kind != kGroupLasso && !P.from_points && m <= kResidentMaxRows &&
               n <= kResidentCols;
  const bool rows_off_lines = n % kAlignElems != 0;
  S.pad_c = P.has_weights || (!S.resident && !P.from_points && (rows_off_lines || !P.c_on_lines));
  S.pad_x = !S.resident && (rows_off_lines || !P.x_on_lines);
  S.nstrips = ceil_div(n, kSlabCols);
  S.small_slab = P.slab_k && S.nstrips <= 64 && P.nruns <= 64 && S.nstrips * P.nruns <= 4096;
  S.small = S.small_slab || (P.reg_kind != kGroupLasso && !P.from_points && S.ntr <= 64 && S.ntiles <= 4096);
  S.fused = S.small && O.fused_update != 0;
  S.can_pair = P.reg_kind != kGroupLasso && !S.fused && !P.from_points;
  S.adaptive_pairs = P.feedback && S.can_pair && !S.small && O.skip_cost == -1 && O.skip_unchanged != 0;
  S.may_screen = S.can_pair && !S.small && O.skip_cost != 1 && O.skip_unchanged != 0 &&
                 (O.screening > 0 || (O.screening == -1 && (size_t)m * (size_t)n >= kScreenFrom));
  S.points_screen = P.from_points && O.skip_unchanged != 0 &&
                    (O.screening > 0 || (O.screening == -1 && (size_t)m * (size_t)n >= kScreenFrom));
  S.adaptive = P.feedback && (S.adaptive_pairs || S.may_screen || S.points_screen);
  S.refresh_max = O.screening >= 2 ? O.screening : kMaxRefreshPeriod;
  S.sums_strip = P.slab_k ? kSlabCols : kSegCols;
  S.status_at_checks = P.checking || S.adaptive || O.gap_every > 0;
  return S;
}

// What changes from sweep to sweep.
struct State {
  long long k_base = 0;          // iterations the state on the handle had seen before this call
  int k = 0;                     // iterations enqueued by this call
  long long sums_gen = -1;       // sweep whose row-segment sums describe the plain X in memory, or -1
  long long lines_gen = -1;      // the same for the lean sweep's line flags
  long long epoch_gen = -1;      // sweep that last recorded the screening bounds (host's record)
  int refresh_period = kFirstRefreshPeriod;
  bool dense_plan = false;       // the last status reported a dense plan: even/odd pairs
  double plan_density = -1.0;    // fraction of nonzero row segments, once a status has come back
  bool materialized = true;      // phi, varphi, a, b, theta in memory are complete for the sweeps done
  bool norms_pending = false;    // the last vector update left the residual norms as per-workgroup sums
};

inline State start_state(const Static& S, const Problem& P, const Carry& carry) {
  State T;
  T.k_base = P.resume ? carry.iters_done : 0;
  T.dense_plan = P.resume && carry.dense_plan;
  T.plan_density = P.resume ? carry.plan_density : -1.0;
  // (a continued solve starts from the X the last one returned, so its row-segment sums still hold;
  // the warm start's sums are those of 256-column segments)
  T.sums_gen = P.warm ? (P.slab_k ? -1 : 0)
                      : (P.resume && carry.sums_valid && carry.sums_strip == S.sums_strip) ? T.k_base : -1;
  T.lines_gen = (P.resume && carry.lines_valid && T.sums_gen >= 0) ? T.k_base : -1;
  T.epoch_gen = P.resume ? carry.epoch_gen : -1;
  T.refresh_period = P.resume ? carry.refresh_period : kFirstRefreshPeriod;
  if (T.refresh_period > S.refresh_max) T.refresh_period = S.refresh_max;
  return T;
}

// A stretch: the sweeps up to the next status (stopping test at the multiples of check_every; over
// the first iterations of a cold start also looks at the density only, after 16 and then every 32
// iterations: a plan goes through phases -- empty, dense, then as sparse as it will be -- and a wrong
// choice of sweep should not last a whole check interval).
struct Stretch {
  int chunk = 0;
  bool probe = false;      // ends with a status for the host's choice of sweep only (no stopping test)
  bool skip_cost = false;  // even/odd pairs in this stretch
  bool tall = false;       // 64-row tiles in this stretch
  bool gap = false;        // the status at its end carries objective, gap and dual residual
};

inline Stretch next_stretch(const Static& S, const Problem& P, const Options& O, const State& T) {
  Stretch R;
  const int k = T.k;
  R.chunk = P.max_iters - k;
  if (S.status_at_checks) {
    const int to_check = O.check_every - k % O.check_every;  // the tests stay at multiples of check_every
    if (to_check < R.chunk) R.chunk = to_check;
    if (S.adaptive && !P.resume && k < kEarlyLooksUntil) {
      const int next = k < 16 ? 16 : (k / 32 + 1) * 32;
      if (next - k < R.chunk) {
        R.chunk = next - k;
        R.probe = true;
      }
    }
  }
  R.skip_cost = S.can_pair && (O.skip_cost == 1 || (S.adaptive_pairs && T.dense_plan));
  R.tall = !S.small && !R.skip_cost && !P.from_points && P.reg_kind != kGroupLasso && O.skip_unchanged != 0;
  const int end = k + R.chunk;
  R.gap = !R.probe && O.gap_every > 0 && end % O.check_every == 0 && (end / O.check_every) % O.gap_every == 0;
  return R;
}

enum Sweep { kResident = 0, kPro32, kPlain32, kTall64, kScreened8, kLean, kPoints, kSlab, kTwoPass, kPointsLean };
enum Update { kNoUpdate = 0, kSeparate, kMergedSlab, kMergedTiles };

struct Step {
  Sweep sweep = kPlain32;
  long long sw = 0;        // this sweep produces X_sw; its sums live in the buffers of parity sw & 1
  bool first = false;      // X_0 = 0: nothing to read
  int mode = 0;            // even/odd scheme: 0 plain, 1 stores X - rho*C, 2 reads it without C
  bool prev_sums = false;  // the row-segment sums of sweep sw - 1 tell which pieces of X are zero
  bool lines_in = false;   // lean: the line flags of sweep sw - 1 are valid
  bool refresh = false;    // Screened8: reads all of C and records the bounds
  bool pro = false;        // the vector update of sweep sw - 1 rides along at the head of this sweep
  bool tilesum = false;    // the sweep stores the totals of its tiles
  Update update = kNoUpdate;
  int ra_ntr = 0;          // rows of column partials the sweep leaves, and how the reduction groups them
  int ra_cgroup = 1;
  int tt_rows = 0, tt_group = 1;  // merged update: rows of tile totals and their grouping
  int ctl_mode = 0;        // merged update: 0 nothing, 1 after a host-ordered refresh, 2 after a lean sweep
  int profile_kind = 0;    // what drot_get_profile reports for this sweep
  int iters = 1;           // iterations the launch covers (a resident stretch: all of it)
};

// The c-th sweep of stretch R (c = 0 .. chunk-1).  Advances T.
inline Step next_sweep(const Static& S, const Problem& P, const Options& O, State& T, const Stretch& R, int c) {
  Step Q;
  const long long sw = T.k_base + T.k + 1;
  Q.sw = sw;
  Q.first = sw == 1 && !P.warm;
  Q.tilesum = S.small;
  Q.ra_ntr = P.slab_k ? P.nruns : S.ntr;
  Q.ra_cgroup = 1;
  const bool skipping = O.skip_unchanged != 0;
  bool tiles64 = false, lean = false, slab_totals = false;
  if (S.resident) {
    Q.sweep = kResident;
    Q.iters = R.chunk;
    Q.first = sw == 1 && !P.warm;
    Q.profile_kind = 3;
    T.k += R.chunk;
    return Q;  // (the resident kernel does its own vector updates)
  }
  if (P.from_points) {
    Q.sweep = kPoints;
    Q.prev_sums = T.sums_gen == sw - 1 && skipping;
    T.sums_gen = sw;
    // (the reduction adds the eight 32-row tiles of a 256-row strip first, as the screened sweep stores them: the
    // same bits with and without the screening)
    Q.ra_cgroup = kPointsColGroup;
    if (S.points_screen) {
      // every full sweep but the first records the bounds; the screened sweep runs on them while the plan is
      // known to be sparse, until they are due for renewal (after 8, 16, 32, ... sweeps: varphi moves fast at first)
      const bool due = T.epoch_gen < 0 || sw - T.epoch_gen >= T.refresh_period;
      const bool lean_points = !Q.first && !due && Q.prev_sums && T.plan_density >= 0.0 && T.plan_density < 0.25;
      if (lean_points) {
        Q.sweep = kPointsLean;
        Q.profile_kind = 8;
        Q.ra_ntr = ceil_div(P.m, kStripRows);
        Q.ra_cgroup = 1;
      } else {
        if (!Q.first) {
          Q.refresh = true;
          Q.profile_kind = 9;
          if (T.epoch_gen >= 0 && due)
            T.refresh_period = T.refresh_period * 2 < S.refresh_max ? T.refresh_period * 2 : S.refresh_max;
          T.epoch_gen = sw;
        }
      }
    }
  } else if (P.slab_k) {
    Q.sweep = kSlab;
    // (large problems: the slab totals give eta, one launch then does the whole vector update)
    slab_totals = !S.small && (size_t)S.nstrips * (size_t)P.nruns <= P.tilesum_half;
    if (slab_totals) Q.tilesum = true;
    Q.prev_sums = T.sums_gen == sw - 1 && skipping;
    Q.pro = !T.materialized;
    T.sums_gen = sw;
  } else if (P.reg_kind == kGroupLasso) {
    Q.sweep = kTwoPass;
  } else if (!T.materialized) {
    Q.sweep = kPro32;
    Q.pro = true;
    T.sums_gen = sw;
  } else {
    // even/odd scheme: inside a stretch the sweeps pair up as (store X - rho*C, then read it without
    // C); an odd stretch starts with one plain sweep, so X is plain at every stretch end
    int mode = 0;
    if (R.skip_cost) {
      const int paired_from = R.chunk & 1;
      if (c >= paired_from) mode = ((c - paired_from) & 1) ? 2 : 1;
    }
    Q.mode = mode;
    const bool screened = mode == 0 && R.tall && !Q.first && S.may_screen;
    Q.prev_sums = mode == 0 && T.sums_gen == sw - 1 && skipping;
    T.sums_gen = mode == 1 ? -1 : sw;
    // once the plan is known to be sparse (and bounds exist): one wave per tile
    lean = screened && T.epoch_gen >= 0 && Q.prev_sums && T.plan_density >= 0.0 && T.plan_density < 0.25;
    Q.refresh = screened && !lean && (T.epoch_gen < 0 || sw - T.epoch_gen >= T.refresh_period);
    tiles64 = R.tall && !Q.first && mode == 0;
    if (tiles64) Q.tilesum = true;
    Q.profile_kind = screened ? (Q.refresh ? 6 : 5) : tiles64 ? 4 : mode;
    if (screened) {
      if (Q.refresh) {
        // (varphi moves fast at first: the bounds are renewed after 8 sweeps, then 16, 32, ...)
        if (T.epoch_gen >= 0)
          T.refresh_period = T.refresh_period * 2 < S.refresh_max ? T.refresh_period * 2 : S.refresh_max;
        T.epoch_gen = sw;
      }
      if (lean) {
        Q.sweep = kLean;
        Q.lines_in = T.lines_gen == sw - 1;
        T.lines_gen = sw;
        Q.profile_kind = 7;
      } else {
        Q.sweep = kScreened8;
      }
    } else if (tiles64) {
      Q.sweep = kTall64;
    } else {
      Q.sweep = kPlain32;
    }
    // (the 64-row tiles leave fewer rows of column partials, which the reduction adds up in groups
    // of four; the lean sweep stores one row per group)
    Q.ra_ntr = lean ? ceil_div(S.ntr_tall, kColGroup) : tiles64 ? S.ntr_tall : S.ntr;
    Q.ra_cgroup = (tiles64 && !lean) ? kColGroup : 1;
  }
  // the vector update: separate kernels, one merged launch, or left to the head of the next sweep
  if (!S.fused || c == R.chunk - 1) {
    if (slab_totals) {
      Q.update = kMergedSlab;
      Q.tt_rows = P.nruns;
      Q.tt_group = 1;
    } else if (tiles64) {
      Q.update = kMergedTiles;
      Q.tt_rows = lean ? ceil_div(S.ntr_tall, kColGroup) : S.ntr_tall;
      Q.tt_group = lean ? 1 : kColGroup;
      Q.ctl_mode = lean ? 2 : Q.refresh ? 1 : 0;
    } else if (P.from_points) {
      // (the point-cloud sweeps store the totals of their 32-row tiles, the screened one of its strips of eight)
      Q.update = kMergedTiles;
      Q.tilesum = true;
      Q.tt_rows = Q.sweep == kPointsLean ? ceil_div(P.m, kStripRows) : S.ntr;
      Q.tt_group = Q.sweep == kPointsLean ? 1 : kPointsColGroup;
    } else {
      Q.update = kSeparate;
    }
    T.norms_pending = true;
    T.materialized = true;
  } else {
    T.materialized = false;
  }
  T.k += 1;
  return Q;
}

// A status has come back: the density of the plan it reports steers the next stretches
// (hysteresis: the break-even between the skipping sweeps and the even/odd pairs is at about three
// quarters of the row segments nonzero; the early looks never start the pairs: every plan is dense
// in its first iterations).
inline void on_status(const Static& S, State& T, double density, bool was_probe) {
  if (!S.adaptive) return;
  T.plan_density = density;
  if (density > 0.7 && !was_probe) T.dense_plan = S.adaptive_pairs;
  else if (density < 0.5) T.dense_plan = false;
}

// What the handle keeps for a continued solve.  iters: what the final status reports (an early stop
// leaves the sweeps queued behind it undone: be conservative about everything they would have left).
inline Carry finish(const Static& S, const Problem& P, const State& T, bool converged, int iters) {
  Carry C;
  C.dense_plan = T.dense_plan;
  C.plan_density = T.plan_density;
  const bool epoch_ran = T.epoch_gen <= T.k_base + (long long)iters;
  C.epoch_gen = (converged || !epoch_ran) ? -1 : T.epoch_gen;
  C.refresh_period = (converged || !epoch_ran) ? kFirstRefreshPeriod : T.refresh_period;
  C.sums_valid = !converged && P.max_iters > 0 && T.sums_gen == T.k_base + T.k;
  C.lines_valid = C.sums_valid && T.lines_gen == T.k_base + T.k;
  C.sums_strip = S.sums_strip;
  C.iters_done = T.k_base + (P.max_iters == 0 ? 0 : iters);
  return C;
}

// Which pass evaluates the terms of the duality gap for the state after the sweeps enqueued so far.  The
// lean pass visits only the row segments a screening bound does not certify to contribute nothing; it
// needs the bounds of an epoch and flags that describe the X in memory: the line flags of a lean sweep,
// or the row-segment sums of any sweep that leaves them per 256 columns.  (After a stop raised on the
// device the sweeps enqueued behind it did not run and the host's record of the flags is ahead of the
// memory: the caller falls back to the dense pass then.)
enum GapPass { kGapDense = 0, kGapLeanLines, kGapLeanSums };

inline GapPass gap_pass(const Static& S, const Problem& P, const State& T) {
  const long long cur = T.k_base + T.k;
  if (!S.may_screen || P.from_points || P.reg_kind == kGroupLasso || P.slab_k) return kGapDense;
  if (T.epoch_gen < 0 || T.epoch_gen > cur || cur < 1) return kGapDense;
  if (T.lines_gen == cur) return kGapLeanLines;
  if (T.sums_gen == cur) return kGapLeanSums;
  return kGapDense;
}

// Group lasso: the labels of the m rows as runs of equal labels.  The slab kernel applies when every
// class is one run of at most kSlabMaxRows rows (and the runs fit the workspace).
struct LabelRuns {
  bool valid = true;              // every label in [0, num_classes)
  std::vector<int> start, len;    // the runs
  int slab_k = 0;                 // rows per lane of the slab kernel, 0: two-pass path
};

// Two-pass path (any labels): the rows of every class, in ascending order, cut into chunks of at most
// kNormChunkRows rows.  The first pass adds up the squared entries of one chunk per wave, the second
// adds the chunks of a class in order: the group norms come out the same in every run (no atomics).
constexpr int kNormChunkRows = 16;
struct ClassChunks {
  std::vector<int> perm;          // [m] the rows sorted by (class, row)
  std::vector<int> chunk_start;   // [nchunks + 1] offsets into perm
  std::vector<int> class_first;   // [num_classes + 1] the chunks of class c are class_first[c] .. class_first[c+1] - 1
  int nchunks() const { return (int)chunk_start.size() - 1; }
};

inline ClassChunks chunk_classes(const int* labels, int m, int num_classes) {
  ClassChunks K;
  std::vector<int> count((size_t)num_classes + 1, 0);
  for (int i = 0; i < m; ++i) ++count[(size_t)labels[i] + 1];
  for (int c = 0; c < num_classes; ++c) count[(size_t)c + 1] += count[(size_t)c];  // first position of every class
  K.perm.resize((size_t)m);
  std::vector<int> next(count.begin(), count.end() - 1);
  for (int i = 0; i < m; ++i) K.perm[(size_t)next[(size_t)labels[i]]++] = i;       // stable: rows stay in order
  K.class_first.push_back(0);
  K.chunk_start.push_back(0);
  for (int c = 0; c < num_classes; ++c) {
    for (int b = count[(size_t)c]; b < count[(size_t)c + 1]; b += kNormChunkRows) {
      const int e = b + kNormChunkRows < count[(size_t)c + 1] ? b + kNormChunkRows : count[(size_t)c + 1];
      K.chunk_start.push_back(e);
    }
    K.class_first.push_back(K.nchunks());
  }
  return K;
}

inline LabelRuns analyze_labels(const int* labels, int m, int num_classes, int max_runs, bool force_two_pass) {
  LabelRuns L;
  std::vector<char> seen((size_t)num_classes, 0);
  bool one_run_per_class = true;
  int maxlen = 0;
  for (int i = 0; i < m;) {
    const int c = labels[i];
    if (c < 0 || c >= num_classes) {
      L.valid = false;
      return L;
    }
    int e = i + 1;
    while (e < m && labels[e] == c) ++e;
    if (seen[(size_t)c]) one_run_per_class = false;
    seen[(size_t)c] = 1;
    L.start.push_back(i);
    L.len.push_back(e - i);
    if (e - i > maxlen) maxlen = e - i;
    i = e;
  }
  if (!force_two_pass && one_run_per_class && maxlen <= kSlabMaxRows && (int)L.start.size() <= max_runs) {
    L.slab_k = 1;
    while (kSlabRowLanes * L.slab_k < maxlen) L.slab_k *= 2;
  }
  return L;
}

}  // namespace drot_plan
#endif  // DROT_PLAN_H_
