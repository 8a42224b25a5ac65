// Douglas-Rachford splitting for regularized discrete optimal transport on MI355X (gfx950).
//
// One iteration = one sweep over the m x n plan (eq. (8): X <- prox_{rho h}([X + phi 1^T +
// 1 varphi^T - rho C]_+), fused with the row sums, column sums and grand total the marginal
// projection needs) followed by the O(m+n) recursion of eq. (6).  Y is never formed (Section
// 2.1 shows how it drops out of the iteration).  The sweep is HBM bound (12 bytes per element: read X, read C,
// write X; about 8 flops), so there is no MFMA here: the design is coalesced 128-bit row-major
// accesses, DPP wave reductions for the row sums, register column partials folded through LDS,
// and a deterministic two-stage reduction instead of atomics.  Measured on MI355X, this kind of
// read-modify-write stream runs fastest when every wave issues one batch of loads, stores and
// retires (no loop: a wave that loops waits on its own store acknowledgements, loads and stores
// sharing one in-order counter) and when the loads and stores are marked non-temporal; so the
// sweep is loop-free: a wave owns 2 rows x 256 columns, a workgroup 16 such waves (32 rows).
//
// Data layout in HBM
//   X, C        m x n fp32 row-major, pitch n, caller-owned
//   phi/varphi  fp32, what the sweep reads;  a, b, theta, r, s: fp64 vectors of eq. (6)
//   rowpart     [nseg][mp] fp32: row sums of every 256-column segment (mp, np: m, n rounded up to 64)
//   colpart     [ntr][np]  fp32: column sums of every 32-row tile
//
//   colpart     ... or of every 64-row tile (sweeps for sparse plans), or of four of them (lean sweep)
//
// This translation unit is the whole product path.  The kernels live in the drot_*.h files next to
// it (sweep, screened sweeps, point-cloud cost, group lasso, dual vectors, resident solver, gap);
// drot_plan.h decides which of them runs which sweep (pure host logic, also compiled and tested
// without a GPU); this file holds the handle, the functions that enqueue what the plan says, the
// host loop and the C ABI of include/drot.h.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "drot.h"
#include "drot_plan.h"

namespace {
#include "drot_common.h"
#include "drot_sweep.h"
#include "drot_screened.h"
#include "drot_points.h"
#include "drot_group_lasso.h"
#include "drot_vectors.h"
#include "drot_resident.h"
#include "drot_gap.h"

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
namespace plan = drot_plan;
using plan::ceil_div;

// the planner's picture of the kernels' geometry must be the kernels' own
static_assert(plan::kSegCols == kSegCols && plan::kTileRows == kTileRows && plan::kAlignElems == kAlignElems, "tiles");
static_assert(plan::kTallTileRows == kScreenRows * kScreenWaves && plan::kTallTileRows == 64, "64-row tiles");
static_assert(plan::kSlabCols == kSlabCols && plan::kSlabRowLanes == kSlabRowLanes && plan::kSlabMaxRows == kSlabMaxRows, "slabs");
static_assert(plan::kResidentMaxRows == kResidentMaxRows && plan::kResidentCols == kResidentCols, "resident kernel");
static_assert(plan::kColGroup == kColGroup, "column-sum groups of the lean sweep");
static_assert(plan::kStripRows == kStripRows && plan::kPointsColGroup == kPointsColGroup, "strips of the screened point-cloud sweep");

// (e0, e1: events that take the start and the end of the kernel itself, as the hardware stamps them; null: none)
template <bool FIRST, bool PRO>
void launch_slab_k(int k, dim3 grid, hipStream_t stream, hipEvent_t e0, hipEvent_t e1, const SlabArgs& a, const FusedUpdateArgs& f) {
  const dim3 block(kSlabThreads);
  switch (k) {
    case 1: launch_timed((gl_slab_kernel<FIRST, 1, kSlabLanes, PRO>), grid, block, stream, e0, e1, a, f); break;
    case 2: launch_timed((gl_slab_kernel<FIRST, 2, kSlabLanes, PRO>), grid, block, stream, e0, e1, a, f); break;
    case 4: launch_timed((gl_slab_kernel<FIRST, 4, kSlabLanes, PRO>), grid, block, stream, e0, e1, a, f); break;
    default: launch_timed((gl_slab_kernel<FIRST, 8, kSlabLanes, PRO>), grid, block, stream, e0, e1, a, f); break;
  }
}
void launch_slab(bool first, bool pro, int k, dim3 grid, hipStream_t stream, hipEvent_t e0, hipEvent_t e1, const SlabArgs& a,
                 const FusedUpdateArgs& f) {
  if (pro) launch_slab_k<false, true>(k, grid, stream, e0, e1, a, f);
  else if (first) launch_slab_k<true, false>(k, grid, stream, e0, e1, a, f);
  else launch_slab_k<false, false>(k, grid, stream, e0, e1, a, f);
}

constexpr int kMaxProfiled = 256;   // sweeps timed per solve in profile mode
constexpr int kMaxChecks = 65536;   // residual checks recorded per solve

}  // namespace

struct drot_handle_s {
  int device = -1;
  int max_m = 0, max_n = 0;
  plan::Options opt;      // what drot_set_option sets, as the planner reads it
  int compute_gap = 1;
  int continue_next = 0;  // the next solve resumes from the state the last one left
  int profile = 0;        // record HIP events around every sweep launch
  float gap_tol = 0.f;    // > 0: a check passes only with a small enough duality gap
  plan::Carry carry;      // what the last solve left for a continued one
  bool solved = false;
  int last_m = 0, last_n = 0;
  // padded working copies: which caller arrays they were made from (a continued solve reuses them)
  const float* cpad_of = nullptr;
  bool xpad_live = false;
  // sweep timing (profile mode): event pairs recorded on the solve's stream
  hipEvent_t prof_ev[2 * kMaxProfiled] = {};
  int prof_count = 0;
  float prof_ms[kMaxProfiled] = {};   // per sweep, in launch order
  int prof_kind[kMaxProfiled] = {};
  int prof_iters[kMaxProfiled] = {};  // iterations the timed launch covers (1 unless resident)
  int prof_used = 0;
  double prof_counts_host[2 * kMaxProfiled] = {};  // [sweep][0]: row segments of C read, [1]: nonzero row segments of X after it
  // device workspace
  float *phi = nullptr, *varphi = nullptr;
  // a, b, rowpart, colpart, tilesum are double buffers (two halves), indexed by iteration parity
  double *a = nullptr, *b = nullptr, *theta = nullptr, *sum_p = nullptr, *r = nullptr, *s = nullptr, *part = nullptr,
         *resid = nullptr;
  float *rowpart = nullptr, *colpart = nullptr, *tilesum = nullptr, *gap_part = nullptr;
  size_t rowpart_half = 0, colpart_half = 0, tilesum_half = 0;
  float *mprime = nullptr, *varphi0 = nullptr;  // screened sweep: per-row-segment bounds and the epoch's varphi
  float* mprime2 = nullptr;                     //   second largest and the column of the largest
  unsigned char* jstar = nullptr;
  int* screen_ctl = nullptr;        // control words of the lean sweep's refresh schedule
  unsigned char* xlines = nullptr;  // [nseg][m] nonzero 128-byte lines of every row segment of X (lean sweep)
  int* wg_reads = nullptr;          // per-workgroup read counts of the lean sweep
  int* wave_reads = nullptr;        // profiling: per-wave read counts of a screened sweep (allocated with the events)
  double* prof_counts = nullptr;    // profiling: [kMaxProfiled][2] as prof_counts_host (device)
  float* gbuf = nullptr;  // group-lasso accumulators, grown on demand
  size_t gbuf_len = 0;
  // padded working copies of C and X (pitch rounded up to 32 elements), made when the caller's
  // arrays do not start every row on a 128-byte line; grown on demand
  float *cpad = nullptr, *xpad = nullptr;
  size_t cpad_len = 0, xpad_len = 0;
  float* ptbuf = nullptr;  // on-the-fly cost: packed point clouds and their squared norms
  size_t ptbuf_len = 0;
  int* runbuf = nullptr;  // group-resident path: run_start[], run_len[] of the label runs
  size_t runbuf_len = 0;
  int* chunkbuf = nullptr;  // two-pass path: perm[m], chunk_start[nchunks + 1], class_first[num_classes + 1]
  size_t chunkbuf_len = 0;
  float* gpart = nullptr;   // two-pass path: [nchunks][n] squared sums of the chunks
  size_t gpart_len = 0;
  int max_runs = 0;       // rows of colpart available
  int* done = nullptr;
  DeviceStatus* status = nullptr;
  // pinned host mirror of the status block, two slots for the pipelined residual checks
  DeviceStatus* host_status = nullptr;
  hipEvent_t ev[2] = {nullptr, nullptr};
  drot_info info{};
  std::vector<drot_check> checks;  // the residual checks of the last solve
};

namespace {

#define DROT_HIP(expr)                                                                   \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess) {                                                              \
      fprintf(stderr, "drot: %s failed: %s\n", #expr, hipGetErrorString(e_));            \
      return DROT_ERR_HIP;                                                               \
    }                                                                                    \
  } while (0)

template <typename T>
int dev_alloc(T** ptr, size_t count) {
  hipError_t e = hipMalloc(reinterpret_cast<void**>(ptr), count * sizeof(T));
  if (e != hipSuccess) {
    *ptr = nullptr;
    return DROT_ERR_ALLOC;
  }
  return DROT_OK;
}

// Replaces *buf by an allocation of at least `need` elements if it is smaller (contents are lost).
template <typename T>
int grow_buffer(T** buf, size_t* len, size_t need, hipStream_t stream) {
  if (*len >= need) return DROT_OK;
  if (hipStreamSynchronize(stream) != hipSuccess) return DROT_ERR_HIP;
  (void)hipFree(*buf);
  *buf = nullptr;
  *len = 0;
  if (dev_alloc(buf, need) != DROT_OK) return DROT_ERR_ALLOC;
  *len = need;
  return DROT_OK;
}

void free_all(drot_handle h) {
  float* fbufs[] = {h->phi, h->varphi, h->rowpart, h->colpart, h->tilesum, h->gap_part, h->gbuf, h->mprime, h->mprime2,
                    h->varphi0, h->cpad, h->xpad, h->ptbuf, h->gpart};
  double* dbufs[] = {h->a, h->b, h->theta, h->sum_p, h->r, h->s, h->part, h->resid, h->prof_counts};
  int* ibufs[] = {h->done, h->runbuf, h->chunkbuf, h->wave_reads, h->screen_ctl, h->wg_reads};
  for (float* b : fbufs) (void)hipFree(b);
  for (double* b : dbufs) (void)hipFree(b);
  for (int* b : ibufs) (void)hipFree(b);
  (void)hipFree(h->status);
  (void)hipFree(h->xlines);
  (void)hipFree(h->jstar);
  if (h->host_status) (void)hipHostFree(h->host_status);
  for (auto& e : h->ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& e : h->prof_ev)
    if (e) (void)hipEventDestroy(e);
}

// Creates the events and counters of profile mode: everything or nothing.
int enable_profile(drot_handle h) {
  hipEvent_t made[2 * kMaxProfiled] = {};
  int nmade = 0;
  bool ok = true;
  auto make = [&](hipEvent_t& e) {
    if (!ok || e) return;
    if (hipEventCreate(&e) != hipSuccess) {
      e = nullptr;
      ok = false;
      return;
    }
    made[nmade++] = e;
  };
  for (auto& e : h->prof_ev) make(e);
  int* wave_reads = nullptr;
  double* prof_counts = nullptr;
  int rc = ok ? DROT_OK : DROT_ERR_HIP;
  if (rc == DROT_OK && !h->prof_counts) {
    // read counts of the screened sweeps: one int per wave of the largest grid; two totals per timed sweep
    const size_t waves = (size_t)ceil_div(h->max_n, kSegCols) * (size_t)ceil_div(h->max_m, 64) * kScreenWaves;
    if (dev_alloc(&wave_reads, waves) != DROT_OK || dev_alloc(&prof_counts, (size_t)2 * kMaxProfiled) != DROT_OK)
      rc = DROT_ERR_ALLOC;
  }
  if (rc != DROT_OK) {
    (void)hipFree(wave_reads);
    (void)hipFree(prof_counts);
    auto forget = [&](hipEvent_t& e) {
      for (int k = 0; k < nmade; ++k)
        if (e == made[k]) e = nullptr;
    };
    for (auto& e : h->prof_ev) forget(e);
    for (int k = 0; k < nmade; ++k) (void)hipEventDestroy(made[k]);
    (void)hipGetLastError();
    return rc;
  }
  if (!h->prof_counts) {
    h->wave_reads = wave_reads;
    h->prof_counts = prof_counts;
  }
  return DROT_OK;
}

// dst[i][j] = src[i][j] for an m x n matrix held with two different row pitches (in elements).
void copy_rows(float* dst, size_t dpitch, const float* src, size_t spitch, int m, int n, hipStream_t stream) {
  const int rows16 = ceil_div(m, 16);
  hipLaunchKernelGGL(copy_rows_kernel, dim3(ceil_div(n, 1024), rows16 < 65535 ? rows16 : 65535), dim3(256), 0, stream, dst,
                     dpitch, src, spitch, m, n);
}

// Where the cost comes from: a stored matrix, or two point clouds (C_ij = scale * ||xs_i - xt_j||^2).
struct CostSource {
  const float* C = nullptr;
  const float* xs = nullptr;  // [m][d]
  const float* xt = nullptr;  // [n][d]
  int d = 0;
  float scale = 0.f;
};

// Everything one call of the solver works with: the problem as handed over, the plan, and the kernel
// argument blocks that stay the same from sweep to sweep.
struct Solve {
  drot_handle h = nullptr;
  hipStream_t stream = nullptr;
  plan::Problem P;
  plan::Options O;
  plan::Static S;
  plan::State T;
  int m = 0, n = 0;
  drot_reg_kind reg_kind = DROT_REG_NONE;
  float rho = 0.f, lambda = 0.f, mu = 0.f, tol = 0.f;
  const float *p = nullptr, *q = nullptr;
  const int* row_class = nullptr;
  size_t ngroups = 0;
  float* X_out = nullptr;
  const float* Cw = nullptr;  // the arrays the kernels work on: the caller's, or the padded copies
  float* Xw = nullptr;
  int ldc = 0, ldx = 0;
  VecState V{};
  SweepArgs SA{};
  PointArgs PT{};
  ReduceArgs RA{};
  UpdateArgs UA{};
  float thr = 0.f;  // rho * mu
  ChunkArgs CK{};   // two-pass group lasso: the classes' rows in chunks
  int num_classes = 0;

  double* a_buf(long long g) const { return h->a + (size_t)(g & 1) * (size_t)h->max_m; }
  double* b_buf(long long g) const { return h->b + (size_t)(g & 1) * (size_t)h->max_n; }
  // (row-segment sums: two halves only where the vector update rides at the head of the next sweep and reads the old
  // sums while the new ones are written; everywhere else a sweep reads nothing but its own old sums, before it writes
  // them, so one buffer serves, and a sweep may leave alone what it knows to be unchanged)
  float* rowp(long long g) const { return h->rowpart + (S.fused ? (size_t)(g & 1) * h->rowpart_half : 0); }
  float* colp(long long g) const { return h->colpart + (size_t)(g & 1) * h->colpart_half; }
  float* tsum(long long g) const { return h->tilesum + (size_t)(g & 1) * h->tilesum_half; }
};

// The vector update of sweep sw - 1 as it rides along at the head of sweep sw (small problems).
FusedUpdateArgs fused_args(const Solve& Z, long long sw, int nseg, int ntr) {
  drot_handle h = Z.h;
  return FusedUpdateArgs{Z.rowp(sw - 1), Z.colp(sw - 1), Z.tsum(sw - 1), Z.p, Z.q, Z.a_buf(sw - 2), Z.b_buf(sw - 2),
                         Z.a_buf(sw - 1), Z.b_buf(sw - 1), h->theta + ((sw - 2) & 1), h->theta + ((sw - 1) & 1),
                         h->sum_p, h->phi, h->varphi, nseg, ntr};
}

// One sweep launch (S1-S4), as the plan describes it.
void enqueue_sweep(Solve& Z, const plan::Step& Q, bool timed, hipEvent_t e0, hipEvent_t e1) {
  drot_handle h = Z.h;
  hipStream_t stream = Z.stream;
  const plan::Static& S = Z.S;
  const int m = Z.m, n = Z.n;
  const long long sw = Q.sw;
  const bool nt = S.nt;
  const dim3 grid(S.nseg, S.ntr), block(kBlock), sweep_block(64 * kSweepWaves);
  SweepArgs A = Z.SA;
  A.rowpart = Z.rowp(sw);
  A.colpart = Z.colp(sw);
  A.tilesum = Q.tilesum ? Z.tsum(sw) : nullptr;
  A.rowpart_prev = Q.prev_sums ? Z.rowp(sw - 1) : nullptr;
  const FusedUpdateArgs none{};
  switch (Q.sweep) {
    case plan::kResident: {
      const long long last = sw + Q.iters - 1;  // the state leaves in that generation's buffers
      const ResidentArgs RS{Z.Xw, Z.Cw, Z.p, Z.q, Z.V, Z.a_buf(sw - 1), Z.b_buf(sw - 1), Z.a_buf(last), Z.b_buf(last),
                            (int)((sw - 1) & 1), (int)(last & 1), m, n, Z.ldx, Z.ldc, Z.rho, A.scale, Q.iters,
                            Q.first ? 1 : 0};
      if (n <= 64) launch_resident<1>(RS, stream, e0, e1);
      else if (n <= 128) launch_resident<2>(RS, stream, e0, e1);
      else launch_resident<4>(RS, stream, e0, e1);
      break;
    }
    case plan::kPoints:
      if (Q.first) launch_timed((sweep_points_kernel<true, false>), grid, sweep_block, stream, e0, e1, A, Z.PT, h->mprime, h->mprime2, h->jstar, h->varphi0);
      else if (Q.refresh && nt) launch_timed((sweep_points_kernel<false, true, true>), grid, sweep_block, stream, e0, e1, A, Z.PT, h->mprime, h->mprime2, h->jstar, h->varphi0);
      else if (Q.refresh) launch_timed((sweep_points_kernel<false, false, true>), grid, sweep_block, stream, e0, e1, A, Z.PT, h->mprime, h->mprime2, h->jstar, h->varphi0);
      else if (nt) launch_timed((sweep_points_kernel<false, true>), grid, sweep_block, stream, e0, e1, A, Z.PT, h->mprime, h->mprime2, h->jstar, h->varphi0);
      else launch_timed((sweep_points_kernel<false, false>), grid, sweep_block, stream, e0, e1, A, Z.PT, h->mprime, h->mprime2, h->jstar, h->varphi0);
      break;
    case plan::kPointsLean: {
      const ScreenArgs SC{h->mprime, h->mprime, h->varphi0, nullptr, h->varphi0, h->screen_ctl, h->wg_reads, nullptr, h->xlines,
                          h->mprime2, h->mprime2, h->jstar, h->jstar};
      const dim3 pgrid(S.nseg, ceil_div(m, kStripRows));
      if (nt) launch_timed((lean_points_kernel<true>), pgrid, dim3(256), stream, e0, e1, A, Z.PT, SC);
      else launch_timed((lean_points_kernel<false>), pgrid, dim3(256), stream, e0, e1, A, Z.PT, SC);
      break;
    }
    case plan::kSlab: {
      const SlabArgs SL{A, h->runbuf, h->runbuf + Z.P.nruns, Z.thr};
      const dim3 slab_grid(S.nstrips, Z.P.nruns > 0 ? Z.P.nruns : 1);
      launch_slab(Q.first, Q.pro, Z.P.slab_k, slab_grid, stream, e0, e1, SL, fused_args(Z, sw, S.nstrips, Z.P.nruns));
      break;
    }
    case plan::kTwoPass: {
      const GroupArgs G{A, Z.row_class, h->gbuf, Z.thr};
      const dim3 cgrid(S.nseg, ceil_div(Z.CK.nchunks, kWavesPerBlock));
      const dim3 fgrid(ceil_div(n, kBlock), Z.num_classes < 65535 ? Z.num_classes : 65535);
      // (three launches: the start of the first and the end of the last are what is timed)
      if (Q.first) launch_timed(gl_norm_kernel<true>, cgrid, block, stream, e0, nullptr, G, Z.CK);
      else launch_timed(gl_norm_kernel<false>, cgrid, block, stream, e0, nullptr, G, Z.CK);
      hipLaunchKernelGGL(gl_norm_finish_kernel, fgrid, block, 0, stream, Z.CK, h->gbuf, n, Z.num_classes, (const int*)h->done);
      if (Q.first) launch_timed(gl_apply_kernel<true>, grid, block, stream, nullptr, e1, G);
      else launch_timed(gl_apply_kernel<false>, grid, block, stream, nullptr, e1, G);
      break;
    }
    case plan::kPro32: {
      // update sw-1 (from the sums of X_{sw-1} and the state of generation sw-2) rides along
      const FusedUpdateArgs F = fused_args(Z, sw, S.nseg, S.ntr);
      if (nt) launch_timed((sweep_kernel<false, true, true>), grid, sweep_block, stream, e0, e1, A, F);
      else launch_timed((sweep_kernel<false, false, true>), grid, sweep_block, stream, e0, e1, A, F);
      break;
    }
    case plan::kPlain32:
      if (Q.first) {
        if (Q.mode == 1) launch_timed((sweep_kernel<true, false, false, 1>), grid, sweep_block, stream, e0, e1, A, none);
        else launch_timed((sweep_kernel<true, false, false, 0>), grid, sweep_block, stream, e0, e1, A, none);
      } else if (nt) {
        if (Q.mode == 1) launch_timed((sweep_kernel<false, true, false, 1>), grid, sweep_block, stream, e0, e1, A, none);
        else if (Q.mode == 2) launch_timed((sweep_kernel<false, true, false, 2>), grid, sweep_block, stream, e0, e1, A, none);
        else launch_timed((sweep_kernel<false, true, false, 0>), grid, sweep_block, stream, e0, e1, A, none);
      } else {
        if (Q.mode == 1) launch_timed((sweep_kernel<false, false, false, 1>), grid, sweep_block, stream, e0, e1, A, none);
        else if (Q.mode == 2) launch_timed((sweep_kernel<false, false, false, 2>), grid, sweep_block, stream, e0, e1, A, none);
        else launch_timed((sweep_kernel<false, false, false, 0>), grid, sweep_block, stream, e0, e1, A, none);
      }
      break;
    case plan::kTall64: {
      const dim3 tgrid(S.nseg, S.ntr_tall), tblock(64 * kScreenWaves);
      if (nt) launch_timed((sweep_kernel<false, true, false, 0, kScreenRows, kScreenWaves>), tgrid, tblock, stream, e0, e1, A, none);
      else launch_timed((sweep_kernel<false, false, false, 0, kScreenRows, kScreenWaves>), tgrid, tblock, stream, e0, e1, A, none);
      break;
    }
    case plan::kScreened8: {
      const ScreenArgs SC{h->mprime, h->mprime, h->varphi0, timed ? h->wave_reads : nullptr, h->varphi0,
                          h->screen_ctl, h->wg_reads, nullptr, h->xlines, h->mprime2, h->mprime2, h->jstar, h->jstar};
      const dim3 sgrid(S.nseg, S.ntr_tall), sblock(64 * kScreenWaves);
      if (Q.refresh) {
        if (nt) launch_timed((screened_sweep_kernel<true, true>), sgrid, sblock, stream, e0, e1, A, SC);
        else launch_timed((screened_sweep_kernel<false, true>), sgrid, sblock, stream, e0, e1, A, SC);
      } else {
        if (nt) launch_timed((screened_sweep_kernel<true, false>), sgrid, sblock, stream, e0, e1, A, SC);
        else launch_timed((screened_sweep_kernel<false, false>), sgrid, sblock, stream, e0, e1, A, SC);
      }
      break;
    }
    case plan::kLean: {
      const ScreenArgs SC{h->mprime, h->mprime, h->varphi0, nullptr, h->varphi0, h->screen_ctl, h->wg_reads,
                          Q.lines_in ? h->xlines : nullptr, h->xlines, h->mprime2, h->mprime2, h->jstar, h->jstar};
      const dim3 lgrid(S.nseg, ceil_div(S.ntr_tall, kLeanWaves)), lblock(64 * kLeanWaves);
      if (nt) launch_timed((screened_lean_kernel<true>), lgrid, lblock, stream, e0, e1, A, SC, S.ntr_tall);
      else launch_timed((screened_lean_kernel<false>), lgrid, lblock, stream, e0, e1, A, SC, S.ntr_tall);
      break;
    }
  }
}

// The vector update (S5) that completes the state in memory after sweep Q.sw.
void enqueue_update(Solve& Z, const plan::Step& Q) {
  if (Q.update == plan::kNoUpdate) return;
  drot_handle h = Z.h;
  hipStream_t stream = Z.stream;
  const plan::Static& S = Z.S;
  const long long sw = Q.sw;
  ReduceArgs RA = Z.RA;
  RA.rowpart = Z.rowp(sw);
  RA.colpart = Z.colp(sw);
  RA.ntr = Q.ra_ntr;
  RA.cgroup = Q.ra_cgroup;
  UpdateArgs UA = Z.UA;
  UA.a_in = Z.a_buf(sw - 1);
  UA.b_in = Z.b_buf(sw - 1);
  UA.a_out = Z.a_buf(sw);
  UA.b_out = Z.b_buf(sw);
  UA.par = (int)((sw - 1) & 1);
  UA.tilesum = S.small ? Z.tsum(sw) : nullptr;
  UA.ntiles = S.small_slab ? S.nstrips * Z.P.nruns : S.ntiles;
  // (four entries per lane where that still leaves a workgroup for every other compute unit)
  const bool wide = ceil_div(Z.m, 256) + ceil_div(Z.n, 256) >= 64;
  const int per_wg = wide ? 256 : 64;
  const dim3 merged_grid(ceil_div(Z.m, per_wg) + ceil_div(Z.n, per_wg)), merged_block(64 * kMergedWaves);
  auto merged = [&](const TileTotals& TT, const ScreenCtlArgs& KA) {
    if (wide) hipLaunchKernelGGL(reduce_update_kernel<4>, merged_grid, merged_block, 0, stream, RA, UA, TT, KA);
    else hipLaunchKernelGGL(reduce_update_kernel<1>, merged_grid, merged_block, 0, stream, RA, UA, TT, KA);
  };
  if (Q.update == plan::kMergedSlab) {
    const TileTotals TT{Z.tsum(sw), Q.tt_rows, S.nstrips, Q.tt_group};
    const ScreenCtlArgs KA{nullptr, nullptr, 0, 0, 0, 0};
    merged(TT, KA);
  } else if (Q.update == plan::kMergedTiles) {
    const TileTotals TT{Z.tsum(sw), Q.tt_rows, S.nseg, Q.tt_group};
    // (the price of a renewal: all row segments of C, read by a sweep that streams them better than
    // the scattered reads it saves)
    const double price = 0.75 * (double)Z.m * (double)S.nseg;
    const ScreenCtlArgs KA{h->screen_ctl, h->wg_reads, S.nseg * ceil_div(S.ntr_tall, kLeanWaves), Q.ctl_mode,
                           price < 1.0e9 ? (int)price : 1000000000, Z.O.screening >= 2 ? Z.O.screening : 1024};
    merged(TT, KA);
  } else {
    hipLaunchKernelGGL(reduce_kernel, dim3(S.nbm + S.nbn), dim3(kReduceThreads), 0, stream, RA);
    hipLaunchKernelGGL(update_kernel, dim3(ceil_div(Z.m + Z.n, kReduceThreads)), dim3(kReduceThreads), 0, stream, UA);
  }
}

// S7: objective, duality gap and dual residual of the state in memory into the status block.  guard:
// the stop flag, for the passes that belong to a check (after a stop they would only repeat it).
// flags_current: the host's record of the flags (line flags, row-segment sums) describes the X in memory, i.e. no
// sweep enqueued so far can have been skipped by a stop raised on the device.
void enqueue_gap(Solve& Z, const int* guard, bool flags_current) {
  drot_handle h = Z.h;
  hipStream_t stream = Z.stream;
  const plan::Static& S = Z.S;
  float* gx = h->gbuf;
  float* gw = h->gbuf ? h->gbuf + Z.ngroups : nullptr;
  if (Z.reg_kind == DROT_REG_GROUP_LASSO)
    hipLaunchKernelGGL(fill_kernel, dim3(ceil_div((int)((2 * Z.ngroups + 255) / 256), 4)), dim3(256), 0, stream, h->gbuf,
                       2 * Z.ngroups, 0.f, guard);
  const GapArgs GA{Z.Xw, Z.Cw, h->phi, h->varphi, Z.row_class, h->gap_part, gx, gw, Z.m, Z.n, S.nseg, Z.ldx, Z.ldc, Z.rho,
                   Z.PT, guard};
  const plan::GapPass pass = flags_current ? plan::gap_pass(S, Z.P, Z.T) : plan::kGapDense;
  if (pass != plan::kGapDense) {
    const GapLeanArgs GL{GA, h->mprime, h->mprime2, h->jstar, h->varphi0, pass == plan::kGapLeanLines ? h->xlines : nullptr,
                         Z.rowp(Z.T.k_base + Z.T.k), Z.SA.n_mem, Z.SA.mp, S.ntr_tall, S.ntr};
    hipLaunchKernelGGL(gap_lean_kernel, dim3(S.nseg, ceil_div(S.ntr_tall, kLeanWaves)), dim3(64 * kLeanWaves), 0, stream, GL);
  } else {
    hipLaunchKernelGGL(gap_kernel, dim3(S.nseg, S.ntr), dim3(kBlock), 0, stream, GA);
  }
  hipLaunchKernelGGL(gap_final_kernel, dim3(1), dim3(1024), 0, stream, Z.V, (const float*)h->gap_part, S.ntiles,
                     (const float*)gx, (const float*)gw, Z.ngroups, Z.p, Z.q, Z.m, Z.n, (double)Z.rho, (int)Z.reg_kind,
                     (double)Z.lambda, (double)Z.mu, guard);
}

// S6: the status of the state in memory after k iterations of this call; with a tolerance it is the
// stopping test.  gap_fresh: objective, gap and dual residual in the status block were just evaluated.
void enqueue_status(Solve& Z, int k, bool test, bool gap_fresh) {
  if (Z.T.norms_pending)
    hipLaunchKernelGGL(residual_norms_kernel, dim3(1), dim3(kReduceThreads), 0, Z.stream, Z.V, Z.S.nbm, Z.S.nbn);
  Z.T.norms_pending = false;
  hipLaunchKernelGGL(status_kernel, dim3(1), dim3(1), 0, Z.stream, Z.V, k, test ? (double)Z.tol : 0.0,
                     test ? (double)Z.h->gap_tol : 0.0, gap_fresh ? 1 : 0);
}

void record_check(drot_handle h, const DeviceStatus& st) {
  if (st.iters <= 0 || (int)h->checks.size() >= kMaxChecks) return;
  if (!h->checks.empty() && h->checks.back().iters == st.iters) return;  // (after a stop the block no longer changes)
  drot_check c;
  c.iters = st.iters;
  c.gap_evaluated = st.gap_iters == st.iters ? 1 : 0;
  c.r_row = (float)std::sqrt(st.r2);
  c.r_col = (float)std::sqrt(st.s2);
  c.objective = c.gap_evaluated ? st.cost + st.h : 0.0;
  c.gap = c.gap_evaluated ? st.gap : 0.0;
  c.dual_res = c.gap_evaluated ? st.dual_res : 0.0;
  h->checks.push_back(c);
}

// Arguments as handed over by the entry points.
struct SolveCall {
  CostSource cost;
  const float *p = nullptr, *q = nullptr;
  int m = 0, n = 0;
  float stepsize = 0.f;
  drot_reg_kind reg_kind = DROT_REG_NONE;
  const drot_reg_params* reg_params = nullptr;
  int max_iters = 0;
  float tol = 0.f;
  float* X_out = nullptr;
  const float *phi0 = nullptr, *varphi0 = nullptr;
  bool warm = false;
  void* stream = nullptr;
  bool fixed_schedule = false;  // the host never reads the status block during the solve (drot_solve_static)
};

// Checks the arguments, analyses the labels, grows the on-demand buffers, builds the plan and the
// argument blocks, and enqueues what precedes the first sweep.
int prepare(drot_handle h, const SolveCall& A, Solve& Z) {
  const float* C = A.cost.C;
  const bool from_points = C == nullptr;
  const int m = A.m, n = A.n;
  if (!h || !A.p || !A.q || !A.X_out) return DROT_ERR_INVALID_ARG;
  if (from_points) {
    if (!A.cost.xs || !A.cost.xt || A.cost.d < 1 || !(A.cost.scale > 0.f)) return DROT_ERR_INVALID_ARG;
    if (A.reg_kind == DROT_REG_GROUP_LASSO) return DROT_ERR_INVALID_ARG;  // stored-cost paths only
  }
  if (A.warm && (!A.phi0 || !A.varphi0)) return DROT_ERR_INVALID_ARG;
  if (m < 1 || n < 1 || m > h->max_m || n > h->max_n || A.max_iters < 0) return DROT_ERR_INVALID_ARG;
  if (A.reg_kind != DROT_REG_NONE && A.reg_kind != DROT_REG_QUADRATIC && A.reg_kind != DROT_REG_GROUP_LASSO)
    return DROT_ERR_INVALID_ARG;
  if (!(A.tol == A.tol) || !(A.stepsize == A.stepsize)) return DROT_ERR_INVALID_ARG;  // NaN
  float lambda = 0.f, mu = 0.f;
  int num_classes = 0;
  const int* row_class = nullptr;
  if (A.reg_kind != DROT_REG_NONE) {
    if (!A.reg_params) return DROT_ERR_INVALID_ARG;
    lambda = A.reg_params->lambda;
    if (!(lambda >= 0.f)) return DROT_ERR_INVALID_ARG;
    if (A.reg_kind == DROT_REG_GROUP_LASSO) {
      mu = A.reg_params->mu;
      num_classes = A.reg_params->num_classes;
      row_class = A.reg_params->row_class;
      if (!(mu >= 0.f) || num_classes < 1 || !row_class) return DROT_ERR_INVALID_ARG;
    }
  }
  // weighted l1 term <W, X>: on X >= 0 it shifts the cost, so the solve runs on a working copy C + W
  const float* weights = A.reg_params ? A.reg_params->weights : nullptr;
  if (weights && (from_points || reinterpret_cast<uintptr_t>(weights) % 4)) return DROT_ERR_INVALID_ARG;
  int cur_dev = -1;
  DROT_HIP(hipGetDevice(&cur_dev));
  if (cur_dev != h->device) return DROT_ERR_INVALID_ARG;  // the workspace lives on the creating device
  const bool resume = h->continue_next != 0 && !A.warm;
  if (resume && (!h->solved || m != h->last_m || n != h->last_n)) return DROT_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(A.X_out) % 4 || reinterpret_cast<uintptr_t>(C) % 4) return DROT_ERR_INVALID_ARG;
  if (from_points && (reinterpret_cast<uintptr_t>(A.cost.xs) % 4 || reinterpret_cast<uintptr_t>(A.cost.xt) % 4))
    return DROT_ERR_INVALID_ARG;
  hipStream_t stream = reinterpret_cast<hipStream_t>(A.stream);

  Z.h = h;
  Z.stream = stream;
  Z.m = m;
  Z.n = n;
  Z.reg_kind = A.reg_kind;
  Z.rho = A.stepsize > 0.f ? A.stepsize : 2.0f / (float)(m + n);
  Z.lambda = lambda;
  Z.mu = mu;
  Z.tol = A.tol;
  Z.p = A.p;
  Z.q = A.q;
  Z.row_class = row_class;
  Z.X_out = A.X_out;
  Z.thr = Z.rho * mu;
  // 1/(1 + rho*lambda) evaluated in fp64 from the fp32 inputs, rounded once
  const float qscale = (float)(1.0 / (1.0 + (double)Z.rho * (double)lambda));

  plan::Problem& P = Z.P;
  P.m = m;
  P.n = n;
  P.reg_kind = (int)A.reg_kind;
  P.from_points = from_points;
  P.warm = A.warm;
  P.resume = resume;
  P.has_weights = weights != nullptr;
  P.c_on_lines = reinterpret_cast<uintptr_t>(C) % 128 == 0;
  P.x_on_lines = reinterpret_cast<uintptr_t>(A.X_out) % 128 == 0;
  P.tilesum_half = h->tilesum_half;
  P.feedback = !A.fixed_schedule;
  P.checking = A.tol > 0.f;
  P.max_iters = A.max_iters;
  Z.O = h->opt;
  if (h->gap_tol > 0.f && Z.O.gap_every < 1) Z.O.gap_every = 1;

  if (A.reg_kind == DROT_REG_GROUP_LASSO) {
    Z.ngroups = (size_t)num_classes * (size_t)n;
    const int rc = grow_buffer(&h->gbuf, &h->gbuf_len, 2 * Z.ngroups, stream);
    if (rc != DROT_OK) return rc;
    // If every class is one run of consecutive rows short enough to sit in a workgroup's registers,
    // take the group-resident kernel; otherwise the general two-pass path.
    std::vector<int> labels((size_t)m);
    DROT_HIP(hipMemcpyAsync(labels.data(), row_class, sizeof(int) * (size_t)m, hipMemcpyDeviceToHost, stream));
    DROT_HIP(hipStreamSynchronize(stream));
    const plan::LabelRuns L = plan::analyze_labels(labels.data(), m, num_classes, h->max_runs, Z.O.force_two_pass != 0);
    if (!L.valid) return DROT_ERR_INVALID_ARG;
    P.nruns = (int)L.start.size();
    P.slab_k = L.slab_k;
    if (L.slab_k) {
      const int rc2 = grow_buffer(&h->runbuf, &h->runbuf_len, 2 * L.start.size(), stream);
      if (rc2 != DROT_OK) return rc2;
      std::vector<int> table(L.start);  // run_start[0..nruns), run_len[0..nruns)
      table.insert(table.end(), L.len.begin(), L.len.end());
      DROT_HIP(hipMemcpy(h->runbuf, table.data(), sizeof(int) * table.size(), hipMemcpyHostToDevice));
    } else {
      // two passes: the rows of every class in chunks, so that the group norms add up in a fixed order
      const plan::ClassChunks K = plan::chunk_classes(labels.data(), m, num_classes);
      std::vector<int> table(K.perm);
      table.insert(table.end(), K.chunk_start.begin(), K.chunk_start.end());
      table.insert(table.end(), K.class_first.begin(), K.class_first.end());
      int rc2 = grow_buffer(&h->chunkbuf, &h->chunkbuf_len, table.size(), stream);
      if (rc2 == DROT_OK) rc2 = grow_buffer(&h->gpart, &h->gpart_len, (size_t)K.nchunks() * (size_t)n, stream);
      if (rc2 != DROT_OK) return rc2;
      DROT_HIP(hipMemcpy(h->chunkbuf, table.data(), sizeof(int) * table.size(), hipMemcpyHostToDevice));
      Z.CK = ChunkArgs{h->chunkbuf, h->chunkbuf + m, h->chunkbuf + m + K.nchunks() + 1, h->gpart, K.nchunks()};
    }
    Z.num_classes = num_classes;
  }
  Z.S = plan::make_static(P, Z.O);
  Z.T = plan::start_state(Z.S, P, h->carry);
  const plan::Static& S = Z.S;

  Z.V = VecState{h->phi, h->varphi, h->a, h->b, h->theta, h->sum_p, h->r, h->s, h->part, h->resid, h->done, h->status};
  hipLaunchKernelGGL(mask_tail_kernel, dim3(1), dim3(256), 0, stream, h->varphi, h->varphi0, n);
  if (resume) hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(1), 0, stream, Z.V);
  else if (!A.warm) hipLaunchKernelGGL(init_kernel, dim3(1), dim3(1024), 0, stream, Z.V, A.p, A.q, m, n);

  // Rows that do not start on 128-byte lines are slow to stream: work on padded copies then.  A
  // continued solve finds them as the last one left them.
  Z.Cw = C;
  Z.Xw = A.X_out;
  Z.ldc = Z.ldx = n;
  const size_t padded = (size_t)m * (size_t)S.ld_pad;
  auto grow_padded = [&](float** buf, size_t* len) -> int {
    if (*len >= padded) return DROT_OK;
    const int rc = grow_buffer(buf, len, padded, stream);
    if (rc != DROT_OK) return rc;
    // the pad columns must hold finite values: they are read (and masked out) by the last lanes of a row
    hipLaunchKernelGGL(fill_kernel, dim3(1024), dim3(256), 0, stream, *buf, padded, 0.f, (const int*)nullptr);
    return DROT_OK;
  };
  if (S.pad_c) {
    const size_t had = h->cpad_len;
    const int rc = grow_padded(&h->cpad, &h->cpad_len);
    if (rc != DROT_OK) return rc;
    Z.Cw = h->cpad;
    Z.ldc = S.ld_pad;
    const bool reuse = resume && had >= padded && h->cpad_of == C;
    if (weights)
      hipLaunchKernelGGL(add_weights_kernel, dim3(ceil_div(n, 256), m < 65535 ? m : 65535), dim3(256), 0, stream, h->cpad, C,
                         weights, m, n, S.ld_pad);
    else if (!reuse)
      copy_rows(h->cpad, (size_t)S.ld_pad, C, (size_t)n, m, n, stream);
    h->cpad_of = weights ? nullptr : C;
  }
  if (S.pad_x) {
    const size_t had = h->xpad_len;
    const int rc = grow_padded(&h->xpad, &h->xpad_len);
    if (rc != DROT_OK) return rc;
    Z.Xw = h->xpad;
    Z.ldx = S.ld_pad;
    const bool reuse = resume && had >= padded && h->xpad_live;
    if ((resume && !reuse) || A.warm)  // the plan to start from is in X_out
      copy_rows(h->xpad, (size_t)S.ld_pad, A.X_out, (size_t)n, m, n, stream);
  }
  h->xpad_live = false;  // (until this solve has returned)
  Z.SA = SweepArgs{Z.Xw, Z.Cw, h->phi, h->varphi, nullptr, nullptr, nullptr, h->done, m, n, Z.ldx, Z.ldc, Z.rho,
                   A.reg_kind == DROT_REG_NONE ? 1.0f : qscale,
                   (S.pad_x && (S.pad_c || from_points)) ? S.ld_pad : n, nullptr, ceil_div(m, 64) * 64, ceil_div(n, 64) * 64};
  // (the sweeps' edge handling counts on rows that are whole 128-byte lines: the planner's pad_c, pad_x see to it)
  if (!S.resident && Z.SA.n_mem % kAlignElems != 0) return DROT_ERR_INVALID_ARG;
  // on-the-fly cost: pack the point clouds for the matrix cores and take their squared norms
  if (from_points) {
    const int dq = ceil_div(A.cost.d, 16) * 4;
    const int ncb = ceil_div(n, 16);
    const size_t need = ((size_t)m + (size_t)ncb * 16) * 4 * (size_t)dq + (size_t)m + (size_t)n;
    const int rc = grow_buffer(&h->ptbuf, &h->ptbuf_len, need, stream);
    if (rc != DROT_OK) return rc;
    float* xs_pack = h->ptbuf;
    float* xt_pack = xs_pack + (size_t)m * 4 * dq;
    float* xs_sq = xt_pack + (size_t)ncb * 16 * 4 * dq;
    float* xt_sq = xs_sq + m;
    hipLaunchKernelGGL(pack_points_kernel, dim3(ceil_div(m, 256)), dim3(256), 0, stream, A.cost.xs, m, A.cost.d, dq, xs_pack, xs_sq, 0);
    hipLaunchKernelGGL(pack_points_kernel, dim3(ceil_div(ncb * 16, 256)), dim3(256), 0, stream, A.cost.xt, n, A.cost.d, dq, xt_pack, xt_sq, 1);
    Z.PT = PointArgs{xs_pack, xt_pack, xs_sq, xt_sq, dq, A.cost.scale, ncb};
  }
  // the partial sums the reduction reads: per 256-column segment and 32-row tile, or, on the
  // group-resident path, per 32-column strip and label run
  Z.RA = ReduceArgs{Z.V, h->rowpart, h->colpart, A.p, A.q, m, n, P.slab_k ? S.nstrips : S.nseg,
                    P.slab_k ? P.nruns : S.ntr, S.nbm, S.nbn, Z.SA.mp, Z.SA.np, 1};
  Z.UA = UpdateArgs{Z.V, nullptr, 0, nullptr, nullptr, nullptr, nullptr, m, n, S.nbm, S.nbn, 0};

  if (A.warm) {
    // sums of X_0 (a sweep that only adds up), residuals, then the eq. (6) state of the starting point
    hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(1), 0, stream, Z.V);
    SweepArgs W = Z.SA;
    W.rowpart = Z.rowp(0);
    W.colpart = Z.colp(0);
    hipLaunchKernelGGL((sweep_kernel<false, false, false, 3>), dim3(S.nseg, S.ntr), dim3(64 * kSweepWaves), 0, stream, W,
                       FusedUpdateArgs{});
    ReduceArgs RW = Z.RA;
    RW.rowpart = Z.rowp(0);
    RW.colpart = Z.colp(0);
    RW.nseg = S.nseg;
    RW.ntr = S.ntr;
    hipLaunchKernelGGL(reduce_kernel, dim3(S.nbm + S.nbn), dim3(kReduceThreads), 0, stream, RW);
    hipLaunchKernelGGL(warm_init_kernel, dim3(1), dim3(1024), 0, stream, Z.V, A.p, A.phi0, A.varphi0, m, n);
  }
  if (A.max_iters == 0 && !resume && !A.warm) {
    hipLaunchKernelGGL(fill_kernel, dim3(1024), dim3(256), 0, stream, A.X_out, (size_t)m * n, 0.f, (const int*)nullptr);
    if (S.pad_x)  // (the gap pass reads the working copy, which may hold an earlier solve's plan)
      hipLaunchKernelGGL(fill_kernel, dim3(1024), dim3(256), 0, stream, h->xpad, padded, 0.f, (const int*)nullptr);
  }
  DROT_HIP(hipGetLastError());
  return DROT_OK;
}

// The host loop: stretches of sweeps and vector updates, a status at the end of each where one is due,
// read one stretch late so that the queue never drains.
int iterate(Solve& Z, bool* converged_out) {
  drot_handle h = Z.h;
  hipStream_t stream = Z.stream;
  const plan::Static& S = Z.S;
  int slot = 0, checks = 0;
  bool converged = false;
  bool was_probe[2] = {false, false};
  h->prof_used = 0;
  while (Z.T.k < Z.P.max_iters && !converged) {
    const plan::Stretch R = plan::next_stretch(S, Z.P, Z.O, Z.T);
    const int k_end = Z.T.k + R.chunk;
    for (int c = 0; Z.T.k < k_end; ++c) {
      const plan::Step Q = plan::next_sweep(S, Z.P, Z.O, Z.T, R, c);
      const bool timed = h->profile && h->prof_used < kMaxProfiled;
      const int pe = h->prof_used;
      if (timed) {
        h->prof_kind[pe] = Q.profile_kind;
        h->prof_iters[pe] = Q.iters;
        ++h->prof_used;
      }
      // (profile mode: the pair of events takes the start and the end of the sweep kernel itself)
      enqueue_sweep(Z, Q, timed, timed ? h->prof_ev[2 * pe] : nullptr, timed ? h->prof_ev[2 * pe + 1] : nullptr);
      if (timed) {
        const bool per_workgroup = Q.sweep == plan::kLean || Q.sweep == plan::kPointsLean;
        if (Q.sweep == plan::kScreened8 || per_workgroup)  // (one count per wave of the 8-wave tiles, one per workgroup of the lean kernels)
          hipLaunchKernelGGL(sum_counts_kernel<int>, dim3(1), dim3(1024), 0, stream,
                             (const int*)(per_workgroup ? h->wg_reads : h->wave_reads),
                             per_workgroup ? S.nseg * ceil_div(S.ntr_tall, kLeanWaves) : S.nseg * S.ntr_tall * kScreenWaves,
                             h->prof_counts + 2 * pe);
      }
      enqueue_update(Z, Q);
      if (timed && Q.update != plan::kNoUpdate && Q.sweep != plan::kResident)
        // (the reduction leaves, per workgroup of 64 rows, how many of their row-segment sums are not zero)
        hipLaunchKernelGGL(sum_counts_kernel<double>, dim3(1), dim3(1024), 0, stream,
                           (const double*)(h->part + 2 * (S.nbm + S.nbn)), S.nbm, h->prof_counts + 2 * pe + 1);
    }
    if (S.status_at_checks) {
      // the test runs on the device; the host reads it one stretch late so the queue never drains
      if (R.gap) enqueue_gap(Z, h->done, true);  // (behind the stop flag: it runs only if every sweep before it ran)
      enqueue_status(Z, Z.T.k, Z.P.checking && !R.probe, R.gap);
      if (!Z.P.feedback) {  // (the stop flag alone ends the solve: the sweeps queued behind it return at once)
        DROT_HIP(hipGetLastError());
        continue;
      }
      DROT_HIP(hipMemcpyAsync(&h->host_status[slot], h->status, sizeof(DeviceStatus), hipMemcpyDeviceToHost, stream));
      DROT_HIP(hipEventRecord(h->ev[slot], stream));
      was_probe[slot] = R.probe;
      if (checks > 0) {
        DROT_HIP(hipEventSynchronize(h->ev[slot ^ 1]));
        const DeviceStatus& st = h->host_status[slot ^ 1];
        if (st.converged) converged = true;
        if (!was_probe[slot ^ 1]) record_check(h, st);
        plan::on_status(S, Z.T, st.nz_segments / ((double)Z.m * (double)S.nseg), was_probe[slot ^ 1]);
      }
      slot ^= 1;
      ++checks;
      DROT_HIP(hipGetLastError());
    }
  }
  if (checks > 0) {  // the last stretch's status has not been looked at yet
    DROT_HIP(hipEventSynchronize(h->ev[slot ^ 1]));
    if (!was_probe[slot ^ 1]) record_check(h, h->host_status[slot ^ 1]);
  }
  *converged_out = converged;
  return DROT_OK;
}

int solve_impl(drot_handle h, const SolveCall& A) {
  Solve Z;
  int rc = prepare(h, A, Z);
  if (rc != DROT_OK) {
    if (h && rc != DROT_ERR_INVALID_ARG) {  // (work may be queued: let it drain, and trust nothing it left)
      (void)hipStreamSynchronize(reinterpret_cast<hipStream_t>(A.stream));
      h->solved = false;
      h->carry = plan::Carry{};
    }
    return rc;
  }
  hipStream_t stream = Z.stream;
  const plan::Static& S = Z.S;
  h->carry.sums_valid = h->carry.lines_valid = false;  // (until this solve has returned)
  h->checks.clear();
  auto fail = [&](int code) {
    (void)hipStreamSynchronize(stream);
    (void)hipGetLastError();
    h->solved = false;
    h->carry = plan::Carry{};
    return code;
  };
  bool converged = false;
  rc = iterate(Z, &converged);
  if (rc != DROT_OK) return fail(rc);
  const int k = Z.T.k;
  // final state: residuals of the returned iterate (no-op if the stop flag is already up)
  if (k > 0) enqueue_status(Z, k, Z.P.checking, false);
  // (a stop seen in the loop means the last stretch was enqueued behind it and did not run; without feedback
  // the host cannot tell)
  if (h->compute_gap) enqueue_gap(Z, nullptr, !converged && (Z.P.feedback || !Z.P.checking));
  const bool untouched = A.max_iters == 0 && !Z.P.resume && !A.warm;
  if (S.pad_x && !untouched) copy_rows(A.X_out, (size_t)Z.n, h->xpad, (size_t)S.ld_pad, Z.m, Z.n, stream);
  if (hipMemcpyAsync(&h->host_status[0], h->status, sizeof(DeviceStatus), hipMemcpyDeviceToHost, stream) != hipSuccess ||
      hipStreamSynchronize(stream) != hipSuccess || hipGetLastError() != hipSuccess)
    return fail(DROT_ERR_HIP);

  const DeviceStatus& st = h->host_status[0];
  h->prof_count = 0;
  if (h->profile) {
    const int timed = h->prof_used;
    if (timed > 0 && hipMemcpy(h->prof_counts_host, h->prof_counts, sizeof(double) * 2 * (size_t)timed,
                               hipMemcpyDeviceToHost) != hipSuccess)
      return fail(DROT_ERR_HIP);
    for (int e = 0; e < timed; ++e) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, h->prof_ev[2 * e], h->prof_ev[2 * e + 1]) != hipSuccess) return fail(DROT_ERR_HIP);
      h->prof_ms[e] = ms / (float)h->prof_iters[e];  // per iteration (a resident stretch is one launch)
    }
    h->prof_count = timed;
  }
  const int iters = A.max_iters == 0 ? 0 : st.iters;
  h->info.iters = iters;
  h->info.converged = st.converged;
  // with zero iterations X = 0 and no sums were formed: report the residuals as not evaluated
  h->info.r_row = A.max_iters == 0 ? INFINITY : (float)std::sqrt(st.r2);
  h->info.r_col = A.max_iters == 0 ? INFINITY : (float)std::sqrt(st.s2);
  h->info.objective = h->compute_gap ? st.cost + st.h : 0.0;
  h->info.gap = h->compute_gap ? st.gap : 0.0;
  h->info.dual_res = h->compute_gap ? st.dual_res : 0.0;
  h->carry = plan::finish(S, Z.P, Z.T, st.converged != 0, iters);
  h->xpad_live = S.pad_x && !untouched;
  h->solved = true;
  h->last_m = Z.m;
  h->last_n = Z.n;
  if (Z.P.checking && !st.converged) return DROT_MAX_ITERS;
  return DROT_OK;
}

// ------------------------------------------------------------------------------------------
// drot_solve_static: the same solve out of a workspace that is part of the loaded code object, for
// callers that cannot allocate.  Every GPU holds its own copy of the array at its own address.
// ------------------------------------------------------------------------------------------
constexpr int kStaticMaxM = DROT_STATIC_MAX_M, kStaticMaxN = DROT_STATIC_MAX_N;
constexpr size_t kScratchBytes = (size_t)6 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch`, per device (the array's name is no device address on the host)
std::mutex g_scratch_mutex;

int static_workspace(int device, unsigned char** out) {
  if (device < 0 || device >= kMaxDevices) return DROT_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      fprintf(stderr, "drot: hipGetSymbolAddress(scratch) failed: %s\n", hipGetErrorString(e));
      return DROT_ERR_HIP;
    }
    g_scratch_ptr[device] = ptr;
  }
  *out = static_cast<unsigned char*>(g_scratch_ptr[device]);
  return DROT_OK;
}

// Points the workspace fields of a handle into `base` (a stretch of at least kScratchBytes bytes, 256-byte
// aligned), sized for problems up to kStaticMaxM x kStaticMaxN without group lasso.  Returns the bytes used.
size_t carve_static(drot_handle_s& H, unsigned char* base) {
  size_t off = 0;
  auto take = [&](auto** field, size_t count) {
    using T = std::remove_pointer_t<std::remove_pointer_t<decltype(field)>>;
    *field = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off = (off + count * sizeof(T) + 255) & ~(size_t)255;
  };
  const size_t M = kStaticMaxM, N = kStaticMaxN;
  static_assert(kStaticMaxM % 64 == 0 && kStaticMaxN % 64 == 0, "the pitches of the partial sums are the sizes themselves");
  const size_t nseg = ceil_div(kStaticMaxN, kSegCols), ntr = ceil_div(kStaticMaxM, kTileRows);
  const size_t nb = ceil_div(kStaticMaxM, 64) + ceil_div(kStaticMaxN, 64);
  H.max_m = kStaticMaxM;
  H.max_n = kStaticMaxN;
  H.rowpart_half = nseg * M;  // (256-column segments only: no group-resident path here)
  H.colpart_half = ntr * N;
  H.tilesum_half = nseg * ntr > 4096 ? nseg * ntr : 4096;
  H.max_runs = 0;
  take(&H.phi, M);
  take(&H.varphi, nseg * kSegCols);  // (to the end of the last column segment: see mask_tail_kernel)
  take(&H.a, 2 * M);
  take(&H.b, 2 * N);
  take(&H.theta, 2);
  take(&H.sum_p, 1);
  take(&H.r, M);
  take(&H.s, N);
  take(&H.part, 3 * nb);
  take(&H.resid, 3);
  take(&H.rowpart, 2 * H.rowpart_half);
  take(&H.colpart, 2 * H.colpart_half);
  take(&H.tilesum, 2 * H.tilesum_half);
  take(&H.mprime, nseg * M);
  take(&H.mprime2, nseg * M);
  take(&H.jstar, nseg * M);
  take(&H.varphi0, nseg * kSegCols);
  take(&H.screen_ctl, (size_t)kCtlWords);
  take(&H.xlines, nseg * M);
  take(&H.wg_reads, nseg * (size_t)ceil_div(ceil_div(kStaticMaxM, 64), kLeanWaves));
  take(&H.gap_part, nseg * ntr * 3);
  take(&H.done, 1);
  take(&H.status, 1);
  return off;
}

// Result block and dual vectors from the workspace into the caller's device buffers.
__global__ __launch_bounds__(256) void export_kernel(const DeviceStatus* __restrict__ st, drot_info* __restrict__ info,
                                                     const float* __restrict__ phi, const float* __restrict__ varphi,
                                                     float* __restrict__ phi_out, float* __restrict__ varphi_out, int m, int n,
                                                     int max_iters) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x, stride = gridDim.x * blockDim.x;
  if (phi_out)
    for (int i = t; i < m; i += stride) phi_out[i] = phi[i];
  if (varphi_out)
    for (int j = t; j < n; j += stride) varphi_out[j] = varphi[j];
  if (t == 0 && info) {
    info->iters = max_iters == 0 ? 0 : st->iters;
    info->converged = st->converged;
    info->r_row = max_iters == 0 ? INFINITY : (float)sqrt(st->r2);
    info->r_col = max_iters == 0 ? INFINITY : (float)sqrt(st->s2);
    info->objective = st->cost + st->h;
    info->gap = st->gap;
    info->dual_res = st->dual_res;
  }
}

int solve_static_impl(SolveCall A, float* phi_out, float* varphi_out, drot_info* info_out) {
  if (!A.cost.C || !A.p || !A.q || !A.X_out) return DROT_ERR_INVALID_ARG;
  if (A.m < 1 || A.n < 1 || A.max_iters < 0) return DROT_ERR_INVALID_ARG;
  if (A.m > kStaticMaxM || A.n > kStaticMaxN) {
    fprintf(stderr, "drot_solve_static: %d x %d exceeds the static workspace (at most %d x %d)\n", A.m, A.n, kStaticMaxM,
            kStaticMaxN);
    return DROT_ERR_TOO_LARGE;
  }
  // the paths that need memory of a size only known at run time are not available here
  if (A.reg_kind == DROT_REG_GROUP_LASSO || (A.reg_params && A.reg_params->weights)) return DROT_ERR_INVALID_ARG;
  if (A.n % kAlignElems != 0 || reinterpret_cast<uintptr_t>(A.cost.C) % 128 != 0 ||
      reinterpret_cast<uintptr_t>(A.X_out) % 128 != 0) {
    fprintf(stderr, "drot_solve_static: rows of C and X_out must start on 128-byte lines (n %% 32 == 0, aligned bases)\n");
    return DROT_ERR_INVALID_ARG;
  }
  static_assert(sizeof(drot_handle_s) < (1 << 16), "lives on the stack here");
  drot_handle_s H;  // a handle whose workspace is the static array; it owns nothing
  if (carve_static(H, nullptr) > kScratchBytes) return DROT_ERR_ALLOC;
  DROT_HIP(hipGetDevice(&H.device));
  unsigned char* base = nullptr;
  int rc = static_workspace(H.device, &base);
  if (rc != DROT_OK) return rc;
  carve_static(H, base);
  A.fixed_schedule = true;
  Solve Z;
  rc = prepare(&H, A, Z);
  if (rc != DROT_OK) return rc;
  if (Z.S.pad_c || Z.S.pad_x) return DROT_ERR_INVALID_ARG;  // (checked above; nothing has been queued that matters)
  bool converged = false;
  rc = iterate(Z, &converged);
  if (rc != DROT_OK) return rc;
  if (Z.T.k > 0) enqueue_status(Z, Z.T.k, Z.P.checking, false);
  enqueue_gap(Z, nullptr, false);
  hipLaunchKernelGGL(export_kernel, dim3(16), dim3(256), 0, Z.stream, (const DeviceStatus*)H.status, info_out,
                     (const float*)H.phi, (const float*)H.varphi, phi_out, varphi_out, A.m, A.n, A.max_iters);
  DROT_HIP(hipGetLastError());
  return DROT_OK;
}

}  // namespace

extern "C" {

const char* drot_strerror(int code) {
  switch (code) {
    case DROT_OK: return "ok";
    case DROT_MAX_ITERS: return "maximum number of iterations reached before the tolerance";
    case DROT_ERR_INVALID_ARG: return "invalid argument";
    case DROT_ERR_ALLOC: return "device or pinned-host allocation failed";
    case DROT_ERR_HIP: return "HIP runtime error";
    case DROT_ERR_NOT_INITIALIZED: return "no solve has been run on this handle";
    case DROT_ERR_TOO_LARGE: return "the problem exceeds the fixed workspace of drot_solve_static";
    default: return "unknown code";
  }
}

int drot_create(drot_handle* out, int max_m, int max_n) {
  if (!out || max_m < 1 || max_n < 1) return DROT_ERR_INVALID_ARG;
  *out = nullptr;
  drot_handle h = new (std::nothrow) drot_handle_s();
  if (!h) return DROT_ERR_ALLOC;
  if (hipGetDevice(&h->device) != hipSuccess) {
    delete h;
    return DROT_ERR_HIP;
  }
  h->max_m = max_m;
  h->max_n = max_n;
  const size_t nseg = (size_t)ceil_div(max_n, kSegCols);
  const size_t ntr = (size_t)ceil_div(max_m, kTileRows);
  const size_t nb = (size_t)ceil_div(max_m, 64) + (size_t)ceil_div(max_n, 64);
  int rc = DROT_OK;
  auto take = [&](int r) { if (rc == DROT_OK) rc = r; };
  take(dev_alloc(&h->phi, (size_t)max_m));
  take(dev_alloc(&h->varphi, nseg * kSegCols));  // (to the end of the last column segment: see mask_tail_kernel)
  take(dev_alloc(&h->a, 2 * (size_t)max_m));
  take(dev_alloc(&h->b, 2 * (size_t)max_n));
  take(dev_alloc(&h->theta, 2));
  take(dev_alloc(&h->sum_p, 1));
  take(dev_alloc(&h->r, (size_t)max_m));
  take(dev_alloc(&h->s, (size_t)max_n));
  take(dev_alloc(&h->part, 3 * nb));
  take(dev_alloc(&h->resid, 3));
  // (rows of the per-row-segment arrays and of the column sums are pitched at multiples of 64 entries)
  const size_t mpad = (size_t)ceil_div(max_m, 64) * 64, npad = (size_t)ceil_div(max_n, 64) * 64;
  h->rowpart_half = (size_t)ceil_div(max_n, kSlabCols) * mpad;  // 32-column strips (group-resident path) are the finest
  h->colpart_half = ntr * npad;
  h->tilesum_half = nseg * ntr > 4096 ? nseg * ntr : 4096;  // (the group-resident path has up to 4096 slabs)
  take(dev_alloc(&h->rowpart, 2 * h->rowpart_half));
  take(dev_alloc(&h->colpart, 2 * h->colpart_half));
  take(dev_alloc(&h->tilesum, 2 * h->tilesum_half));
  take(dev_alloc(&h->mprime, nseg * mpad));
  take(dev_alloc(&h->mprime2, nseg * mpad));
  take(dev_alloc(&h->jstar, nseg * mpad));
  take(dev_alloc(&h->varphi0, nseg * kSegCols));
  take(dev_alloc(&h->screen_ctl, (size_t)kCtlWords));
  take(dev_alloc(&h->xlines, nseg * mpad));
  take(dev_alloc(&h->wg_reads, nseg * (size_t)ceil_div(ceil_div(max_m, 64), kLeanWaves)));
  h->max_runs = (int)ntr;
  take(dev_alloc(&h->gap_part, nseg * ntr * 3));
  take(dev_alloc(&h->done, 1));
  take(dev_alloc(&h->status, 1));
  if (rc == DROT_OK && hipHostMalloc(reinterpret_cast<void**>(&h->host_status), 2 * sizeof(DeviceStatus)) != hipSuccess) {
    h->host_status = nullptr;
    rc = DROT_ERR_ALLOC;
  }
  for (auto& e : h->ev)
    if (rc == DROT_OK && hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
      e = nullptr;
      rc = DROT_ERR_HIP;
    }
  if (rc != DROT_OK) {
    free_all(h);
    delete h;
    (void)hipGetLastError();
    return rc;
  }
  *out = h;
  return DROT_OK;
}

int drot_destroy(drot_handle h) {
  if (!h) return DROT_ERR_INVALID_ARG;
  free_all(h);
  delete h;
  return DROT_OK;
}

int drot_set_option(drot_handle h, drot_option option, int value) {
  if (!h) return DROT_ERR_INVALID_ARG;
  auto in = [&](int lo, int hi) { return value >= lo && value <= hi; };
  switch (option) {
    case DROT_OPT_CHECK_EVERY:
      if (value < 1) return DROT_ERR_INVALID_ARG;
      h->opt.check_every = value;
      return DROT_OK;
    case DROT_OPT_COMPUTE_GAP: h->compute_gap = value ? 1 : 0; return DROT_OK;
    case DROT_OPT_GAP_EVERY:
      if (value < 0) return DROT_ERR_INVALID_ARG;
      h->opt.gap_every = value;
      return DROT_OK;
    case DROT_OPT_CONTINUE: h->continue_next = value ? 1 : 0; return DROT_OK;
    case DROT_OPT_PROFILE:
      if (value) {
        const int rc = enable_profile(h);
        if (rc != DROT_OK) return rc;
      }
      h->profile = value ? 1 : 0;
      return DROT_OK;
    case DROT_OPT_SKIP_UNCHANGED:
      if (!in(-1, 1)) return DROT_ERR_INVALID_ARG;
      h->opt.skip_unchanged = value;
      return DROT_OK;
    case DROT_OPT_SCREENING:
      if (!in(-1, 100000)) return DROT_ERR_INVALID_ARG;
      h->opt.screening = value;
      return DROT_OK;
    case DROT_OPT_SKIP_COST:
      if (!in(-1, 1)) return DROT_ERR_INVALID_ARG;
      h->opt.skip_cost = value;
      return DROT_OK;
    case DROT_OPT_FUSED_UPDATE:
      if (!in(-1, 0)) return DROT_ERR_INVALID_ARG;
      h->opt.fused_update = value;
      return DROT_OK;
    case DROT_OPT_RESIDENT:
      if (!in(-1, 0)) return DROT_ERR_INVALID_ARG;
      h->opt.resident = value;
      return DROT_OK;
    case DROT_OPT_GROUP_TWO_PASS: h->opt.force_two_pass = value ? 1 : 0; return DROT_OK;
    case DROT_OPT_NONTEMPORAL:
      if (!in(-1, 1)) return DROT_ERR_INVALID_ARG;
      h->opt.nontemporal = value;
      return DROT_OK;
  }
  return DROT_ERR_INVALID_ARG;
}

int drot_set_gap_tolerance(drot_handle h, float gap_tol) {
  if (!h || !(gap_tol >= 0.f)) return DROT_ERR_INVALID_ARG;
  h->gap_tol = gap_tol;
  return DROT_OK;
}

int drot_get_checks(drot_handle h, drot_check* out, int capacity, int* count) {
  if (!h || !out || capacity < 0 || !count) return DROT_ERR_INVALID_ARG;
  if (!h->solved) return DROT_ERR_NOT_INITIALIZED;
  *count = (int)h->checks.size();
  for (int e = 0; e < *count && e < capacity; ++e) out[e] = h->checks[(size_t)e];
  return DROT_OK;
}

int drot_get_profile(drot_handle h, drot_sweep_timing* out, int capacity, int* count) {
  if (!h || !out || capacity < 0 || !count) return DROT_ERR_INVALID_ARG;
  if (!h->solved) return DROT_ERR_NOT_INITIALIZED;
  *count = h->prof_count;
  const double segments = (double)h->last_m * (double)ceil_div(h->last_n, kSegCols);
  for (int e = 0; e < h->prof_count && e < capacity; ++e) {
    const int kind = h->prof_kind[e];
    out[e].ms = h->prof_ms[e];
    out[e].kind = kind;
    out[e].c_fraction = (kind >= 5 && kind <= 8) ? h->prof_counts_host[2 * e] / segments : (kind == 2 ? 0.0 : 1.0);
    out[e].x_fraction = kind >= 4 ? h->prof_counts_host[2 * e + 1] / segments : -1.0;
  }
  return DROT_OK;
}

int drot_solve(drot_handle h, const float* C, const float* p, const float* q, int m, int n, float stepsize,
               drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters, float tol,
               float* X_out, void* stream) {
  if (!C) return DROT_ERR_INVALID_ARG;
  SolveCall A;
  A.cost.C = C;
  A.p = p; A.q = q; A.m = m; A.n = n; A.stepsize = stepsize; A.reg_kind = reg_kind; A.reg_params = reg_params;
  A.max_iters = max_iters; A.tol = tol; A.X_out = X_out; A.stream = stream;
  return solve_impl(h, A);
}

int drot_solve_points(drot_handle h, const float* xs, const float* xt, int d, float cost_scale, const float* p,
                      const float* q, int m, int n, float stepsize, drot_reg_kind reg_kind,
                      const drot_reg_params* reg_params, int max_iters, float tol, float* X_out, void* stream) {
  if (!xs || !xt) return DROT_ERR_INVALID_ARG;
  SolveCall A;
  A.cost.xs = xs; A.cost.xt = xt; A.cost.d = d; A.cost.scale = cost_scale;
  A.p = p; A.q = q; A.m = m; A.n = n; A.stepsize = stepsize; A.reg_kind = reg_kind; A.reg_params = reg_params;
  A.max_iters = max_iters; A.tol = tol; A.X_out = X_out; A.stream = stream;
  return solve_impl(h, A);
}

int drot_solve_points_warm(drot_handle h, const float* xs, const float* xt, int d, float cost_scale, const float* p,
                           const float* q, int m, int n, float stepsize, drot_reg_kind reg_kind,
                           const drot_reg_params* reg_params, int max_iters, float tol, float* X_inout, const float* phi0,
                           const float* varphi0, void* stream) {
  if (!xs || !xt) return DROT_ERR_INVALID_ARG;
  SolveCall A;
  A.cost.xs = xs; A.cost.xt = xt; A.cost.d = d; A.cost.scale = cost_scale;
  A.p = p; A.q = q; A.m = m; A.n = n; A.stepsize = stepsize; A.reg_kind = reg_kind; A.reg_params = reg_params;
  A.max_iters = max_iters; A.tol = tol; A.X_out = X_inout; A.phi0 = phi0; A.varphi0 = varphi0; A.warm = true;
  A.stream = stream;
  return solve_impl(h, A);
}

int drot_solve_warm(drot_handle h, const float* C, const float* p, const float* q, int m, int n, float stepsize,
                    drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters, float tol,
                    float* X_inout, const float* phi0, const float* varphi0, void* stream) {
  if (!C) return DROT_ERR_INVALID_ARG;
  SolveCall A;
  A.cost.C = C;
  A.p = p; A.q = q; A.m = m; A.n = n; A.stepsize = stepsize; A.reg_kind = reg_kind; A.reg_params = reg_params;
  A.max_iters = max_iters; A.tol = tol; A.X_out = X_inout; A.phi0 = phi0; A.varphi0 = varphi0; A.warm = true;
  A.stream = stream;
  return solve_impl(h, A);
}

int drot_solve_static(const float* C, const float* p, const float* q, int m, int n, float stepsize,
                      drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters, float tol, float* X_out,
                      float* phi_out, float* varphi_out, drot_info* info_out, void* stream) {
  SolveCall A;
  A.cost.C = C;
  A.p = p; A.q = q; A.m = m; A.n = n; A.stepsize = stepsize; A.reg_kind = reg_kind; A.reg_params = reg_params;
  A.max_iters = max_iters; A.tol = tol; A.X_out = X_out; A.stream = stream;
  return solve_static_impl(A, phi_out, varphi_out, info_out);
}

int drot_get_info(drot_handle h, drot_info* out) {
  if (!h || !out) return DROT_ERR_INVALID_ARG;
  if (!h->solved) return DROT_ERR_NOT_INITIALIZED;
  *out = h->info;
  return DROT_OK;
}

int drot_get_duals(drot_handle h, float* phi_out, float* varphi_out) {
  if (!h) return DROT_ERR_INVALID_ARG;
  if (!h->solved) return DROT_ERR_NOT_INITIALIZED;
  if (phi_out)
    DROT_HIP(hipMemcpy(phi_out, h->phi, sizeof(float) * (size_t)h->last_m, hipMemcpyDeviceToDevice));
  if (varphi_out)
    DROT_HIP(hipMemcpy(varphi_out, h->varphi, sizeof(float) * (size_t)h->last_n, hipMemcpyDeviceToDevice));
  return DROT_OK;
}

}  // extern "C"
