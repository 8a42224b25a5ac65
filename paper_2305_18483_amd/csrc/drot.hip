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
//   rowpart     [nseg][m]  fp32: row sums of every 256-column segment
//   colpart     [ntr][n]   fp32: column sums of every 32-row tile
//
//   colpart     ... or of every 64-row tile (sweeps for sparse plans), or of four of them (lean sweep)
//
// This translation unit is the whole product path.  The kernels live in the drot_*.h files next to
// it (sweep, screened sweeps, point-cloud cost, group lasso, dual vectors, resident solver, gap);
// this file holds the launch helpers, the handle, the host loop and the C ABI of include/drot.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "drot.h"

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
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Non-temporal accesses pay off once X and C together no longer fit the 256 MB memory-side cache;
// below that, keeping the lines cached is the better choice.  Measured crossover on MI355X:
// cacheable wins at 8mn = 290 MB (7.2 vs 6.1 TB/s), non-temporal wins at 393 MB (6.1 vs 5.7 TB/s).
inline bool use_nontemporal(int m, int n) { return 8.0 * (double)m * (double)n > 320.0 * 1024 * 1024; }
template <bool FIRST, bool PRO>
void launch_slab_k(int k, dim3 grid, hipStream_t stream, const SlabArgs& a, const FusedUpdateArgs& f) {
  const dim3 block(kSlabThreads);
  switch (k) {
    case 1: hipLaunchKernelGGL((gl_slab_kernel<FIRST, 1, kSlabLanes, PRO>), grid, block, 0, stream, a, f); break;
    case 2: hipLaunchKernelGGL((gl_slab_kernel<FIRST, 2, kSlabLanes, PRO>), grid, block, 0, stream, a, f); break;
    case 4: hipLaunchKernelGGL((gl_slab_kernel<FIRST, 4, kSlabLanes, PRO>), grid, block, 0, stream, a, f); break;
    default: hipLaunchKernelGGL((gl_slab_kernel<FIRST, 8, kSlabLanes, PRO>), grid, block, 0, stream, a, f); break;
  }
}
void launch_slab(bool first, bool pro, int k, dim3 grid, hipStream_t stream, const SlabArgs& a, const FusedUpdateArgs& f) {
  if (pro) launch_slab_k<false, true>(k, grid, stream, a, f);
  else if (first) launch_slab_k<true, false>(k, grid, stream, a, f);
  else launch_slab_k<false, false>(k, grid, stream, a, f);
}

constexpr int kMaxProfiled = 256;  // sweeps timed per solve in profile mode
// Screening on automatic: from this many entries up (about 3400 x 3400).  Measured to a residual of
// 1e-4 on two kinds of problem: equal at 3000 x 3000, 15 % faster at 3500 x 3500, 30-40 % at
// 4096 x 4096 and 5000 x 5000; below, the whole of C streams from the caches as fast.
constexpr size_t kScreenFrom = (size_t)11 << 20;

}  // namespace

struct drot_handle_s {
  int device = -1;
  int max_m = 0, max_n = 0;
  int check_every = 100;
  int compute_gap = 1;
  int continue_next = 0;  // the next solve resumes from the state the last one left
  int profile = 0;        // record HIP events around every sweep launch
  int force_two_pass = 0; // group lasso: always take the general two-pass path
  int nontemporal = -1;   // -1: by problem size, 0: never, 1: always
  int screening = -1;       // sparse plans also skip the reads of C that a bound certifies useless: -1 for problems
                            // of kScreenFrom entries and more, 1 always, k >= 2 always and with the bounds renewed at
                            // least every k sweeps (default 256), 0 never
  int skip_unchanged = -1;  // -1/1: unchanged row segments are not written back, 0: every segment is stored
  bool dense_plan = false;  // what the last solve's density feedback ended on
  double plan_density = -1.0;
  long long epoch_gen = -1;  // screening: sweep that recorded the bounds in mprime (continued solves)
  bool sums_valid = false;   // rowpart of the last generation describes the X the solve returned
  int sums_strip = 0;        // ... in pieces of this many columns (256, or 32 on the group-resident path)
  int refresh_period = 8;
  int resident = -1;      // -1: tiny problems run in the one-workgroup resident kernel, 0: never
  int fused_update = -1;  // -1: for small problems, 0: never (always separate reduce + update kernels)
  int skip_cost = -1;     // even/odd scheme (C read every second sweep): -1 where it applies unless the update is fused, 0 never, 1 where it applies
  bool solved = false;
  int last_m = 0, last_n = 0;
  long long iters_done = 0;  // iterations applied to the state held by this handle
  // sweep timing (profile mode): event pairs recorded on the solve's stream
  hipEvent_t prof_ev[2 * kMaxProfiled] = {};
  hipEvent_t cal_ev[8] = {};  // four empty event pairs per profiled solve: what a pair costs without a kernel between
  double prof_overhead_ms = 0.0;
  int prof_count = 0;
  double prof_sweep_ms = 0.0;
  float prof_ms[kMaxProfiled] = {};  // per sweep, in launch order
  int prof_kind[kMaxProfiled] = {};  // 0: reads X and C, 1: the same and stores X - rho*C, 2: reads the shifted X only, 3: resident stretch, 4: as 0 on 64-row tiles with the zero-segment skipping
  int prof_iters[kMaxProfiled] = {}; // iterations the timed launch covers (1 unless resident)
  int prof_used = 0;
  // device workspace
  float *phi = nullptr, *varphi = nullptr;
  // a, b, rowpart, colpart, tilesum are double buffers (two halves), indexed by iteration parity
  double *a = nullptr, *b = nullptr, *theta = nullptr, *sum_p = nullptr, *r = nullptr, *s = nullptr, *part = nullptr,
         *resid = nullptr;
  float *rowpart = nullptr, *colpart = nullptr, *tilesum = nullptr, *gap_part = nullptr;
  size_t rowpart_half = 0, colpart_half = 0, tilesum_half = 0;
  float *mprime = nullptr, *varphi0 = nullptr;  // screened sweep: per-row-segment bounds and the epoch's varphi
  int* screen_ctl = nullptr;      // control words of the lean sweep's refresh schedule
  unsigned char* xlines = nullptr;  // [nseg][m] nonzero 128-byte lines of every row segment of X (lean sweep)
  bool lines_valid = false;       // xlines describes the X the last solve returned
  int* wg_reads = nullptr;        // per-workgroup read counts of the lean sweep
  int* wave_reads = nullptr;      // profiling: per-wave read counts of a screened sweep (allocated with the events)
  size_t wave_reads_len = 0;
  double* prof_reads = nullptr;   // profiling: [kMaxProfiled] row segments of C read by each timed sweep (device)
  double prof_reads_host[kMaxProfiled] = {};
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
  int max_runs = 0;       // rows of colpart available
  int* done = nullptr;
  DeviceStatus* status = nullptr;
  // pinned host mirror of the status block, two slots for the pipelined residual checks
  DeviceStatus* host_status = nullptr;
  hipEvent_t ev[2] = {nullptr, nullptr};
  drot_info info{};
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

void free_all(drot_handle h) {
  float* fbufs[] = {h->phi, h->varphi, h->rowpart, h->colpart, h->tilesum, h->gap_part, h->gbuf, h->mprime, h->varphi0};
  double* dbufs[] = {h->a, h->b, h->theta, h->sum_p, h->r, h->s, h->part, h->resid};
  for (float* b : fbufs) (void)hipFree(b);
  for (double* b : dbufs) (void)hipFree(b);
  (void)hipFree(h->done);
  (void)hipFree(h->status);
  (void)hipFree(h->runbuf);
  (void)hipFree(h->cpad);
  (void)hipFree(h->ptbuf);
  (void)hipFree(h->xpad);
  if (h->host_status) (void)hipHostFree(h->host_status);
  for (auto& e : h->ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& e : h->prof_ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& e : h->cal_ev)
    if (e) (void)hipEventDestroy(e);
  (void)hipFree(h->wave_reads);
  (void)hipFree(h->prof_reads);
  (void)hipFree(h->screen_ctl);
  (void)hipFree(h->xlines);
  (void)hipFree(h->wg_reads);
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
  take(dev_alloc(&h->varphi, (size_t)max_n + 4));
  take(dev_alloc(&h->a, 2 * (size_t)max_m));
  take(dev_alloc(&h->b, 2 * (size_t)max_n));
  take(dev_alloc(&h->theta, 2));
  take(dev_alloc(&h->sum_p, 1));
  take(dev_alloc(&h->r, (size_t)max_m));
  take(dev_alloc(&h->s, (size_t)max_n));
  take(dev_alloc(&h->part, 3 * nb));
  take(dev_alloc(&h->resid, 3));
  h->rowpart_half = (size_t)ceil_div(max_n, kSlabCols) * (size_t)max_m;  // 32-column strips (group-resident path) are the finest
  h->colpart_half = ntr * (size_t)max_n;
  h->tilesum_half = nseg * ntr > 4096 ? nseg * ntr : 4096;  // (the group-resident path has up to 4096 slabs)
  take(dev_alloc(&h->rowpart, 2 * h->rowpart_half));
  take(dev_alloc(&h->colpart, 2 * h->colpart_half));
  take(dev_alloc(&h->tilesum, 2 * h->tilesum_half));
  take(dev_alloc(&h->mprime, nseg * (size_t)max_m));
  take(dev_alloc(&h->varphi0, (size_t)max_n));
  take(dev_alloc(&h->screen_ctl, (size_t)kCtlWords));
  take(dev_alloc(&h->xlines, nseg * (size_t)max_m));
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

int drot_set_check_every(drot_handle h, int check_every) {
  if (!h || check_every < 1) return DROT_ERR_INVALID_ARG;
  h->check_every = check_every;
  return DROT_OK;
}

int drot_set_compute_gap(drot_handle h, int enable) {
  if (!h) return DROT_ERR_INVALID_ARG;
  h->compute_gap = enable ? 1 : 0;
  return DROT_OK;
}

int drot_set_continue(drot_handle h, int enable) {
  if (!h) return DROT_ERR_INVALID_ARG;
  h->continue_next = enable ? 1 : 0;
  return DROT_OK;
}

int drot_set_group_two_pass(drot_handle h, int enable) {
  if (!h) return DROT_ERR_INVALID_ARG;
  h->force_two_pass = enable ? 1 : 0;
  return DROT_OK;
}

int drot_set_nontemporal(drot_handle h, int mode) {
  if (!h || mode < -1 || mode > 1) return DROT_ERR_INVALID_ARG;
  h->nontemporal = mode;
  return DROT_OK;
}

int drot_set_fused_update(drot_handle h, int mode) {
  if (!h || mode < -1 || mode > 0) return DROT_ERR_INVALID_ARG;
  h->fused_update = mode;
  return DROT_OK;
}

int drot_set_skip_unchanged(drot_handle h, int mode) {
  if (!h || mode < -1 || mode > 1) return DROT_ERR_INVALID_ARG;
  h->skip_unchanged = mode;
  return DROT_OK;
}

int drot_set_screening(drot_handle h, int mode) {
  if (!h || mode < -1 || mode > 100000) return DROT_ERR_INVALID_ARG;
  h->screening = mode;
  return DROT_OK;
}

int drot_set_resident(drot_handle h, int mode) {
  if (!h || mode < -1 || mode > 0) return DROT_ERR_INVALID_ARG;
  h->resident = mode;
  return DROT_OK;
}

int drot_set_skip_cost(drot_handle h, int mode) {
  if (!h || mode < -1 || mode > 1) return DROT_ERR_INVALID_ARG;
  h->skip_cost = mode;
  return DROT_OK;
}

int drot_set_profile(drot_handle h, int enable) {
  if (!h) return DROT_ERR_INVALID_ARG;
  if (enable) {
    // everything or nothing: a failure part of the way leaves the handle as it was
    hipEvent_t made[2 * kMaxProfiled + 8] = {};
    int nmade = 0;
    bool ok = true;
    auto make = [&](hipEvent_t& e) {
      if (!ok || e) return;
      if (hipEventCreate(&e) != hipSuccess) { e = nullptr; ok = false; return; }
      made[nmade++] = e;
    };
    for (auto& e : h->prof_ev) make(e);
    for (auto& e : h->cal_ev) make(e);
    int* wave_reads = nullptr;
    double* prof_reads = nullptr;
    // read counts of the screened sweeps: one int per wave of the largest grid, one total per timed sweep
    const size_t waves = (size_t)ceil_div(h->max_n, kSegCols) * (size_t)ceil_div(h->max_m, kScreenRows * kScreenWaves) * kScreenWaves;
    int rc = ok ? DROT_OK : DROT_ERR_HIP;
    if (rc == DROT_OK && !h->prof_reads) {
      if (hipMalloc(reinterpret_cast<void**>(&wave_reads), sizeof(int) * waves) != hipSuccess ||
          hipMalloc(reinterpret_cast<void**>(&prof_reads), sizeof(double) * kMaxProfiled) != hipSuccess)
        rc = DROT_ERR_ALLOC;
    }
    if (rc != DROT_OK) {
      (void)hipFree(wave_reads);
      (void)hipFree(prof_reads);
      for (int e = 0; e < nmade; ++e) (void)hipEventDestroy(made[e]);
      for (auto& e : h->prof_ev) for (int k = 0; k < nmade; ++k) if (e == made[k]) e = nullptr;
      for (auto& e : h->cal_ev) for (int k = 0; k < nmade; ++k) if (e == made[k]) e = nullptr;
      (void)hipGetLastError();
      return rc;
    }
    if (!h->prof_reads) {
      h->wave_reads = wave_reads;
      h->wave_reads_len = waves;
      h->prof_reads = prof_reads;
    }
  }
  h->profile = enable ? 1 : 0;
  return DROT_OK;
}

int drot_get_profile(drot_handle h, double* sweep_ms_avg, int* sweeps_timed) {
  if (!h || !sweep_ms_avg || !sweeps_timed) return DROT_ERR_INVALID_ARG;
  if (!h->solved) return DROT_ERR_NOT_INITIALIZED;
  *sweeps_timed = h->prof_count;
  *sweep_ms_avg = h->prof_count > 0 ? h->prof_sweep_ms / h->prof_count : 0.0;
  return DROT_OK;
}

int drot_get_profile_sweeps(drot_handle h, float* sweep_ms, int* sweep_kind, int capacity, int* sweeps_timed) {
  if (!h || !sweep_ms || capacity < 0 || !sweeps_timed) return DROT_ERR_INVALID_ARG;
  if (!h->solved) return DROT_ERR_NOT_INITIALIZED;
  *sweeps_timed = h->prof_count;
  for (int e = 0; e < h->prof_count && e < capacity; ++e) {
    sweep_ms[e] = h->prof_ms[e];
    if (sweep_kind) sweep_kind[e] = h->prof_kind[e];
  }
  return DROT_OK;
}

int drot_get_profile_reads(drot_handle h, double* c_fraction, int capacity, int* sweeps_timed) {
  if (!h || !c_fraction || capacity < 0 || !sweeps_timed) return DROT_ERR_INVALID_ARG;
  if (!h->solved) return DROT_ERR_NOT_INITIALIZED;
  *sweeps_timed = h->prof_count;
  const double segments = (double)h->last_m * (double)ceil_div(h->last_n, kSegCols);
  for (int e = 0; e < h->prof_count && e < capacity; ++e)
    c_fraction[e] = h->prof_kind[e] >= 5 ? h->prof_reads_host[e] / segments
                    : (h->prof_kind[e] == 2 ? 0.0 : 1.0);
  return DROT_OK;
}

// Where the cost comes from: a stored matrix, or two point clouds (C_ij = scale * ||xs_i - xt_j||^2).
struct CostSource {
  const float* C = nullptr;
  const float* xs = nullptr;  // [m][d]
  const float* xt = nullptr;  // [n][d]
  int d = 0;
  float scale = 0.f;
};

static int solve_impl(drot_handle h, const CostSource& cost, const float* p, const float* q, int m, int n,
                      float stepsize, drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters,
                      float tol, float* X_out, const float* phi0, const float* varphi0, bool warm, void* stream_v) {
  const float* C = cost.C;
  const bool from_points = cost.C == nullptr;
  if (!h || !p || !q || !X_out) return DROT_ERR_INVALID_ARG;
  if (from_points) {
    if (!cost.xs || !cost.xt || cost.d < 1 || !(cost.scale > 0.f) || warm) return DROT_ERR_INVALID_ARG;
    if (reg_kind == DROT_REG_GROUP_LASSO) return DROT_ERR_INVALID_ARG;  // stored-cost paths only
  }
  if (warm && (!phi0 || !varphi0)) return DROT_ERR_INVALID_ARG;
  if (m < 1 || n < 1 || m > h->max_m || n > h->max_n || max_iters < 0) return DROT_ERR_INVALID_ARG;
  if (reg_kind != DROT_REG_NONE && reg_kind != DROT_REG_QUADRATIC && reg_kind != DROT_REG_GROUP_LASSO)
    return DROT_ERR_INVALID_ARG;
  if (!(tol == tol) || !(stepsize == stepsize)) return DROT_ERR_INVALID_ARG;  // NaN
  float lambda = 0.f, mu = 0.f;
  int num_classes = 0;
  const int* row_class = nullptr;
  if (reg_kind != DROT_REG_NONE) {
    if (!reg_params) return DROT_ERR_INVALID_ARG;
    lambda = reg_params->lambda;
    if (!(lambda >= 0.f)) return DROT_ERR_INVALID_ARG;
    if (reg_kind == DROT_REG_GROUP_LASSO) {
      mu = reg_params->mu;
      num_classes = reg_params->num_classes;
      row_class = reg_params->row_class;
      if (!(mu >= 0.f) || num_classes < 1 || !row_class) return DROT_ERR_INVALID_ARG;
    }
  }
  // weighted l1 term <W, X>: on X >= 0 it shifts the cost, so the solve runs on a working copy C + W
  const float* weights = reg_params ? reg_params->weights : nullptr;
  if (weights && (from_points || reinterpret_cast<uintptr_t>(weights) % 4)) return DROT_ERR_INVALID_ARG;
  int cur_dev = -1;
  DROT_HIP(hipGetDevice(&cur_dev));
  if (cur_dev != h->device) return DROT_ERR_INVALID_ARG;  // the workspace lives on the creating device
  const bool resume = h->continue_next != 0 && !warm;
  if (resume && (!h->solved || m != h->last_m || n != h->last_n)) return DROT_ERR_INVALID_ARG;
  hipStream_t stream = reinterpret_cast<hipStream_t>(stream_v);
  const float rho = stepsize > 0.f ? stepsize : 2.0f / (float)(m + n);
  // 1/(1 + rho*lambda) evaluated in fp64 from the fp32 inputs, rounded once
  const float qscale = (float)(1.0 / (1.0 + (double)rho * (double)lambda));

  if (reinterpret_cast<uintptr_t>(X_out) % 4 || reinterpret_cast<uintptr_t>(C) % 4) return DROT_ERR_INVALID_ARG;
  if (from_points && (reinterpret_cast<uintptr_t>(cost.xs) % 4 || reinterpret_cast<uintptr_t>(cost.xt) % 4))
    return DROT_ERR_INVALID_ARG;
  const int nseg = ceil_div(n, kSegCols);
  const int ntr = ceil_div(m, kTileRows);
  const int ntiles = nseg * ntr;
  const bool nt = h->nontemporal < 0 ? use_nontemporal(m, n) : h->nontemporal != 0;
  // Rows that do not start on 128-byte lines are slow to stream: work on padded copies then.
  const int ld_pad = ceil_div(n, kAlignElems) * kAlignElems;
  // Tiny problems: one workgroup holds X and C in registers for a whole stretch of iterations.
  const bool resident = h->resident != 0 && reg_kind != DROT_REG_GROUP_LASSO && !from_points &&
                        m <= kResidentMaxRows && n <= kResidentCols;
  const bool pad_c = weights != nullptr ||
                     (!resident && !from_points && ((n % kAlignElems != 0) || (reinterpret_cast<uintptr_t>(C) % 128 != 0)));
  const bool pad_x = !resident && ((n % kAlignElems != 0) || (reinterpret_cast<uintptr_t>(X_out) % 128 != 0));
  auto grow = [&](float** buf, size_t* len) -> int {
    const size_t need = (size_t)m * (size_t)ld_pad;
    if (*len >= need) return DROT_OK;
    if (hipStreamSynchronize(stream) != hipSuccess) return DROT_ERR_HIP;
    (void)hipFree(*buf);
    *buf = nullptr;
    *len = 0;
    if (dev_alloc(buf, need) != DROT_OK) return DROT_ERR_ALLOC;
    *len = need;
    // the pad columns must hold finite values: they are read (and masked out) by the last lanes of a row
    hipLaunchKernelGGL(fill_kernel, dim3(1024), dim3(256), 0, stream, *buf, need, 0.f, (const int*)nullptr);
    return DROT_OK;
  };
  const int nbm = ceil_div(m, 64), nbn = ceil_div(n, 64);

  size_t ngroups = 0;
  if (reg_kind == DROT_REG_GROUP_LASSO) {
    ngroups = (size_t)num_classes * (size_t)n;
    if (h->gbuf_len < 2 * ngroups) {
      DROT_HIP(hipStreamSynchronize(stream));
      (void)hipFree(h->gbuf);
      h->gbuf = nullptr;
      h->gbuf_len = 0;
      if (dev_alloc(&h->gbuf, 2 * ngroups) != DROT_OK) return DROT_ERR_ALLOC;
      h->gbuf_len = 2 * ngroups;
    }
  }

  // Group lasso: if every class is one run of consecutive rows short enough to sit in a workgroup's
  // registers, take the group-resident kernel; otherwise the general two-pass path.
  int slab_k = 0, nruns = 0;
  if (reg_kind == DROT_REG_GROUP_LASSO) {
    std::vector<int> labels((size_t)m);
    DROT_HIP(hipMemcpyAsync(labels.data(), row_class, sizeof(int) * (size_t)m, hipMemcpyDeviceToHost, stream));
    DROT_HIP(hipStreamSynchronize(stream));
    std::vector<int> runs;  // start, len pairs
    std::vector<char> seen((size_t)num_classes, 0);
    bool one_run_per_class = true;
    int maxlen = 0;
    for (int i = 0; i < m;) {
      const int c = labels[(size_t)i];
      if (c < 0 || c >= num_classes) return DROT_ERR_INVALID_ARG;
      int e = i + 1;
      while (e < m && labels[(size_t)e] == c) ++e;
      if (seen[(size_t)c]) one_run_per_class = false;
      seen[(size_t)c] = 1;
      runs.push_back(i);
      runs.push_back(e - i);
      if (e - i > maxlen) maxlen = e - i;
      i = e;
    }
    nruns = (int)(runs.size() / 2);
    if (!h->force_two_pass && one_run_per_class && maxlen <= kSlabMaxRows && nruns <= h->max_runs) {
      slab_k = 1;
      while (kSlabRowLanes * slab_k < maxlen) slab_k *= 2;
      if (h->runbuf_len < runs.size()) {
        (void)hipFree(h->runbuf);
        h->runbuf = nullptr;
        h->runbuf_len = 0;
        if (dev_alloc(&h->runbuf, runs.size()) != DROT_OK) return DROT_ERR_ALLOC;
        h->runbuf_len = runs.size();
      }
      // de-interleave: run_start[0..nruns), run_len[0..nruns)
      std::vector<int> table(runs.size());
      for (int r = 0; r < nruns; ++r) {
        table[(size_t)r] = runs[2 * (size_t)r];
        table[(size_t)nruns + r] = runs[2 * (size_t)r + 1];
      }
      DROT_HIP(hipMemcpy(h->runbuf, table.data(), sizeof(int) * table.size(), hipMemcpyHostToDevice));
    }
  }

  VecState V{h->phi, h->varphi, h->a, h->b, h->theta, h->sum_p, h->r, h->s, h->part, h->resid, h->done, h->status};
  const long long k_base = resume ? h->iters_done : 0;
  if (resume) hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(1), 0, stream, V);
  else if (!warm) hipLaunchKernelGGL(init_kernel, dim3(1), dim3(1024), 0, stream, V, p, q, m, n);

  const float* Cw = C;      // the arrays the kernels work on
  float* Xw = X_out;
  int ldc = n, ldx = n;
  if (pad_c) {
    const int rc = grow(&h->cpad, &h->cpad_len);
    if (rc != DROT_OK) return rc;
    Cw = h->cpad;
    ldc = ld_pad;
    if (weights)
      hipLaunchKernelGGL(add_weights_kernel, dim3(ceil_div(n, 256), m < 65535 ? m : 65535), dim3(256), 0, stream,
                         h->cpad, C, weights, m, n, ld_pad);
    else
      DROT_HIP(hipMemcpy2DAsync(h->cpad, sizeof(float) * (size_t)ld_pad, C, sizeof(float) * (size_t)n,
                                sizeof(float) * (size_t)n, (size_t)m, hipMemcpyDeviceToDevice, stream));
  }
  if (pad_x) {
    const int rc = grow(&h->xpad, &h->xpad_len);
    if (rc != DROT_OK) return rc;
    Xw = h->xpad;
    ldx = ld_pad;
    if (resume || warm)  // the plan to start from is in X_out
      DROT_HIP(hipMemcpy2DAsync(h->xpad, sizeof(float) * (size_t)ld_pad, X_out, sizeof(float) * (size_t)n,
                                sizeof(float) * (size_t)n, (size_t)m, hipMemcpyDeviceToDevice, stream));
  }
  SweepArgs S{Xw, Cw, h->phi, h->varphi, h->rowpart, h->colpart, nullptr, h->done,
              m, n, ldx, ldc, rho, reg_kind == DROT_REG_NONE ? 1.0f : qscale,
              (pad_x && (pad_c || from_points)) ? ld_pad : n, nullptr};
  // on-the-fly cost: pack the point clouds for the matrix cores and take their squared norms
  PointArgs PT{};
  if (from_points) {
    const int dq = ceil_div(cost.d, 16) * 4;
    const size_t need = (size_t)(m + n) * 4 * (size_t)dq + (size_t)m + (size_t)n;
    if (h->ptbuf_len < need) {
      DROT_HIP(hipStreamSynchronize(stream));
      (void)hipFree(h->ptbuf);
      h->ptbuf = nullptr;
      h->ptbuf_len = 0;
      if (dev_alloc(&h->ptbuf, need) != DROT_OK) return DROT_ERR_ALLOC;
      h->ptbuf_len = need;
    }
    float* xs_pack = h->ptbuf;
    float* xt_pack = xs_pack + (size_t)m * 4 * dq;
    float* xs_sq = xt_pack + (size_t)n * 4 * dq;
    float* xt_sq = xs_sq + m;
    hipLaunchKernelGGL(pack_points_kernel, dim3(ceil_div(m, 256)), dim3(256), 0, stream, cost.xs, m, cost.d, dq, xs_pack, xs_sq);
    hipLaunchKernelGGL(pack_points_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, stream, cost.xt, n, cost.d, dq, xt_pack, xt_sq);
    PT = PointArgs{xs_pack, xt_pack, xs_sq, xt_sq, dq, cost.scale};
  }
  GroupArgs G{S, row_class, h->gbuf, rho * mu};
  SlabArgs SL{S, h->runbuf, h->runbuf ? h->runbuf + nruns : nullptr, rho * mu};
  const dim3 slab_grid(ceil_div(n, kSlabCols), nruns > 0 ? nruns : 1);
  // the partial sums the reduction reads: per 256-column segment and 32-row tile, or, on the
  // group-resident path, per 32-column strip and label run
  ReduceArgs RA{V, h->rowpart, h->colpart, p, q, m, n, slab_k ? ceil_div(n, kSlabCols) : nseg,
                slab_k ? nruns : ntr, nbm, nbn, 1};
  UpdateArgs UA{V, nullptr, 0, nullptr, nullptr, nullptr, nullptr, m, n, nbm, nbn, 0};
  // Small problems: the vector update of iteration s-1 is computed at the head of sweep s by every
  // workgroup for its own rows and columns (one launch per iteration instead of three); the
  // separate reduce + update kernels then run only where the state must be complete in memory:
  // before a residual check and at the end.
  // (eta comes from the tile totals whenever the problem is small enough for that path, whether or
  // not the fusion is switched on, so that both settings produce the same bits)
  const int nstrips = ceil_div(n, kSlabCols);
  const bool small_slab = slab_k && nstrips <= 64 && nruns <= 64 && nstrips * nruns <= 4096;
  const bool small = small_slab ||
                     (reg_kind != DROT_REG_GROUP_LASSO && !from_points && ntr <= 64 && ntiles <= 4096);
  const bool fused = small && h->fused_update != 0;
  // Two schemes for the none/quadratic sweeps of large problems.  Sparse plan (the usual case):
  // plain sweeps on 64-row tiles (8 waves of 8 rows) that skip the all-zero row segments of X.
  // Dense plan (strong quadratic term): the even/odd pairs.  With both options on automatic the
  // choice follows the density of the plan, which the reduction counts (nonzero row-segment sums)
  // and the host reads with the status of every stretch of check_every iterations, one stretch late.
  const dim3 update_grid(ceil_div(m + n, kReduceThreads));
  const bool can_pair = reg_kind != DROT_REG_GROUP_LASSO && !fused && !from_points;
  // (two decisions hang on the density the reduction reports: pairs or not, when that is left to the
  // library, and whether the screened sweeps may use their lean kernel)
  const bool adaptive_pairs = can_pair && !small && h->skip_cost == -1 && h->skip_unchanged != 0;
  const bool may_screen = can_pair && !small && h->skip_cost != 1 && h->skip_unchanged != 0 &&
                          (h->screening > 0 || (h->screening == -1 && (size_t)m * (size_t)n >= kScreenFrom));
  const bool adaptive = adaptive_pairs || may_screen;
  bool dense_plan = resume && h->dense_plan;  // (a continued solve keeps what the last one found)
  double plan_density = resume ? h->plan_density : -1.0;  // fraction of nonzero row segments, once a status has come back
  constexpr int kTallRows = 8, kTallWaves = 8;
  const int ntr_tall = ceil_div(m, kTallWaves * kTallRows);
  auto a_buf = [&](long long g) { return h->a + (size_t)(g & 1) * (size_t)h->max_m; };
  auto b_buf = [&](long long g) { return h->b + (size_t)(g & 1) * (size_t)h->max_n; };
  auto rowp = [&](long long g) { return h->rowpart + (size_t)(g & 1) * h->rowpart_half; };
  auto colp = [&](long long g) { return h->colpart + (size_t)(g & 1) * h->colpart_half; };
  auto tsum = [&](long long g) { return h->tilesum + (size_t)(g & 1) * h->tilesum_half; };
  const dim3 grid(nseg, ntr), block(kBlock), sweep_block(64 * kSweepWaves);

  if (warm) {
    // sums of X_0 (a sweep that only adds up), residuals, then the eq. (6) state of the starting point
    hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(1), 0, stream, V);
    S.rowpart = rowp(0);
    S.colpart = colp(0);
    hipLaunchKernelGGL((sweep_kernel<false, false, false, 3>), grid, sweep_block, 0, stream, S, FusedUpdateArgs{});
    RA.rowpart = rowp(0);
    RA.colpart = colp(0);
    RA.nseg = nseg;
    RA.ntr = ntr;
    hipLaunchKernelGGL(reduce_kernel, dim3(nbm + nbn), dim3(kReduceThreads), 0, stream, RA);
    hipLaunchKernelGGL(warm_init_kernel, dim3(1), dim3(1024), 0, stream, V, p, phi0, varphi0, m, n);
    RA.nseg = slab_k ? ceil_div(n, kSlabCols) : nseg;
    RA.ntr = slab_k ? nruns : ntr;
  }
  if (max_iters == 0 && !resume && !warm) {
    hipLaunchKernelGGL(fill_kernel, dim3(1024), dim3(256), 0, stream, X_out, (size_t)m * n, 0.f, (const int*)nullptr);
    if (pad_x)  // (the gap pass reads the working copy, which may hold an earlier solve's plan)
      hipLaunchKernelGGL(fill_kernel, dim3(1024), dim3(256), 0, stream, h->xpad, (size_t)m * ld_pad, 0.f, (const int*)nullptr);
  }

  const bool checking = tol > 0.f;
  int k = 0, slot = 0, checks = 0;
  bool converged = false;
  bool materialized = true;  // phi, varphi, a, b, theta in memory are complete for the sweeps done so far
  bool was_probe[2] = {false, false};
  bool norms_pending = false;  // the last vector update left the residual norms as per-workgroup sums
  h->prof_used = 0;
  if (h->profile)  // empty event pairs: the time a pair reports with nothing between its two records
    for (auto& e : h->cal_ev) DROT_HIP(hipEventRecord(e, stream));
  // generation whose row-segment sums (tile layout) describe the plain X in memory, if any: lets the
  // plain sweep skip reading all-zero segments
  // (a continued solve starts from the X the last one returned, so its row-segment sums still hold)
  const int sums_strip = slab_k ? kSlabCols : kSegCols;
  // (the warm start's sums are those of 256-column segments)
  long long sums_gen = warm ? (slab_k ? -1 : 0) : (resume && h->sums_valid && h->sums_strip == sums_strip) ? k_base : -1;
  long long lines_gen = (resume && h->lines_valid && sums_gen >= 0) ? k_base : -1;  // the same for the lean sweep's line masks
  h->sums_valid = h->lines_valid = false;  // (until this solve has returned)
  // screened sweeps: the sweep that last recorded the bounds M (with its varphi as varphi0), if any
  // (varphi moves fast at first: the bounds are renewed after 8 sweeps, then 16, 32, ... up to the
  // period; a continued solve carries on with the bounds and the schedule of the last one)
  const int refresh_max = h->screening >= 2 ? h->screening : 256;
  long long epoch_gen = resume ? h->epoch_gen : -1;
  int refresh_period = resume ? h->refresh_period : 8;
  if (refresh_period > refresh_max) refresh_period = refresh_max;
  while (k < max_iters && !converged) {
    int chunk = max_iters - k;
    bool probe = false;  // this stretch ends with a status for the host's choice of sweep only (no stopping test)
    if (checking || adaptive) {
      const int to_check = h->check_every - k % h->check_every;  // the tests stay at multiples of check_every
      if (to_check < chunk) chunk = to_check;
      if (adaptive && !resume && k < 512) {
        // how sparse the plan is decides the sweep, and a cold start goes through phases (empty, then
        // dense, then as sparse as it will be, or not): over the first 512 iterations have a look
        // after 16 and then every 32 iterations too.  These early readings can move the solver to the
        // lean sweep and away from it again, never to the even/odd pairs.
        const int next = k < 16 ? 16 : (k / 32 + 1) * 32;
        if (next > 0 && next - k < chunk) {
          chunk = next - k;
          probe = true;
        }
      }
    }
    const bool skip_cost = can_pair && (h->skip_cost == 1 || (adaptive_pairs && dense_plan));
    const bool tall = !small && !skip_cost && !from_points && reg_kind != DROT_REG_GROUP_LASSO && h->skip_unchanged != 0;
    if (resident) {
      const long long sw = k_base + k + 1;         // first sweep of the stretch
      const long long last = sw + chunk - 1;       // its last one: the state leaves in that generation's buffers
      const bool timed = h->profile && h->prof_used < kMaxProfiled;
      if (timed) DROT_HIP(hipEventRecord(h->prof_ev[2 * h->prof_used], stream));
      const ResidentArgs RS{Xw, Cw, p, q, V, a_buf(sw - 1), b_buf(sw - 1), a_buf(last), b_buf(last),
                            (int)((sw - 1) & 1), (int)(last & 1), m, n, ldx, ldc, rho, S.scale, chunk,
                            (sw == 1 && !warm) ? 1 : 0};
      if (n <= 64) launch_resident<1>(RS, stream);
      else if (n <= 128) launch_resident<2>(RS, stream);
      else launch_resident<4>(RS, stream);
      if (timed) {
        DROT_HIP(hipEventRecord(h->prof_ev[2 * h->prof_used + 1], stream));
        h->prof_kind[h->prof_used] = 3;
        h->prof_iters[h->prof_used] = chunk;
        ++h->prof_used;
      }
      k += chunk;
    }
    for (int c = 0; !resident && c < chunk; ++c, ++k) {
      const long long sw = k_base + k + 1;  // this sweep produces X_sw; its sums live in the sw-parity buffers
      const bool first = (sw == 1) && !warm;  // X_0 = 0: nothing to read
      const bool timed = h->profile && h->prof_used < kMaxProfiled;
      const int pe = h->prof_used;
      if (timed) {
        DROT_HIP(hipEventRecord(h->prof_ev[2 * pe], stream));
        h->prof_kind[pe] = 0;
        h->prof_iters[pe] = 1;
        ++h->prof_used;
      }
      S.rowpart = SL.S.rowpart = G.S.rowpart = rowp(sw);
      S.colpart = SL.S.colpart = G.S.colpart = colp(sw);
      S.tilesum = small ? tsum(sw) : nullptr;
      bool tiles64 = false, lean = false, refresh = false, slab_totals = false;
      if (from_points) {
        S.rowpart_prev = (sums_gen == sw - 1 && h->skip_unchanged != 0) ? rowp(sw - 1) : nullptr;
        sums_gen = sw;
        if (first) hipLaunchKernelGGL((sweep_points_kernel<true, false>), grid, sweep_block, 0, stream, S, PT);
        else if (nt) hipLaunchKernelGGL((sweep_points_kernel<false, true>), grid, sweep_block, 0, stream, S, PT);
        else hipLaunchKernelGGL((sweep_points_kernel<false, false>), grid, sweep_block, 0, stream, S, PT);
      } else if (slab_k) {
        // (large problems: the slab totals give eta, one launch then does the whole vector update)
        slab_totals = !small && (size_t)nstrips * (size_t)nruns <= h->tilesum_half;
        if (slab_totals) S.tilesum = tsum(sw);
        SL.S.tilesum = S.tilesum;
        const FusedUpdateArgs F{rowp(sw - 1), colp(sw - 1), tsum(sw - 1), p, q, a_buf(sw - 2), b_buf(sw - 2),
                                a_buf(sw - 1), b_buf(sw - 1), h->theta + ((sw - 2) & 1), h->theta + ((sw - 1) & 1),
                                h->sum_p, h->phi, h->varphi, nstrips, nruns};
        SL.S.rowpart_prev = (sums_gen == sw - 1 && h->skip_unchanged != 0) ? rowp(sw - 1) : nullptr;
        sums_gen = sw;
        launch_slab(first, !materialized, slab_k, slab_grid, stream, SL, F);
      } else if (reg_kind == DROT_REG_GROUP_LASSO) {
        hipLaunchKernelGGL(fill_kernel, dim3(ceil_div((int)((ngroups + 255) / 256), 4)), dim3(256), 0, stream,
                           h->gbuf, ngroups, 0.f, (const int*)h->done);
        if (first) {
          hipLaunchKernelGGL(gl_norm_kernel<true>, grid, block, 0, stream, G);
          hipLaunchKernelGGL(gl_apply_kernel<true>, grid, block, 0, stream, G);
        } else {
          hipLaunchKernelGGL(gl_norm_kernel<false>, grid, block, 0, stream, G);
          hipLaunchKernelGGL(gl_apply_kernel<false>, grid, block, 0, stream, G);
        }
      } else if (!materialized) {
        // update sw-1 (from the sums of X_{sw-1} and the state of generation sw-2) rides along
        const FusedUpdateArgs F{rowp(sw - 1), colp(sw - 1), tsum(sw - 1), p, q, a_buf(sw - 2), b_buf(sw - 2),
                                a_buf(sw - 1), b_buf(sw - 1), h->theta + ((sw - 2) & 1), h->theta + ((sw - 1) & 1),
                                h->sum_p, h->phi, h->varphi, nseg, ntr};
        S.rowpart_prev = nullptr;
        if (nt) hipLaunchKernelGGL((sweep_kernel<false, true, true>), grid, sweep_block, 0, stream, S, F);
        else hipLaunchKernelGGL((sweep_kernel<false, false, true>), grid, sweep_block, 0, stream, S, F);
        sums_gen = sw;
      } else {
        // even/odd scheme: inside a chunk the sweeps pair up as (store X - rho*C, then read it
        // without C); an odd chunk starts with one plain sweep, so X is plain at every chunk end
        int mode = 0;
        if (skip_cost) {
          const int paired_from = chunk & 1;  // index in the chunk of the first paired sweep
          if (c >= paired_from) mode = ((c - paired_from) & 1) ? 2 : 1;
        }
        const bool screened = mode == 0 && tall && !first && may_screen;
        S.rowpart_prev = (mode == 0 && sums_gen == sw - 1 && h->skip_unchanged != 0) ? rowp(sw - 1) : nullptr;
        sums_gen = mode == 1 ? -1 : sw;
        // once the plan is known to be sparse (and bounds exist): one wave per tile, walking through the few
        // rows left; that sweep renews the bounds by itself, on a schedule kept on the device
        lean = screened && epoch_gen >= 0 && S.rowpart_prev != nullptr && plan_density >= 0.0 && plan_density < 0.25;
        refresh = screened && !lean && (epoch_gen < 0 || sw - epoch_gen >= refresh_period);
        if (timed) h->prof_kind[pe] = screened ? (refresh ? 6 : 5) : (mode == 0 && tall && !first) ? 4 : mode;
        const FusedUpdateArgs none{};
        // the sweeps on 64-row tiles also store the totals of their tiles: one launch then does both
        // halves of the vector update
        tiles64 = tall && !first && mode == 0;
        if (tiles64) S.tilesum = tsum(sw);
        if (screened) {
          const dim3 sgrid(nseg, ceil_div(m, kScreenRows * kScreenWaves)), sblock(64 * kScreenWaves);
          if (refresh) {  // (the sweep itself stores varphi as the epoch's varphi0)
            if (epoch_gen >= 0) refresh_period = refresh_period * 2 < refresh_max ? refresh_period * 2 : refresh_max;
            epoch_gen = sw;
          }
          const ScreenArgs SC{h->mprime, h->mprime, h->varphi0, timed ? h->wave_reads : nullptr,
                              h->varphi0, h->screen_ctl, h->wg_reads,
                              (lean && lines_gen == sw - 1) ? h->xlines : nullptr, h->xlines};
          if (lean) {
            lines_gen = sw;
            const int ntr64 = ceil_div(m, 64);
            const dim3 lgrid(nseg, ceil_div(ntr64, kLeanWaves)), lblock(64 * kLeanWaves);
            if (nt) hipLaunchKernelGGL((screened_lean_kernel<true>), lgrid, lblock, 0, stream, S, SC, ntr64);
            else hipLaunchKernelGGL((screened_lean_kernel<false>), lgrid, lblock, 0, stream, S, SC, ntr64);
            if (timed) h->prof_kind[pe] = 7;
          } else if (refresh) {
            if (nt) hipLaunchKernelGGL((screened_sweep_kernel<true, true>), sgrid, sblock, 0, stream, S, SC);
            else hipLaunchKernelGGL((screened_sweep_kernel<false, true>), sgrid, sblock, 0, stream, S, SC);
          } else {
            if (nt) hipLaunchKernelGGL((screened_sweep_kernel<true, false>), sgrid, sblock, 0, stream, S, SC);
            else hipLaunchKernelGGL((screened_sweep_kernel<false, false>), sgrid, sblock, 0, stream, S, SC);
          }
        } else if (first) {
          if (mode == 1) hipLaunchKernelGGL((sweep_kernel<true, false, false, 1>), grid, sweep_block, 0, stream, S, none);
          else hipLaunchKernelGGL((sweep_kernel<true, false, false, 0>), grid, sweep_block, 0, stream, S, none);
        } else if (nt) {
          if (mode == 1) hipLaunchKernelGGL((sweep_kernel<false, true, false, 1>), grid, sweep_block, 0, stream, S, none);
          else if (mode == 2) hipLaunchKernelGGL((sweep_kernel<false, true, false, 2>), grid, sweep_block, 0, stream, S, none);
          else if (tall) hipLaunchKernelGGL((sweep_kernel<false, true, false, 0, kTallRows, kTallWaves>), dim3(nseg, ntr_tall), dim3(64 * kTallWaves), 0, stream, S, none);
          else hipLaunchKernelGGL((sweep_kernel<false, true, false, 0>), grid, sweep_block, 0, stream, S, none);
        } else {
          if (mode == 1) hipLaunchKernelGGL((sweep_kernel<false, false, false, 1>), grid, sweep_block, 0, stream, S, none);
          else if (mode == 2) hipLaunchKernelGGL((sweep_kernel<false, false, false, 2>), grid, sweep_block, 0, stream, S, none);
          else if (tall) hipLaunchKernelGGL((sweep_kernel<false, false, false, 0, kTallRows, kTallWaves>), dim3(nseg, ntr_tall), dim3(64 * kTallWaves), 0, stream, S, none);
          else hipLaunchKernelGGL((sweep_kernel<false, false, false, 0>), grid, sweep_block, 0, stream, S, none);
        }
        // (the 64-row tiles leave fewer rows of column partials for the reduction, which adds them up in
        // groups of four; the lean sweep stores one row per group)
        if (!slab_k) {
          RA.ntr = lean ? ceil_div(ntr_tall, kColGroup) : tiles64 ? ntr_tall : ntr;
          RA.cgroup = (tiles64 && !lean) ? kColGroup : 1;
        }
      }
      if (timed) {
        DROT_HIP(hipEventRecord(h->prof_ev[2 * pe + 1], stream));
        if (h->prof_kind[pe] >= 5)  // (one count per wave of the 8-wave tiles, one per workgroup of the lean kernel)
          hipLaunchKernelGGL(sum_reads_kernel, dim3(1), dim3(1024), 0, stream,
                             (const int*)(h->prof_kind[pe] == 7 ? h->wg_reads : h->wave_reads),
                             h->prof_kind[pe] == 7 ? nseg * ceil_div(ceil_div(m, 64), kLeanWaves)
                                                   : nseg * ceil_div(m, 64) * kScreenWaves,
                             h->prof_reads + pe);
      }
      if (!fused || c == chunk - 1) {
        // complete the state in memory: update sw from the sums of X_sw
        RA.rowpart = rowp(sw);
        RA.colpart = colp(sw);
        UA.a_in = a_buf(sw - 1);
        UA.b_in = b_buf(sw - 1);
        UA.a_out = a_buf(sw);
        UA.b_out = b_buf(sw);
        UA.par = (int)((sw - 1) & 1);
        UA.tilesum = small ? tsum(sw) : nullptr;
        UA.ntiles = small_slab ? nstrips * nruns : ntiles;
        if (slab_totals) {
          const TileTotals TT{tsum(sw), nruns, nstrips, 1};
          const ScreenCtlArgs KA{nullptr, nullptr, 0, 0, 0, 0};
          hipLaunchKernelGGL(reduce_update_kernel, dim3(nbm + nbn), dim3(64 * kMergedWaves), 0, stream, RA, UA, TT, KA);
        } else if (tiles64) {
          const TileTotals TT{tsum(sw), lean ? ceil_div(ntr_tall, kColGroup) : ntr_tall, nseg, lean ? 1 : kColGroup};
          // (the price of a renewal: all row segments of C, read by a sweep that streams them better than
          // the scattered reads it saves)
          const double price = 0.75 * (double)m * (double)nseg;
          const ScreenCtlArgs KA{h->screen_ctl, h->wg_reads, nseg * ceil_div(ntr_tall, kLeanWaves),
                                 lean ? 2 : refresh ? 1 : 0, price < 1.0e9 ? (int)price : 1000000000,
                                 h->screening >= 2 ? h->screening : 1024};
          hipLaunchKernelGGL(reduce_update_kernel, dim3(nbm + nbn), dim3(64 * kMergedWaves), 0, stream, RA, UA, TT, KA);
        } else {
          hipLaunchKernelGGL(reduce_kernel, dim3(nbm + nbn), dim3(kReduceThreads), 0, stream, RA);
          hipLaunchKernelGGL(update_kernel, update_grid, dim3(kReduceThreads), 0, stream, UA);
        }
        norms_pending = true;
        materialized = true;
      } else {
        materialized = false;
      }
    }
    if (checking || adaptive) {
      // the test runs on the device; the host reads it one chunk late so the queue never drains
      if (norms_pending) hipLaunchKernelGGL(residual_norms_kernel, dim3(1), dim3(kReduceThreads), 0, stream, V, nbm, nbn);
      norms_pending = false;
      hipLaunchKernelGGL(status_kernel, dim3(1), dim3(1), 0, stream, V, k, (checking && !probe) ? (double)tol : 0.0);
      DROT_HIP(hipMemcpyAsync(&h->host_status[slot], h->status, sizeof(DeviceStatus), hipMemcpyDeviceToHost, stream));
      DROT_HIP(hipEventRecord(h->ev[slot], stream));
      was_probe[slot] = probe;
      if (checks > 0) {
        DROT_HIP(hipEventSynchronize(h->ev[slot ^ 1]));
        if (h->host_status[slot ^ 1].converged) converged = true;
        if (adaptive) {  // (hysteresis: the break-even is at about three quarters of the segments nonzero)
          const double density = h->host_status[slot ^ 1].nz_segments / ((double)m * (double)nseg);
          plan_density = density;
          if (density > 0.7 && !was_probe[slot ^ 1]) dense_plan = adaptive_pairs;
          else if (density < 0.5) dense_plan = false;
        }
      }
      slot ^= 1;
      ++checks;
    }
  }
  // final state: residuals of the returned iterate (no-op if the stop flag is already up)
  if (k > 0) {
    if (norms_pending) hipLaunchKernelGGL(residual_norms_kernel, dim3(1), dim3(kReduceThreads), 0, stream, V, nbm, nbn);
    hipLaunchKernelGGL(status_kernel, dim3(1), dim3(1), 0, stream, V, k, checking ? (double)tol : 0.0);
  }
  if (h->compute_gap) {
    float* gx = h->gbuf;
    float* gw = h->gbuf ? h->gbuf + ngroups : nullptr;
    if (reg_kind == DROT_REG_GROUP_LASSO)
      hipLaunchKernelGGL(fill_kernel, dim3(ceil_div((int)((2 * ngroups + 255) / 256), 4)), dim3(256), 0, stream,
                         h->gbuf, 2 * ngroups, 0.f, (const int*)nullptr);
    GapArgs GA{Xw, Cw, h->phi, h->varphi, row_class, h->gap_part, gx, gw, m, n, nseg, ldx, ldc, rho, PT};
    hipLaunchKernelGGL(gap_kernel, grid, block, 0, stream, GA);
    hipLaunchKernelGGL(gap_final_kernel, dim3(1), dim3(1024), 0, stream, V, (const float*)h->gap_part, ntiles,
                       (const float*)gx, (const float*)gw, ngroups, p, q, m, n, (double)rho, (int)reg_kind,
                       (double)lambda, (double)mu);
  }
  if (pad_x && !(max_iters == 0 && !resume && !warm))
    DROT_HIP(hipMemcpy2DAsync(X_out, sizeof(float) * (size_t)n, h->xpad, sizeof(float) * (size_t)ld_pad,
                              sizeof(float) * (size_t)n, (size_t)m, hipMemcpyDeviceToDevice, stream));
  DROT_HIP(hipMemcpyAsync(&h->host_status[0], h->status, sizeof(DeviceStatus), hipMemcpyDeviceToHost, stream));
  DROT_HIP(hipStreamSynchronize(stream));
  DROT_HIP(hipGetLastError());

  const DeviceStatus& st = h->host_status[0];
  h->prof_count = 0;
  h->prof_sweep_ms = 0.0;
  if (h->profile) {
    const int timed = h->prof_used;
    if (timed > 0) DROT_HIP(hipMemcpy(h->prof_reads_host, h->prof_reads, sizeof(double) * (size_t)timed, hipMemcpyDeviceToHost));
    // What an event pair reports for an empty interval (the smallest of four) is taken off every
    // measurement: for kernels of tens of microseconds it is a third of the reading.
    float overhead = 1e30f;
    for (int c = 0; c < 4; ++c) {
      float ms = 0.f;
      DROT_HIP(hipEventElapsedTime(&ms, h->cal_ev[2 * c], h->cal_ev[2 * c + 1]));
      if (ms < overhead) overhead = ms;
    }
    h->prof_overhead_ms = (double)overhead;
    for (int e = 0; e < timed; ++e) {
      float ms = 0.f;
      DROT_HIP(hipEventElapsedTime(&ms, h->prof_ev[2 * e], h->prof_ev[2 * e + 1]));
      ms = ms > overhead ? ms - overhead : 0.f;
      ms /= (float)h->prof_iters[e];  // per iteration (a resident stretch is one launch)
      h->prof_sweep_ms += (double)ms;
      h->prof_ms[e] = ms;
    }
    h->prof_count = timed;
  }
  h->iters_done = k_base + (max_iters == 0 ? 0 : st.iters);
  h->info.iters = max_iters == 0 ? 0 : st.iters;
  h->info.converged = st.converged;
  // with zero iterations X = 0 and no sums were formed: report the residuals as not evaluated
  h->info.r_row = max_iters == 0 ? INFINITY : (float)std::sqrt(st.r2);
  h->info.r_col = max_iters == 0 ? INFINITY : (float)std::sqrt(st.s2);
  h->info.objective = h->compute_gap ? st.cost + st.h : 0.0;
  h->info.gap = h->compute_gap ? st.gap : 0.0;
  h->info.dual_res = h->compute_gap ? st.dual_res : 0.0;
  h->dense_plan = dense_plan;
  h->plan_density = plan_density;
  // After an early stop the sweeps queued past it did nothing, a refresh among them included: the
  // host's record of the last refresh may then name a sweep that never ran.  The bounds in memory
  // still belong to their varphi0 (the refresh sweep stores both), but the schedule starts afresh.
  const bool epoch_ran = epoch_gen <= k_base + (long long)st.iters;
  h->epoch_gen = (st.converged || !epoch_ran) ? -1 : epoch_gen;
  h->refresh_period = (st.converged || !epoch_ran) ? 8 : refresh_period;
  // (after an early stop the sweeps launched past it did nothing: be conservative)
  h->sums_valid = !st.converged && max_iters > 0 && sums_gen == k_base + k;
  h->lines_valid = h->sums_valid && lines_gen == k_base + k;
  h->sums_strip = sums_strip;
  h->solved = true;
  h->last_m = m;
  h->last_n = n;
  if (checking && !st.converged) return DROT_MAX_ITERS;
  return DROT_OK;
}

int drot_solve(drot_handle h, const float* C, const float* p, const float* q, int m, int n, float stepsize,
               drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters, float tol,
               float* X_out, void* stream) {
  if (!C) return DROT_ERR_INVALID_ARG;
  CostSource cost;
  cost.C = C;
  return solve_impl(h, cost, p, q, m, n, stepsize, reg_kind, reg_params, max_iters, tol, X_out, nullptr, nullptr, false,
                    stream);
}

int drot_solve_points(drot_handle h, const float* xs, const float* xt, int d, float cost_scale, const float* p,
                      const float* q, int m, int n, float stepsize, drot_reg_kind reg_kind,
                      const drot_reg_params* reg_params, int max_iters, float tol, float* X_out, void* stream) {
  if (!xs || !xt) return DROT_ERR_INVALID_ARG;
  CostSource cost;
  cost.xs = xs;
  cost.xt = xt;
  cost.d = d;
  cost.scale = cost_scale;
  return solve_impl(h, cost, p, q, m, n, stepsize, reg_kind, reg_params, max_iters, tol, X_out, nullptr, nullptr, false,
                    stream);
}

int drot_solve_warm(drot_handle h, const float* C, const float* p, const float* q, int m, int n, float stepsize,
                    drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters, float tol,
                    float* X_inout, const float* phi0, const float* varphi0, void* stream) {
  if (!C) return DROT_ERR_INVALID_ARG;
  CostSource cost;
  cost.C = C;
  return solve_impl(h, cost, p, q, m, n, stepsize, reg_kind, reg_params, max_iters, tol, X_inout, phi0, varphi0, true,
                    stream);
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
