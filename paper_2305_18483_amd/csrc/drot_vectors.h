// Start state, reduction of the partial sums and the eq. (6) update of the dual vectors.
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

// ------------------------------------------------------------------------------------------
// S0: starting point of the Initialization paragraph: X_0 = 0 (never materialised: the first
// sweep does not read X), phi_0, varphi_0 constants, and a_0 = Y_0 1 - p, b_0 = Y_0^T 1 - q,
// theta_0 = 1^T a_0/(m+n) with Y_0 = phi_0 1^T + 1 varphi_0^T, the values that make eq. (6)
// reproduce eq. (4).  One workgroup.
// ------------------------------------------------------------------------------------------
struct VecState {
  float* phi;
  float* varphi;
  double* a;
  double* b;
  double* theta;   // [2], indexed by iteration parity
  double* sum_p;   // [1] sum of p
  double* r;       // [m] row residuals X 1 - p of the last sweep
  double* s;       // [n] column residuals
  double* part;    // [3][nbm + nbn]: per-workgroup sum of residuals, sum of squared residuals, nonzero row partials
  double* resid;   // [3]: ||r||^2, ||s||^2, number of nonzero row partial sums
  int* done;
  DeviceStatus* status;
};

__global__ __launch_bounds__(1024) void init_kernel(VecState V, const float* __restrict__ p,
                                                    const float* __restrict__ q, int m, int n) {
  __shared__ double red[1024];
  const int t = threadIdx.x;
  const double mn = (double)m + (double)n;
  const double phi0 = (1.0 + (double)m / mn) / (3.0 * mn);
  const double varphi0 = (1.0 + (double)n / mn) / (3.0 * mn);
  double sp = 0.0;
  for (int i = t; i < m; i += blockDim.x) {
    const double pi = (double)p[i];
    sp += pi;
    V.phi[i] = (float)phi0;
    V.a[i] = (double)n * (phi0 + varphi0) - pi;
  }
  for (int j = t; j < n; j += blockDim.x) {
    V.varphi[j] = (float)varphi0;
    V.b[j] = (double)m * (phi0 + varphi0) - (double)q[j];
  }
  const double sum_p = block_sum_f64(sp, red);
  if (t == 0) {
    *V.sum_p = sum_p;
    V.theta[0] = ((double)m * (double)n * (phi0 + varphi0) - sum_p) / mn;
    V.theta[1] = 0.0;
    *V.done = 0;
    *V.status = DeviceStatus{};
  }
}

// varphi and the screening epoch's copy of it hold the mask value from column n to the end of the last
// 256-column segment (the sweeps load them without an edge case).  One workgroup.
__global__ __launch_bounds__(256) void mask_tail_kernel(float* __restrict__ varphi, float* __restrict__ varphi0, int n) {
  const int j = n + (int)threadIdx.x;
  if (j < (n + kSegCols - 1) / kSegCols * kSegCols) {
    varphi[j] = kMaskedOut;
    varphi0[j] = kMaskedOut;
  }
}

// Re-arms the stop flag and the status block when a solve continues from the handle's state.
__global__ void reset_kernel(VecState V) {
  *V.done = 0;
  *V.status = DeviceStatus{};
}

// Warm start: state of eq. (6) for a caller-supplied starting point (X_0, phi_0, varphi_0), i.e.
// Y_0 = X_0 + phi_0 1^T + 1 varphi_0^T (eq. (5)): a_0 = Y_0 1 - p = (X_0 1 - p) + n phi_0 + (1^T varphi_0) 1,
// b_0 = (X_0^T 1 - q) + m varphi_0 + (1^T phi_0) 1, theta_0 = 1^T a_0 / (m+n).  The residuals
// X_0 1 - p and X_0^T 1 - q come from reduce_kernel (V.r, V.s).  One workgroup.
__global__ __launch_bounds__(1024) void warm_init_kernel(VecState V, const float* __restrict__ p,
                                                         const float* __restrict__ phi0,
                                                         const float* __restrict__ varphi0, int m, int n) {
  __shared__ double red[1024];
  const int t = threadIdx.x;
  double sp = 0.0, sphi = 0.0, svarphi = 0.0;
  for (int i = t; i < m; i += blockDim.x) { sp += (double)p[i]; sphi += (double)phi0[i]; }
  for (int j = t; j < n; j += blockDim.x) svarphi += (double)varphi0[j];
  sp = block_sum_f64(sp, red);
  sphi = block_sum_f64(sphi, red);
  svarphi = block_sum_f64(svarphi, red);
  double sa = 0.0;
  for (int i = t; i < m; i += blockDim.x) {
    const double f = (double)phi0[i];
    const double ai = V.r[i] + (double)n * f + svarphi;
    V.a[i] = ai;
    V.phi[i] = phi0[i];
    sa += ai;
  }
  for (int j = t; j < n; j += blockDim.x) {
    const double f = (double)varphi0[j];
    V.b[j] = V.s[j] + (double)m * f + sphi;
    V.varphi[j] = varphi0[j];
  }
  sa = block_sum_f64(sa, red);
  if (t == 0) {
    *V.sum_p = sp;
    V.theta[0] = sa / ((double)m + (double)n);
    V.theta[1] = 0.0;
  }
}

// ------------------------------------------------------------------------------------------
// S5, first half: r = X1 - p and s = X^T1 - q from the partial sums, in fp64.  A workgroup owns
// 64 rows or 64 columns; its 16 waves split the partials.  Leaves per workgroup the sum and the
// sum of squares of its residuals (for eta and for the stopping test, S6).
// ------------------------------------------------------------------------------------------
struct ReduceArgs {
  VecState V;
  const float* rowpart;
  const float* colpart;
  const float* p;
  const float* q;
  int m, n, nseg, ntr, nbm, nbn;
  int mp, np;  // pitches of the rows of rowpart and of colpart
  int cgroup;  // 1, kColGroup or kPointsColGroup: consecutive rows of colpart are first added up in fp32, in groups of that many
};

constexpr int kReduceThreads = 1024;

// One of the 16 shares of a column's partial sums when G consecutive rows are added in fp32 first.  share, nparts
// and ntr are wave-uniform; idx is the lane's entry, already clamped to the last one that exists.
template <int G>
__device__ __forceinline__ double gather_grouped(const float* __restrict__ part, int share, int nparts, int ntr, int idx, int pitch) {
  constexpr int kStride = 16, kGroups = 32 / G > 1 ? 32 / G / 2 : 1;  // (16 loads in flight per batch)
  double acc = 0.0;
  for (int k0 = share; k0 < nparts; k0 += kStride * kGroups) {
    float v[kGroups][G];
#pragma unroll
    for (int b = 0; b < kGroups; ++b)
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int k = (k0 + b * kStride) * G + g;  // (a row past the end: the last row is fetched and not used)
        const float w = (part + (size_t)min(k, ntr - 1) * pitch)[idx];
        v[b][g] = k < ntr ? w : 0.f;
      }
#pragma unroll
    for (int b = 0; b < kGroups; ++b)
      if (k0 + b * kStride < nparts) {
        float t = v[b][0];
#pragma unroll
        for (int g = 1; g < G; ++g) t += v[b][g];
        acc += (double)t;
      }
  }
  return acc;
}

// First part: the partial sums of 64 entries split 16 ways (share c takes the partials c, c + 16,
// ...), each share added up in order.  NW waves: wave w forms the shares w, w + NW, ... of entry
// idx and leaves them in red[share][lane]; nz_out counts the nonzero partials this wave saw.
// Which partial a load fetches depends on the wave and the workgroup only, so the row of the
// partials is a scalar base address and the lane adds its entry: no per-lane address arithmetic.
// Lanes past the last entry read the last entry (their results are never stored, their nonzero
// counts masked out).
template <int NW>
__device__ __forceinline__ void reduce_gather(const ReduceArgs& A, double* red, int& nz_out) {
  static_assert(16 % NW == 0, "the 16 shares are dealt out to the waves");
  const int t = threadIdx.x;
  const int sub = __builtin_amdgcn_readfirstlane(t >> 6), l = t & 63;
  const bool rows = (int)blockIdx.x < A.nbm;
  const int idx = (rows ? (int)blockIdx.x : (int)blockIdx.x - A.nbm) * 64 + l;
  const int len = rows ? A.m : A.n, pitch = rows ? A.mp : A.np;
  const int idc = min(idx, len - 1);
  const unsigned long long live = __builtin_amdgcn_ballot_w64(idx < len);
  const bool grouped = !rows && A.cgroup > 1;
  const int nparts = rows ? A.nseg : grouped ? (A.ntr + A.cgroup - 1) / A.cgroup : A.ntr;
  const float* __restrict__ part = rows ? A.rowpart : A.colpart;
  int nz = 0;
  constexpr int kStride = 16, kBatch = 8;
#pragma unroll
  for (int si = 0; si < 16 / NW; ++si) {
    const int share = sub + si * NW;
    double acc = 0.0;
    // column sums stored per tile row: the rows G k .. G k + G - 1 are added first, in fp32 and in order, as the
    // workgroups of the lean sweeps do before they store (a row past the end adds +0).  G = 4: four 64-row tiles
    // (screened_lean_kernel); G = 8: the eight 32-row tiles of a 256-row strip (lean_points_kernel)
    if (grouped && A.cgroup == kColGroup) acc = gather_grouped<kColGroup>(part, share, nparts, A.ntr, idc, pitch);
    else if (grouped) acc = gather_grouped<kPointsColGroup>(part, share, nparts, A.ntr, idc, pitch);
    for (int k0 = share; !grouped && k0 < nparts; k0 += kStride * kBatch) {  // (nparts and share are wave-uniform)
      // a batch of independent loads, then the additions in the order k0, k0 + 16, ... (one load per
      // trip would wait for memory once per partial sum)
      float v[kBatch];
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        const int k = k0 + b * kStride;  // (past the end: the last partial is fetched and not used; no branch, so that
        const float w = (part + (size_t)min(k, nparts - 1) * pitch)[idc];  // the loads of all shares leave together)
        v[b] = k < nparts ? w : 0.f;
      }
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        if (k0 + b * kStride < nparts) acc += (double)v[b];
        nz += __builtin_popcountll(__builtin_amdgcn_ballot_w64(v[b] != 0.f) & live);
      }
    }
    red[share * 64 + l] = acc;
  }
  nz_out = nz;
}

// Second part, after the one barrier that follows the first: wave 0 adds the 16 shares of its 64
// entries (a fixed tree, the one sum_partials_16 ends with), forms the residuals and leaves the
// workgroup's sum, sum of squares and count.  Returns the residual of entry idx in threads
// 0 .. 63 (0 elsewhere).  pq: p_idx or q_idx, fetched by the caller along with the partial sums
// (reduce_entry_pq) so that no second trip to memory follows the barrier.
__device__ __forceinline__ float reduce_entry_pq(const ReduceArgs& A) {
  const int t = threadIdx.x;
  const bool rows = (int)blockIdx.x < A.nbm;
  const int idx = (rows ? (int)blockIdx.x : (int)blockIdx.x - A.nbm) * 64 + t;
  return (t < 64 && idx < (rows ? A.m : A.n)) ? (rows ? A.p[idx] : A.q[idx]) : 0.f;
}

template <int NW>
__device__ __forceinline__ double reduce_finish(const ReduceArgs& A, const double* red, const int* nzw, float pq) {
  const int t = threadIdx.x;
  if (t >= 64) return 0.0;
  const bool rows = (int)blockIdx.x < A.nbm;
  const int idx = (rows ? (int)blockIdx.x : (int)blockIdx.x - A.nbm) * 64 + t;
  const int len = rows ? A.m : A.n;
  double w[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) w[k] = red[k * 64 + t];
  const double total = (((w[0] + w[8]) + (w[4] + w[12])) + ((w[2] + w[10]) + (w[6] + w[14]))) +
                       (((w[1] + w[9]) + (w[5] + w[13])) + ((w[3] + w[11]) + (w[7] + w[15])));
  double res = 0.0;
  if (idx < len) {
    res = total - (double)pq;
    (rows ? A.V.r : A.V.s)[idx] = res;
  }
  const double sum = wave_sum_f64(res), sumsq = wave_sum_f64(res * res);
  if (t == 0) {
    A.V.part[blockIdx.x] = sum;
    A.V.part[A.nbm + A.nbn + blockIdx.x] = sumsq;
    int cnt = 0;
    for (int k = 0; k < NW; ++k) cnt += nzw[k];
    A.V.part[2 * (A.nbm + A.nbn) + blockIdx.x] = (double)cnt;
  }
  return res;
}

__global__ __launch_bounds__(kReduceThreads) void reduce_kernel(ReduceArgs A) {
  if (*A.V.done) return;
  constexpr int NW = kReduceThreads / 64;
  __shared__ double red[16 * 64];
  __shared__ int nzw[NW];
  int nz;
  const float pq = reduce_entry_pq(A);
  reduce_gather<NW>(A, red, nz);
  if ((threadIdx.x & 63) == 0) nzw[threadIdx.x >> 6] = nz;
  __syncthreads();
  reduce_finish<NW>(A, red, nzw, pq);
}

// ------------------------------------------------------------------------------------------
// S5, second half: eq. (6) with f = 1_m, e = 1_n.  eta = 1^T r/(m+n); phi+ = (a - 2r + (2 eta -
// theta))/n, varphi+ = (b - 2s + (2 eta - theta))/m, a -= r, b -= s, theta -= eta.  fp64; phi and
// varphi are rounded to fp32 for the sweep.  Every workgroup re-derives eta from the per-workgroup
// sums (a few hundred doubles); workgroup 0 also stores theta+.  The squared residual norms are
// summed over the workgroups only where somebody reads them (residual_norms_kernel).
// ------------------------------------------------------------------------------------------
struct UpdateArgs {
  VecState V;
  const float* tilesum;  // non-null: eta from the tile totals, exactly as the fused update computes it
  int ntiles;
  const double* a_in;  // a, b before the update and after it (the two halves of a double buffer)
  const double* b_in;
  double* a_out;
  double* b_out;
  int m, n, nbm, nbn, par;
};

// ||r||^2, ||s||^2 and the number of nonzero row-segment sums from the per-workgroup sums of the reduction.
__device__ __forceinline__ void sum_residual_norms(const VecState& V, int nbm, int nbn, double* red) {
  const int t = threadIdx.x;
  double r2 = 0.0, s2 = 0.0;
  const double* sq = V.part + nbm + nbn;
  for (int e = t; e < nbm; e += kReduceThreads) r2 += sq[e];
  for (int e = t; e < nbn; e += kReduceThreads) s2 += sq[nbm + e];
  double nzs = 0.0;
  const double* cnt = V.part + 2 * (nbm + nbn);
  for (int e = t; e < nbm; e += kReduceThreads) nzs += cnt[e];
  r2 = block_sum_f64(r2, red);
  s2 = block_sum_f64(s2, red);
  nzs = block_sum_f64(nzs, red);
  if (t == 0) {
    V.resid[0] = r2;
    V.resid[1] = s2;
    V.resid[2] = nzs;
  }
}

// The update of the 1024 entries of workgroup vb (rows first, then columns), one per thread.
__device__ __forceinline__ void update_body(const UpdateArgs& A, int vb, double* red) {
  const int t = threadIdx.x;
  double acc = 0.0;
  if (A.tilesum) {
    for (int e = t; e < A.ntiles; e += kReduceThreads) acc += (double)A.tilesum[e];
  } else {
    for (int e = t; e < A.nbm; e += kReduceThreads) acc += A.V.part[e];
  }
  double sum_r = block_sum_f64(acc, red);
  if (A.tilesum) sum_r -= *A.V.sum_p;
  const double mn = (double)A.m + (double)A.n;
  const double eta = sum_r / mn;
  const double theta = A.V.theta[A.par];
  const double cst = 2.0 * eta - theta;
  const long long g = (long long)vb * kReduceThreads + t;
  if (g < A.m) {
    const double r = A.V.r[g], ai = A.a_in[g];
    A.V.phi[g] = (float)((ai - 2.0 * r + cst) / (double)A.n);
    A.a_out[g] = ai - r;
  } else if (g < (long long)A.m + A.n) {
    const long long j = g - A.m;
    const double sj = A.V.s[j], bj = A.b_in[j];
    A.V.varphi[j] = (float)((bj - 2.0 * sj + cst) / (double)A.m);
    A.b_out[j] = bj - sj;
  }
  if (vb == 0 && t == 0) A.V.theta[A.par ^ 1] = theta - eta;
}

__global__ __launch_bounds__(kReduceThreads) void update_kernel(UpdateArgs A) {
  if (*A.V.done) return;
  __shared__ double red[kReduceThreads];
  update_body(A, (int)blockIdx.x, red);
}

// What the stopping test and the host's choice of scheme read, after a reduce_update_kernel (which
// leaves the per-workgroup sums only).  One workgroup; launched before a status_kernel.
__global__ __launch_bounds__(kReduceThreads) void residual_norms_kernel(VecState V, int nbm, int nbn) {
  if (*V.done) return;
  __shared__ double red[kReduceThreads];
  sum_residual_norms(V, nbm, nbn, red);
}

// Both halves of S5 in one launch, for the sweeps on 64-row tiles of large problems.  What stands
// between the two halves is one number, eta = (1^T X 1 - 1^T p)/(m+n); with the totals of the tiles
// at hand (the sweep stores them) every workgroup forms it by itself, then reduces its 64 rows or
// columns and updates them on the spot.  Tile totals: rows in groups of 8 in order, the 8 groups
// in order (fp32), then four tiles stacked along the rows in order (in the lean sweep's workgroups,
// or here: tgroup), then all of it in fp64 in a fixed order.
struct TileTotals {
  const float* tilesum;  // [tile_rows][nseg], or one entry per kColGroup tile rows (tgroup = 1)
  int tile_rows;         // rows of tilesum
  int nseg;
  int tgroup;            // kColGroup, kPointsColGroup: add tile rows G k .. G k + G - 1 first; 1: stored that way
};

// The lean sweep's refresh schedule rides along (last workgroup): the control words kCtlRenew ... of the screened sweeps.
struct ScreenCtlArgs {
  int* ctl;              // the control words
  const int* wg_reads;   // [nwg] what the lean sweep's workgroups read
  int nwg;
  int mode;              // 0: nothing; 1: the sweep was a refresh ordered by the host: start afresh; 2: account for a lean sweep
  int price;             // rent that buys a renewal, in row segments of C
  int max_since;         // renew after this many lean sweeps at the latest
};

// A share of the tile totals when G consecutive tile rows are added in fp32 first, in order (the sweeps that
// store one total per group of G tiles add them up that way before they store): entries e0, e0 + 1024, ...
template <int G>
__device__ __forceinline__ double grouped_tile_totals(const TileTotals& T, int e0_lane, int ln) {
  constexpr int kShares = 1024, kGroups = 16 / G;  // (16 loads in flight per batch)
  const int ngroups = ((T.tile_rows + G - 1) / G) * T.nseg;
  double acc = 0.0;
  for (int e0 = e0_lane; e0 - ln < ngroups; e0 += kShares * kGroups) {
    float v[kGroups][G];
#pragma unroll
    for (int b = 0; b < kGroups; ++b) {
      const int e = e0 + b * kShares;
      const int k = e / T.nseg, sg = e - k * T.nseg;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int tr = k * G + g;
        v[b][g] = (e < ngroups && tr < T.tile_rows) ? T.tilesum[tr * T.nseg + sg] : 0.f;
      }
    }
#pragma unroll
    for (int b = 0; b < kGroups; ++b) {
      float t = v[b][0];
#pragma unroll
      for (int g = 1; g < G; ++g) t += v[b][g];
      acc += (double)t;
    }
  }
  return acc;
}

// Workgroups of 8 waves own 64 V rows or columns each, V = 4 for large problems: partial sums are fetched four
// entries to a lane (128-bit loads: the rows of the partial sums are pitched at multiples of 64 entries), so a
// wave's ten loads cover what forty did with one entry per lane, and the totals of the tiles, which every
// workgroup adds up for itself, are added up a quarter as often.  V = 1 where that would leave most compute
// units without a workgroup.  Per entry the order of the additions is the one of reduce_kernel: 16 interleaved
// shares, each in order, then the fixed tree.  The tile totals are dealt out to 1024 shares whatever the
// number of threads, share v taking the entries v, v + 1024, ...
constexpr int kMergedWaves = 8;

// V consecutive entries of one row of the partial sums (one load per lane).
template <int V>
struct PartialLoad;
template <>
struct PartialLoad<4> {
  static __device__ __forceinline__ void load(const float* __restrict__ p, float (&v)[4]) {
    const f4v w = *reinterpret_cast<const f4v*>(p);
    v[0] = w.x;
    v[1] = w.y;
    v[2] = w.z;
    v[3] = w.w;
  }
};
template <>
struct PartialLoad<1> {
  static __device__ __forceinline__ void load(const float* __restrict__ p, float (&v)[1]) { v[0] = *p; }
};

// The 16 shares of V entries' partial sums (the lane's entries i0 .. i0 + V - 1, i0 clamped so that they stay inside
// a row of the partials) are gathered NS shares at once (share0, share0 + step, ...), a batch of 16 loads at a time:
// the loads of a batch leave together (a row past the end: the last row is fetched and not used; no branch), then
// each share's additions follow in their order.  G consecutive rows of the partials are added in fp32 first (G = 1:
// none are).  k0, step, nparts, nrows, pitch are wave-uniform.  nz (G = 1 only): nonzero partials seen per entry.
template <int G, int NS>
struct GatherBatch {
  static constexpr int kStride = 16, kBatch = (G == 1 ? 8 : (G == 4 ? 2 : 1)) * 2 / NS;
};

template <int G, int V, int NS>
__device__ __forceinline__ void gather_batch_load(const float* __restrict__ part, int k0, int step, int nrows, int i0,
                                                  int pitch, float (&v)[NS][GatherBatch<G, NS>::kBatch][G][V]) {
  using B = GatherBatch<G, NS>;
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int b = 0; b < B::kBatch; ++b)
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int k = (k0 + s * step + b * B::kStride) * G + g;
        PartialLoad<V>::load(part + (size_t)min(k, nrows - 1) * pitch + i0, v[s][b][g]);
      }
}

template <int G, int V, int NS>
__device__ __forceinline__ void gather_batch_add(const float (&v)[NS][GatherBatch<G, NS>::kBatch][G][V], int k0, int step,
                                                 int nparts, int nrows, double (&acc)[NS][V], int (&nz)[V]) {
  using B = GatherBatch<G, NS>;
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int b = 0; b < B::kBatch; ++b) {
      const int kb = k0 + s * step + b * B::kStride;
      if (kb < nparts) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          float t = v[s][b][0][e];
#pragma unroll
          for (int g = 1; g < G; ++g) t += kb * G + g < nrows ? v[s][b][g][e] : 0.f;
          if (G == 1) nz[e] += t != 0.f ? 1 : 0;
          acc[s][e] += (double)t;
        }
      }
    }
}

// the batches from k0 on (acc and nz are added to)
template <int G, int V, int NS>
__device__ __forceinline__ void gather_shares(const float* __restrict__ part, int k0, int step, int nparts, int nrows,
                                              int i0, int pitch, double (&acc)[NS][V], int (&nz)[V]) {
  using B = GatherBatch<G, NS>;
  for (; k0 < nparts; k0 += B::kStride * B::kBatch) {
    float v[NS][B::kBatch][G][V];
    gather_batch_load<G, V, NS>(part, k0, step, nrows, i0, pitch, v);
    gather_batch_add<G, V, NS>(v, k0, step, nparts, nrows, acc, nz);
  }
}

// The totals of the tiles stored one per group (tgroup = 1): the thread's NP shares side by side, a batch of 16 loads
// at a time; share s stands at entry u + s * step + lane with u wave-uniform (a scalar base address plus the lane).
template <int NP>
struct TileBatch {
  static constexpr int kShares = 1024, kBatch = 16 / NP;
};

template <int NP>
__device__ __forceinline__ void tile_batch_load(const float* __restrict__ tilesum, int ngroups, int u, int step, int ln,
                                                float (&v)[NP][TileBatch<NP>::kBatch]) {
  using B = TileBatch<NP>;
#pragma unroll
  for (int s = 0; s < NP; ++s)
#pragma unroll
    for (int b = 0; b < B::kBatch; ++b) {
      const int ub = u + s * step + b * B::kShares;
      const int uc = min(ub, ngroups - 1);
      const float w = (tilesum + uc)[min(ln, ngroups - 1 - uc)];
      v[s][b] = ub + ln < ngroups ? w : 0.f;
    }
}

template <int NP>
__device__ __forceinline__ void tile_batch_add(const float (&v)[NP][TileBatch<NP>::kBatch], double (&acc)[NP]) {
#pragma unroll
  for (int s = 0; s < NP; ++s)
#pragma unroll
    for (int b = 0; b < TileBatch<NP>::kBatch; ++b) acc[s] += (double)v[s][b];
}

template <int NP>
__device__ __forceinline__ void plain_tile_totals(const float* __restrict__ tilesum, int ngroups, int u, int step, int ln,
                                                  double (&acc)[NP]) {
  using B = TileBatch<NP>;
  for (; u < ngroups; u += B::kShares * B::kBatch) {
    float v[NP][B::kBatch];
    tile_batch_load<NP>(tilesum, ngroups, u, step, ln, v);
    tile_batch_add<NP>(v, acc);
  }
}

template <int V>
__global__ __launch_bounds__(64 * kMergedWaves) void reduce_update_kernel(ReduceArgs A, UpdateArgs U, TileTotals T,
                                                                          ScreenCtlArgs K) {
  constexpr int NW = kMergedWaves, kShares = 1024, kPerThread = kShares / (64 * NW), kE = 64 * V;
  __shared__ double red[16 * kE];
  __shared__ double eta_part[kShares / 64];
  __shared__ int nzw[NW][kE / 64];
  __shared__ int readw[NW];
  const int t = threadIdx.x;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6), ln = t & 63;
  // the schedule keeper adds up what the lean sweep read (its loads leave with everybody else's)
  const bool keeper = K.mode == 2 && blockIdx.x == gridDim.x - 1;
  int nread = 0, renewed = 0;
  if (keeper) {
    renewed = K.ctl[kCtlRenew];
    constexpr int kBatch = 8;
    for (int e0 = t; e0 < K.nwg; e0 += 64 * NW * kBatch) {
      int v[kBatch];
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        const int e = e0 + b * 64 * NW;
        v[b] = e < K.nwg ? K.wg_reads[e] : 0;
      }
#pragma unroll
      for (int b = 0; b < kBatch; ++b) nread += v[b];
    }
  }
  // which rows or columns; eq. (6) inputs of this thread's entry (threads 0 .. 64 V - 1), fetched early
  const int nwm = (A.m + kE - 1) / kE;
  const bool rows = (int)blockIdx.x < nwm;
  const int base = (rows ? (int)blockIdx.x : (int)blockIdx.x - nwm) * kE;
  const int len = rows ? A.m : A.n, pitch = rows ? A.mp : A.np;
  const int idx = base + t;
  const bool owner = t < kE && idx < len;
  // (fetched by every thread, from an entry that exists: no branch around the loads, nothing waits here)
  const int idc = min(idx, len - 1);
  const double ab_ld = rows ? U.a_in[idc] : U.b_in[idc];
  const float pq_ld = rows ? A.p[idc] : A.q[idc];
  // (the stop flag, theta and the sum of p travel with the other loads; the flag is tested before the first store)
  const int stop_ld = __hip_atomic_load(A.V.done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  const double theta = vector_load_uniform(A.V.theta + U.par), sum_p = vector_load_uniform(A.V.sum_p);
  // the partial sums of this workgroup's entries: wave w forms the shares w and w + 8 of the lane's V entries
  // (lanes past the end of a row of partials fetch its last ones; nobody reads what they leave)
  const int i0 = min(base + V * ln, pitch - V);
  const bool grouped = !rows && A.cgroup > 1;
  const int nparts = rows ? A.nseg : grouped ? (A.ntr + A.cgroup - 1) / A.cgroup : A.ntr;
  const int nrows_part = rows ? A.nseg : A.ntr;
  const float* __restrict__ part = rows ? A.rowpart : A.colpart;
  constexpr int NS = 16 / NW;  // shares of the partial sums per wave: w and w + 8
  int nzv[V];
  double av[NS][V];
#pragma unroll
  for (int e = 0; e < V; ++e) nzv[e] = 0;
#pragma unroll
  for (int si = 0; si < NS; ++si)
#pragma unroll
    for (int e = 0; e < V; ++e) av[si][e] = 0.0;
  // the shares of the tile totals: share v = 64 w + lane of accumulator s, added in index order
  double acc[kPerThread];
#pragma unroll
  for (int s = 0; s < kPerThread; ++s) acc[s] = 0.0;
  const bool tiles_grouped = T.tgroup == kColGroup || T.tgroup == kPointsColGroup;
  if (!tiles_grouped && !grouped) {
    // everything stored ready to add (the lean sweeps): the first batch of the tile totals and the first batch of
    // the partial sums are on their way together before anything is added: one trip to memory instead of two
    using TB = TileBatch<kPerThread>;
    using GB = GatherBatch<1, NS>;
    const int ngroups = T.tile_rows * T.nseg;
    float tv[kPerThread][TB::kBatch];
    float gv[NS][GB::kBatch][1][V];
    tile_batch_load<kPerThread>(T.tilesum, ngroups, 64 * wv, 64 * NW, ln, tv);
    gather_batch_load<1, V, NS>(part, wv, NW, nrows_part, i0, pitch, gv);
    __builtin_amdgcn_sched_barrier(0);
    tile_batch_add<kPerThread>(tv, acc);
    plain_tile_totals<kPerThread>(T.tilesum, ngroups, 64 * wv + TB::kShares * TB::kBatch, 64 * NW, ln, acc);
    gather_batch_add<1, V, NS>(gv, wv, NW, nparts, nrows_part, av, nzv);
    gather_shares<1, V, NS>(part, wv + GB::kStride * GB::kBatch, NW, nparts, nrows_part, i0, pitch, av, nzv);
  } else {
    if (T.tgroup == kColGroup) {
#pragma unroll
      for (int s = 0; s < kPerThread; ++s) acc[s] = grouped_tile_totals<kColGroup>(T, 64 * wv + s * 64 * NW + ln, ln);
    } else if (T.tgroup == kPointsColGroup) {
#pragma unroll
      for (int s = 0; s < kPerThread; ++s) acc[s] = grouped_tile_totals<kPointsColGroup>(T, 64 * wv + s * 64 * NW + ln, ln);
    } else {
      plain_tile_totals<kPerThread>(T.tilesum, T.tile_rows * T.nseg, 64 * wv, 64 * NW, ln, acc);
    }
    if (!grouped) gather_shares<1, V, NS>(part, wv, NW, nparts, nrows_part, i0, pitch, av, nzv);
    else if (A.cgroup == kColGroup) gather_shares<kColGroup, V, NS>(part, wv, NW, nparts, nrows_part, i0, pitch, av, nzv);
    else gather_shares<kPointsColGroup, V, NS>(part, wv, NW, nparts, nrows_part, i0, pitch, av, nzv);
  }
#pragma unroll
  for (int si = 0; si < NS; ++si) {
    double* dst = red + (wv + si * NW) * kE + V * ln;
#pragma unroll
    for (int e = 0; e < V; ++e) dst[e] = av[si][e];
  }
  const double ab_in = owner ? ab_ld : 0.0;
  const float pq = owner ? pq_ld : 0.f;
#pragma unroll
  for (int s = 0; s < kPerThread; ++s) {
    const double w = wave_sum_f64(acc[s]);
    if (ln == 0) eta_part[wv + s * NW] = w;
  }
  if (keeper) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nread += __shfl_xor(nread, off, 64);
  }
  if (ln == 0) readw[wv] = nread;
  {  // nonzero partials per block of 64 entries (64 / V lanes): the entries that exist only
    int cnt = 0;
#pragma unroll
    for (int e = 0; e < V; ++e) cnt += base + V * ln + e < len ? nzv[e] : 0;
    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0xB1, 0xF, 0xF, false);   // the first four steps of wave_sum: the sum of
    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x4E, 0xF, 0xF, false);   // each row of 16 lanes, in every lane of it
    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x141, 0xF, 0xF, false);
    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x140, 0xF, 0xF, false);
    if (V == 4) {
      if ((ln & 15) == 0) nzw[wv][ln >> 4] = cnt;
    } else {  // the whole wave is one block: the four rows of lanes
      const int whole = (__builtin_amdgcn_readlane(cnt, 0) + __builtin_amdgcn_readlane(cnt, 16)) +
                        (__builtin_amdgcn_readlane(cnt, 32) + __builtin_amdgcn_readlane(cnt, 48));
      if (ln == 0) nzw[wv][0] = whole;
    }
  }
  __syncthreads();
  if (__builtin_amdgcn_readfirstlane(stop_ld)) return;
  if (t == 0 && blockIdx.x == gridDim.x - 1 && K.mode != 0) {
    if (K.mode == 1 || renewed) {  // new bounds: nothing paid yet, the floor is what the next sweep reads
      K.ctl[kCtlRenew] = 0;
      K.ctl[kCtlSince] = 0;
      K.ctl[kCtlFloor] = -1;
      K.ctl[kCtlPaid] = 0;
    } else {
      int total = 0;
      for (int k = 0; k < NW; ++k) total += readw[k];
      const int since = K.ctl[kCtlSince] + 1;
      int floor_reads = K.ctl[kCtlFloor], paid = K.ctl[kCtlPaid];
      if (floor_reads < 0) floor_reads = total;
      else if (total > floor_reads) paid += total - floor_reads;
      K.ctl[kCtlSince] = since;
      K.ctl[kCtlFloor] = floor_reads;
      K.ctl[kCtlPaid] = paid;
      if (paid >= K.price || since >= K.max_since) K.ctl[kCtlRenew] = 1;
    }
  }
  if (t >= kE) return;  // (waves 0 .. V - 1 finish: one entry per thread, one block of 64 entries per wave)
  // the 16 shares of the entry (the fixed tree sum_partials_16 ends with), the residual, the block's sums
  double w[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) w[k] = red[k * kE + t];
  const double total_e = (((w[0] + w[8]) + (w[4] + w[12])) + ((w[2] + w[10]) + (w[6] + w[14]))) +
                         (((w[1] + w[9]) + (w[5] + w[13])) + ((w[3] + w[11]) + (w[7] + w[15])));
  double res = 0.0;
  if (owner) {
    res = total_e - (double)pq;
    (rows ? A.V.r : A.V.s)[idx] = res;
  }
  const double sum = wave_sum_f64(res), sumsq = wave_sum_f64(res * res);
  const int blk = (rows ? 0 : A.nbm) + (base >> 6) + wv;  // this wave's block of 64 entries
  const bool blk_exists = (base >> 6) + wv < (rows ? A.nbm : A.nbn);
  double eta_total = 0.0;
  for (int k = 0; k < kShares / 64; ++k) eta_total += eta_part[k];
  const double eta = (eta_total - sum_p) / ((double)A.m + (double)A.n);
  const double cst = 2.0 * eta - theta;
  if (owner) {
    if (rows) {
      A.V.phi[idx] = (float)((ab_in - 2.0 * res + cst) / (double)A.n);
      U.a_out[idx] = ab_in - res;
    } else {
      A.V.varphi[idx] = (float)((ab_in - 2.0 * res + cst) / (double)A.m);
      U.b_out[idx] = ab_in - res;
    }
  }
  if (ln == 0 && blk_exists) {
    A.V.part[blk] = sum;
    A.V.part[A.nbm + A.nbn + blk] = sumsq;
  }
  // rows: how many of the block's row-segment sums are not zero (the density of the plan the host steers by)
  if (ln == 0 && blk_exists) {
    int cnt = 0;
    for (int k = 0; k < NW; ++k) cnt += nzw[k][wv];
    A.V.part[2 * (A.nbm + A.nbn) + blk] = rows ? (double)cnt : 0.0;
  }
  if (blockIdx.x == 0 && t == 0) A.V.theta[U.par ^ 1] = theta - eta;
}
