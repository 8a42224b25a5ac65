// Single-workgroup solver for tiny problems.
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

// ------------------------------------------------------------------------------------------
// Resident solver for tiny problems (at most 128 x 256): one workgroup keeps X and C in registers
// and runs a whole stretch of iterations (the ones between two residual checks) in one launch, so
// an iteration costs two workgroup barriers instead of a kernel launch.  Wave w owns rows
// w, w + 16, ...; a lane owns four columns.  The eq. (6) state lives in registers of "owner"
// threads: thread t < m owns row t (a_t, p_t), thread 256 + j owns column j (b_j, q_j); phi and
// varphi travel through LDS.  Per iteration: (A) every wave updates its rows (first half of
// eq. (8) and the quadratic scaling), leaves the row sums and its column partials in LDS;
// barrier; (B) the owners form the residuals, eta, and the new phi, varphi, a, b, theta in fp64;
// barrier.  Arithmetic and precision are those of the multi-launch path (fp32 sweep and
// fp32 sums over at most 256 elements of a row resp. 8 of a column, fp64 above).
// ------------------------------------------------------------------------------------------
struct ResidentArgs {
  float* X;
  const float* C;
  const float* p;
  const float* q;
  VecState V;
  const double* a_in;
  const double* b_in;
  double* a_out;
  double* b_out;
  int theta_in, theta_out;  // entries of V.theta to read and to write
  int m, n, ldx, ldc;
  float rho, scale;
  int iters;  // sweeps to run (>= 1)
  int first;  // X_0 = 0: nothing to read
};

constexpr int kResidentCols = 256, kResidentMaxRows = 128;

// NW waves, R rows per wave, CPL columns per lane (n <= 64 * CPL).  128 rows of 256 columns need
// 8 waves with twice the registers each; narrower problems use fewer columns per lane instead, so
// that no lane sits idle, and keep 16 waves.
template <int R, int NW, int CPL>
__global__ __launch_bounds__(64 * NW) void resident_kernel(ResidentArgs A) {
  static_assert(NW >= 8 && R * NW <= kResidentMaxRows && 64 * CPL <= kResidentCols, "owner waves 0, 1 and 4..7 must exist");
  if (*A.V.done) return;
  __shared__ float lds_phi[kResidentMaxRows];
  __shared__ float lds_varphi[kResidentCols];
  __shared__ float lds_row[kResidentMaxRows];
  __shared__ float lds_col[NW][64 * CPL];
  __shared__ double red[NW];
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int j0 = lane * CPL;
  const float rho = A.rho, scale = A.scale;

  float x[R][CPL], c[R][CPL];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = wave + NW * r;
#pragma unroll
    for (int e = 0; e < CPL; ++e) {
      c[r][e] = 0.f;
      x[r][e] = 0.f;
      if (row < A.m && j0 + e < A.n) {
        c[r][e] = A.C[(size_t)row * A.ldc + j0 + e];
        if (!A.first) x[r][e] = A.X[(size_t)row * A.ldx + j0 + e];
      }
    }
  }
  const bool row_owner = t < A.m;  // (m <= 128: waves 0 and 1)
  const int jc = t - 256;          // waves 4..7
  const bool col_owner = jc >= 0 && jc < A.n;
  double state = 0.0, target = 0.0;  // a_t and p_t of a row owner, b_j and q_j of a column owner
  if (row_owner) { state = A.a_in[t]; target = (double)A.p[t]; }
  if (col_owner) { state = A.b_in[jc]; target = (double)A.q[jc]; }
  double theta = A.V.theta[A.theta_in];
  const double sum_p = *A.V.sum_p;
  // (divisions by m + n, n and m as multiplications by the fp64 reciprocals: one more rounding of 1e-16)
  const double inv_mn = 1.0 / ((double)A.m + (double)A.n), inv_n = 1.0 / (double)A.n, inv_m = 1.0 / (double)A.m;
  // rows and columns that do not exist get a huge negative dual value: the clamp zeroes them
  if (t < kResidentMaxRows) {
    lds_phi[t] = row_owner ? A.V.phi[t] : kMaskedOut;
    lds_row[t] = 0.f;
  }
  if (jc >= 0 && jc < kResidentCols) lds_varphi[jc] = col_owner ? A.V.varphi[jc] : kMaskedOut;
  __syncthreads();

  const bool owner_wave = wave < 2 || (wave >= 4 && wave < 8);
  double res = 0.0;  // the owner's residual after the latest sweep
  float dual = 0.f;  // the owner's phi_t resp. varphi_j
  for (int it = 0; it < A.iters; ++it) {
    // (A) sweep
    float vp[CPL], colacc[CPL];
#pragma unroll
    for (int e = 0; e < CPL; ++e) {
      vp[e] = lds_varphi[j0 + e];
      colacc[e] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = wave + NW * r;
      const float ph = lds_phi[row];
      float rowacc = 0.f;
#pragma unroll
      for (int e = 0; e < CPL; ++e) {
        const float v = fmaxf(fmaf(-rho, c[r][e], x[r][e] + (vp[e] + ph)), 0.f) * scale;
        x[r][e] = v;
        colacc[e] += v;
        rowacc += v;
      }
      const float tot = wave_sum(rowacc);
      if (lane == 0) lds_row[row] = tot;
    }
#pragma unroll
    for (int e = 0; e < CPL; ++e) lds_col[wave][j0 + e] = colacc[e];
    __syncthreads();
    // (B) eq. (6)
    if (owner_wave) {
      // 1^T X 1, the same bits in every owner wave
      const double tot = wave_sum_f64((double)lds_row[lane] + (double)lds_row[lane + 64]);
      const double eta = (tot - sum_p) * inv_mn;
      const double cst = 2.0 * eta - theta;
      theta -= eta;
      if (wave < 2) {
        res = (double)lds_row[t] - target;
        dual = (float)((state - 2.0 * res + cst) * inv_n);
        state -= res;
        if (row_owner) lds_phi[t] = dual;
      } else if (jc < 64 * CPL) {
        double sj = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) sj += (double)lds_col[w][jc];
        res = sj - target;
        dual = (float)((state - 2.0 * res + cst) * inv_m);
        state -= res;
        if (col_owner) lds_varphi[jc] = dual;
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = wave + NW * r;
#pragma unroll
    for (int e = 0; e < CPL; ++e)
      if (row < A.m && j0 + e < A.n) A.X[(size_t)row * A.ldx + j0 + e] = x[r][e];
  }
  if (row_owner) {
    A.V.phi[t] = dual;
    A.a_out[t] = state;
    A.V.r[t] = res;
  }
  if (col_owner) {
    A.V.varphi[jc] = dual;
    A.b_out[jc] = state;
    A.V.s[jc] = res;
  }
  const double r2 = block_sum_f64(row_owner ? res * res : 0.0, red);
  const double s2 = block_sum_f64(col_owner ? res * res : 0.0, red);
  if (t == 0) {
    A.V.theta[A.theta_out] = theta;
    A.V.resid[0] = r2;
    A.V.resid[1] = s2;
    A.V.resid[2] = 0.0;
  }
}

template <int CPL>
void launch_resident(const ResidentArgs& RS, hipStream_t stream, hipEvent_t e0, hipEvent_t e1) {
  const int m = RS.m;  // (e0, e1: events that take the kernel's own start and end, or null)
  if (m <= 16) launch_timed((resident_kernel<1, 16, CPL>), dim3(1), dim3(1024), stream, e0, e1, RS);
  else if (m <= 32) launch_timed((resident_kernel<2, 16, CPL>), dim3(1), dim3(1024), stream, e0, e1, RS);
  else if (m <= 64) launch_timed((resident_kernel<4, 16, CPL>), dim3(1), dim3(1024), stream, e0, e1, RS);
  else if constexpr (CPL < 4) launch_timed((resident_kernel<8, 16, CPL>), dim3(1), dim3(1024), stream, e0, e1, RS);
  else launch_timed((resident_kernel<16, 8, CPL>), dim3(1), dim3(512), stream, e0, e1, RS);
}

// Working copy of the cost for the weighted l1 term: out[i][j] = C[i][j] + W[i][j] (pitch ld; the
// pad columns keep their zeros).  +inf entries of C (forbidden pairs) stay +inf.
__global__ __launch_bounds__(256) void add_weights_kernel(float* __restrict__ out, const float* __restrict__ C,
                                                          const float* __restrict__ W, int m, int n, int ld) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  for (int i = blockIdx.y; i < m; i += gridDim.y)
    out[(size_t)i * ld + j] = C[(size_t)i * n + j] + W[(size_t)i * n + j];
}

// S6: r_primal of Appendix C; raises the stop flag at the first check that passes so that every
// later kernel of the solve returns at once.  With gap_tol > 0 a check passes only if objective,
// duality gap and dual residual were evaluated for this very iterate (gap_fresh) and
// |gap| <= gap_tol * |objective|, dual_res <= gap_tol (Section 3, "Stopping criteria").
__global__ void status_kernel(VecState V, int iters, double tol, double gap_tol, int gap_fresh) {
  if (*V.done) return;
  const double r2 = V.resid[0], s2 = V.resid[1];
  V.status->r2 = r2;
  V.status->s2 = s2;
  V.status->nz_segments = V.resid[2];
  V.status->iters = iters;
  if (gap_fresh) V.status->gap_iters = iters;
  bool pass = tol > 0.0 && r2 <= tol * tol && s2 <= tol * tol;
  if (pass && gap_tol > 0.0) {
    const double objective = V.status->cost + V.status->h;
    pass = gap_fresh && fabs(V.status->gap) <= gap_tol * fabs(objective) && V.status->dual_res <= gap_tol;
  }
  if (pass) {
    V.status->converged = 1;
    __threadfence();
    *V.done = 1;
  }
}
