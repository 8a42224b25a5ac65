// Status, objective, duality gap and dual residual.
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

// ------------------------------------------------------------------------------------------
// S7: objective, duality gap and dual residual of (X, phi, varphi) (Appendix C).  One read-only
// pass: <C,X>, ||X||_F^2 and ||[phi 1^T + 1 varphi^T - rho C]_+||_F^2 per tile, plus, for the
// group lasso, the same two squared norms per (class, column) group.
// ------------------------------------------------------------------------------------------
struct GapArgs {
  const float* X;
  const float* C;
  const float* phi;
  const float* varphi;
  const int* row_class;  // null unless group lasso
  float* gap_part;       // [ntiles][3]
  float* gx;             // [num_classes][n] sum x^2   (group lasso)
  float* gw;             // [num_classes][n] sum w^2
  int m, n, nseg;
  int ldx, ldc;
  float rho;
  PointArgs pts;         // used instead of C when C is null
  const int* done;       // the stop flag for the passes that belong to a residual check (they skip once it is up), or null
};

__global__ __launch_bounds__(kBlock) void gap_kernel(GapArgs A) {
  if (A.done && *A.done) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y;
  const int j0 = seg * kSegCols + lane * 4;
  const int nvalid = min(max(A.n - j0, 0), 4);
  const f4v vp = load_varphi(A.varphi, j0, nvalid);
  const int rbeg = tr * kTileRows + wave * kLoopRows;
  const int rend = min(rbeg + kLoopRows, A.m);
  float cx = 0.f, xx = 0.f, ww = 0.f;
  int cur = -1;
  f4v ax = {0.f, 0.f, 0.f, 0.f}, aw = {0.f, 0.f, 0.f, 0.f};
  for (int i = rbeg; i < rend; ++i) {
    const f4v c = A.C ? load4(A.C + (size_t)i * A.ldc + j0, nvalid) : cost4_from_points(A.pts, i, j0, nvalid);
    const f4v x = load4(A.X + (size_t)i * A.ldx + j0, nvalid);
    const f4v w = xbar4(f4v{0.f, 0.f, 0.f, 0.f}, c, vp + A.phi[i], A.rho);
    const f4v x2 = x * x, w2 = w * w;
    // (a forbidden pair carries c = +inf and x = 0: it adds nothing to <C,X>)
    const f4v cxv = {x.x > 0.f ? c.x * x.x : 0.f, x.y > 0.f ? c.y * x.y : 0.f, x.z > 0.f ? c.z * x.z : 0.f,
                     x.w > 0.f ? c.w * x.w : 0.f};
    cx += (cxv.x + cxv.y) + (cxv.z + cxv.w);
    xx += (x2.x + x2.y) + (x2.z + x2.w);
    ww += (w2.x + w2.y) + (w2.z + w2.w);
    if (A.row_class) {
      const int cls = A.row_class[i];
      if (cls != cur) {
        if (cur >= 0) {
          flush_group(A.gx + (size_t)cur * A.n + j0, ax, nvalid);
          flush_group(A.gw + (size_t)cur * A.n + j0, aw, nvalid);
        }
        cur = cls;
        ax = f4v{0.f, 0.f, 0.f, 0.f};
        aw = f4v{0.f, 0.f, 0.f, 0.f};
      }
      ax += x2;
      aw += w2;
    }
  }
  if (cur >= 0) {
    flush_group(A.gx + (size_t)cur * A.n + j0, ax, nvalid);
    flush_group(A.gw + (size_t)cur * A.n + j0, aw, nvalid);
  }
  __shared__ float ws[3][kWavesPerBlock];
  const float a0 = wave_sum(cx), a1 = wave_sum(xx), a2 = wave_sum(ww);
  if (lane == 0) { ws[0][wave] = a0; ws[1][wave] = a1; ws[2][wave] = a2; }
  __syncthreads();
  if (threadIdx.x < 3) {
    const int k = threadIdx.x;
    A.gap_part[(size_t)(tr * A.nseg + seg) * 3 + k] = (ws[k][0] + ws[k][1]) + (ws[k][2] + ws[k][3]);
  }
}

// Combines the partials into the terms of the gap formula, in fp64.  With u = phi/rho,
// v = varphi/rho, W = [u 1^T + 1 v^T - C]_+ :  gap = <C,X> + h(X) - (p^T u + q^T v) + h*(W);
// where h* is an indicator the violation is reported as dual_res instead.
__global__ __launch_bounds__(1024) void gap_final_kernel(VecState V, const float* __restrict__ gap_part, int ntiles,
                                                         const float* __restrict__ gx, const float* __restrict__ gw,
                                                         size_t ngroups, const float* __restrict__ p,
                                                         const float* __restrict__ q, int m, int n, double rho,
                                                         int reg_kind, double lambda, double mu, const int* done) {
  if (done && *done) return;
  __shared__ double red[1024];
  const int t = threadIdx.x;
  double cx = 0.0, xx = 0.0, ww = 0.0, dl = 0.0, gl = 0.0, ex2 = 0.0;
  for (int e = t; e < ntiles; e += blockDim.x) {
    cx += (double)gap_part[(size_t)e * 3 + 0];
    xx += (double)gap_part[(size_t)e * 3 + 1];
    ww += (double)gap_part[(size_t)e * 3 + 2];
  }
  for (int i = t; i < m; i += blockDim.x) dl += (double)p[i] * (double)V.phi[i];
  for (int j = t; j < n; j += blockDim.x) dl += (double)q[j] * (double)V.varphi[j];
  if (reg_kind == DROT_REG_GROUP_LASSO) {
    for (size_t g = t; g < ngroups; g += blockDim.x) {
      gl += sqrt((double)gx[g]);
      double ex = sqrt((double)gw[g]) / rho - mu;
      if (ex < 0.0) ex = 0.0;
      ex2 += ex * ex;
    }
  }
  cx = block_sum_f64(cx, red);
  xx = block_sum_f64(xx, red);
  ww = block_sum_f64(ww, red) / (rho * rho);  // ||W||_F^2
  dl = block_sum_f64(dl, red) / rho;
  gl = block_sum_f64(gl, red);
  ex2 = block_sum_f64(ex2, red);
  if (t == 0) {
    double h = 0.0, hconj = 0.0, dres = 0.0;
    if (reg_kind == DROT_REG_NONE || (reg_kind == DROT_REG_QUADRATIC && lambda <= 0.0)) {
      dres = sqrt(ww);
    } else if (reg_kind == DROT_REG_QUADRATIC) {
      h = 0.5 * lambda * xx;
      hconj = ww / (2.0 * lambda);
    } else {
      h = mu * gl + 0.5 * lambda * xx;
      if (lambda > 0.0) hconj = ex2 / (2.0 * lambda);
      else dres = sqrt(ex2);
    }
    V.status->cost = cx;
    V.status->h = h;
    V.status->dual_lin = dl;
    V.status->h_conj = hconj;
    V.status->gap = cx + h - dl + hconj;
    V.status->dual_res = dres;
  }
}
