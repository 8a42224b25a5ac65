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

// One row's terms, added to a lane's three running sums.  Products and sums stay separate operations (no
// contraction into fused multiply-adds), so that every kernel that calls this adds up the same numbers.
__device__ __forceinline__ void gap_accumulate(const f4v& c, const f4v& x, const f4v& w, float& cx, float& xx, float& ww,
                                               f4v& x2, f4v& w2) {
#pragma clang fp contract(off)
  x2 = x * x;
  w2 = w * w;
  // (a forbidden pair carries c = +inf and x = 0: it adds nothing to <C,X>)
  const f4v cxv = {x.x > 0.f ? c.x * x.x : 0.f, x.y > 0.f ? c.y * x.y : 0.f, x.z > 0.f ? c.z * x.z : 0.f,
                   x.w > 0.f ? c.w * x.w : 0.f};
  cx += (cxv.x + cxv.y) + (cxv.z + cxv.w);
  xx += (x2.x + x2.y) + (x2.z + x2.w);
  ww += (w2.x + w2.y) + (w2.z + w2.w);
}

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
    f4v x2, w2;
    gap_accumulate(c, x, w, cx, xx, ww, x2, w2);
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

// ------------------------------------------------------------------------------------------
// The same partial sums for plans known to be sparse, from a fraction of the traffic.  A row segment
// whose X is zero and whose screening bound (the certificate of the screened sweeps, to the letter) is
// not positive adds nothing to any of the three sums: x = 0 there, and [phi_i + varphi_j - rho C_ij]_+,
// which is what the sweep would compute from x = 0, is certified to be zero.  One wave per 64 x 256
// tile decides its 64 row segments at once and walks through those that are left, reading C and the
// nonzero lines of X only there.  The sums are formed in the order of gap_kernel -- per lane over the
// rows of a chunk of 8, across the wave, the four chunks of a 32-row tile as (0 + 1) + (2 + 3) -- and
// the skipped terms are exact zeros, so gap_part comes out bit for bit as gap_kernel leaves it.
// flags: the line flags of the lean sweep (lines) or the row-segment sums (rowsums) of the X in memory.
// grid = (nseg, ceil(tiles of 64 rows / 4)), 256 threads.
// ------------------------------------------------------------------------------------------
struct GapLeanArgs {
  GapArgs G;
  const float* mprime;           // [nseg][m] bounds of the epoch: M,
  const float* mprime2;          //   M2
  const unsigned char* jstar;    //   and j*
  const float* varphi0;          // the epoch's varphi (padded)
  const unsigned char* lines;    // [nseg][m] nonzero 128-byte lines of every row segment of X, or null
  const float* rowsums;          // [nseg][m] row-segment sums of X (used when lines is null)
  int n_mem;                     // columns that may be accessed in a row of X and C
  int mp;                        // pitch of the arrays kept per row segment
  int ntr64, ntr32;              // tiles of 64 and of 32 rows
};

template <bool EDGE>
__device__ __forceinline__ void gap_lean_body(const GapLeanArgs& L, int lane, int seg, int tr, float (*sums)[3]) {
  const GapArgs& A = L.G;
  const int j0 = seg * kSegCols + lane * 4;
  const int nmem = EDGE ? min(max(L.n_mem - j0, 0), 4) : 4;
  const int r0 = tr * 64;
  const int nrows = min(A.m - r0, 64);
  const size_t ldx = (size_t)A.ldx, ldc = (size_t)A.ldc;
  const float* __restrict__ Cp = A.C + (size_t)r0 * ldc + j0;
  const float* __restrict__ Xp = A.X + (size_t)r0 * ldx + j0;
  const size_t ridx = (size_t)seg * L.mp + r0 + lane;
  const f4v vp = load_varphi_padded(A.varphi, j0);
  const f4v vp0 = load_varphi_padded(L.varphi0, j0);
  float ph = kMaskedOut, mpr = 0.f, mpr2 = 0.f;
  unsigned lines = 0, js = 0;
  if (lane < nrows) {
    ph = A.phi[r0 + lane];
    mpr = L.mprime[ridx];
    mpr2 = L.mprime2[ridx];
    js = L.jstar[ridx];
    if (L.lines) lines = L.lines[ridx];
    else lines = fbits(L.rowsums[ridx]) != 0 ? 0xffu : 0u;
  }
  const f4v dv = vp - vp0;
  const float d = fmaxf(fmaxf(dv.x, dv.y), fmaxf(dv.z, dv.w));
  const float a = fmaxf(fmaxf(unmasked_abs(vp.x), unmasked_abs(vp.y)), fmaxf(unmasked_abs(vp.z), unmasked_abs(vp.w)));
  const float delta = wave_max(d), mag = wave_max(a);
  const bool below = certified_zero(mpr, mpr2, js, dv, delta, mag, ph);  // (the certificate of screened_body)
  const bool certified = lane >= nrows || (lines == 0 && below);
  unsigned long long todo = ~__builtin_amdgcn_ballot_w64(certified);
  const unsigned myline = (unsigned)lane >> 3;
  float cx = 0.f, xx = 0.f, ww = 0.f;
  int chunk = -1;
  auto flush = [&]() {
    const float a0 = wave_sum(cx), a1 = wave_sum(xx), a2 = wave_sum(ww);
    if (lane == 0) {
      sums[chunk][0] = a0;
      sums[chunk][1] = a1;
      sums[chunk][2] = a2;
    }
  };
  constexpr int kWalk = 4;
  while (todo != 0) {
    int row[kWalk];
    f4v c[kWalk], x[kWalk];
#pragma unroll
    for (int b = 0; b < kWalk; ++b) {
      row[b] = -1;
      c[b] = f4v{0.f, 0.f, 0.f, 0.f};
      x[b] = f4v{0.f, 0.f, 0.f, 0.f};
      if (todo != 0) {
        row[b] = __builtin_ctzll(todo);
        todo &= todo - 1;
        c[b] = ld4<EDGE, false>(Cp + row[b] * ldc, nmem);
        const unsigned ol = (unsigned)__builtin_amdgcn_readlane((int)lines, row[b]);
        if ((ol >> myline) & 1) x[b] = ld4<EDGE, false>(Xp + row[b] * ldx, nmem);
      }
    }
#pragma unroll
    for (int b = 0; b < kWalk; ++b) {
      const int u = row[b];
      if (u >= 0) {
        if ((u >> 3) != chunk) {
          if (chunk >= 0) flush();
          chunk = u >> 3;
          cx = xx = ww = 0.f;
        }
        const float phu = __builtin_bit_cast(float, __builtin_amdgcn_readlane(fbits(ph), u));
        const f4v w = xbar4(f4v{0.f, 0.f, 0.f, 0.f}, c[b], vp + phu, A.rho);
        f4v x2, w2;
        gap_accumulate(c[b], x[b], w, cx, xx, ww, x2, w2);
      }
    }
  }
  if (chunk >= 0) flush();
}

__global__ __launch_bounds__(64 * kLeanWaves) void gap_lean_kernel(GapLeanArgs L) {
  if (L.G.done && *L.G.done) return;
  __shared__ float sums[kLeanWaves][8][3];  // per wave: the eight chunks of 8 rows of its tile
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y * kLeanWaves + wave;
  if (lane < 24) (&sums[wave][0][0])[lane] = 0.f;
  __syncthreads();
  if (tr < L.ntr64) {
    if ((seg + 1) * kSegCols <= L.G.n) gap_lean_body<false>(L, lane, seg, tr, sums[wave]);
    else gap_lean_body<true>(L, lane, seg, tr, sums[wave]);
  }
  __syncthreads();
  const int t = threadIdx.x;
  if (t < 6 * kLeanWaves) {  // (wave, half, sum): a 32-row tile is four chunks
    const int w = t / 6, half = (t / 3) & 1, k = t % 3;
    const int tr32 = (blockIdx.y * kLeanWaves + w) * 2 + half;
    if (tr32 < L.ntr32) {
      const float(*c)[3] = sums[w] + 4 * half;
      L.G.gap_part[(size_t)(tr32 * L.G.nseg + seg) * 3 + k] = (c[0][k] + c[1][k]) + (c[2][k] + c[3][k]);
    }
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
