// The sweep for h = 0 and the quadratic term (32-row and 64-row tiles, even/odd scheme, fused vector update).
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

// ------------------------------------------------------------------------------------------
// S1-S4: the sweep for h = 0 and h = (lambda/2)||X||^2 (a constant scale, Section 3).
// grid = (nseg, ntr); a workgroup owns 32 rows x 256 columns; each of its 16 waves loads its
// 2 row segments of 1 KiB of X and C, updates, stores and is done.  EDGE marks the last column
// segment when n is not a multiple of 256: only there do lanes check how many of their 4
// columns exist.  NT marks the accesses non-temporal (used when X and C cannot stay in cache).
//
// Alignment (what the shifted work areas of the paper's Section "General Optimization" are for):
// row segments that straddle 128-byte lines cost 10-28 % here, so the host hands this kernel
// rows that start on a line: the caller's arrays when n % 32 == 0 and the base is aligned, else
// working copies with the pitch rounded up to 32 elements (ldx, ldc).
// ------------------------------------------------------------------------------------------
// The four columns of a lane in X or C.  In the last column segment (EDGE) a lane's columns either all
// lie inside the row as it is laid out in memory or all outside (nmem is 4 or 0): rows are a multiple
// of 32 columns long there, the caller's when n % 32 == 0, the padded working copies' otherwise, and
// the columns between n and the pitch hold zeros.  So the edge costs one predicate, not scalar accesses.
template <bool EDGE, bool NT>
__device__ __forceinline__ f4v ld4(const float* __restrict__ ptr, int nmem) {
  if (EDGE && nmem != 4) return f4v{0.f, 0.f, 0.f, 0.f};
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f4u*>(ptr));
  return *reinterpret_cast<const f4u*>(ptr);
}
template <bool EDGE, bool NT>
__device__ __forceinline__ void st4(float* __restrict__ ptr, f4v v, int nmem) {
  if (EDGE && nmem != 4) return;
  if (NT) __builtin_nontemporal_store(v, reinterpret_cast<f4u*>(ptr));
  else *reinterpret_cast<f4u*>(ptr) = v;
}

// Folds the column partials of the NW waves of a workgroup through LDS and writes the tile's
// column sums (fixed order: deterministic).
template <int NW>
__device__ __forceinline__ void write_col_partials(f4v colacc, int lane, int wave, int seg, int tr, int n, int np,
                                                   float* __restrict__ colpart) {
  __shared__ float cs[NW][kSegCols];
  *reinterpret_cast<f4v*>(&cs[wave][lane * 4]) = colacc;
  __syncthreads();
  const int t = threadIdx.x;
  if (t < kSegCols) {
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < NW; ++k) sum += cs[k][t];
    const int j = seg * kSegCols + t;
    if (j < n) colpart[(size_t)tr * np + j] = sum;
  }
}

// Total of a tile from the totals of its NW waves, in wave order.
template <int NW>
__device__ __forceinline__ void write_tile_total(float wave_total, int lane, int wave, int seg, int tr,
                                                 float* __restrict__ tilesum) {
  __shared__ float wt[NW];
  if (lane == 0) wt[wave] = wave_total;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < NW; ++k) tot += wt[k];
    tilesum[tr * gridDim.x + seg] = tot;
  }
}

// MODE selects the paper's even/odd scheme (Section "Quadratically Regularized DROT"): 0 = plain
// (read X and C, store X); 1 = read X and C, store X - rho*C; 2 = read the shifted X only (no C)
// and store the plain X.  A 1-sweep followed by a 2-sweep moves 20 bytes per element instead of 24.
// MODE 3 only forms the row and column sums of X as it stands (no update, no store): the warm start.
// Sum of `count` fp32 partials part[k*stride], k = 0..count-1, in the order every form of the vector
// update uses: 16 interleaved subsequences added left to right, then a fixed tree over the 16.
__device__ __forceinline__ double sum_partials_16(const float* __restrict__ part, size_t stride, int count) {
  double q16[16];
#pragma unroll
  for (int w = 0; w < 16; ++w) q16[w] = 0.0;
  for (int k0 = 0; k0 < count; k0 += 16) {
    // 16 independent loads in flight (clamped index, the excess ones add +0, which changes no bit)
    float v[16];
#pragma unroll
    for (int w = 0; w < 16; ++w) v[w] = part[(size_t)min(k0 + w, count - 1) * stride];
#pragma unroll
    for (int w = 0; w < 16; ++w) q16[w] += (k0 + w < count) ? (double)v[w] : 0.0;
  }
  return (((q16[0] + q16[8]) + (q16[4] + q16[12])) + ((q16[2] + q16[10]) + (q16[6] + q16[14]))) +
         (((q16[1] + q16[9]) + (q16[5] + q16[13])) + ((q16[3] + q16[11]) + (q16[7] + q16[15])));
}

// Vector update of eq. (6) for the 32 rows and 256 columns of one tile, computed redundantly by
// every workgroup that needs them from the previous sweep's partial sums (worth it while the
// partials are few: small m).  Same arithmetic as reduce_kernel + update_kernel; the workgroups
// of the first tile column / tile row also store the new a, phi / b, varphi, workgroup (0,0)
// the new theta.  Results land in LDS for the sweep that follows.
__device__ __forceinline__ void fused_update(const SweepArgs& A, const FusedUpdateArgs& F, int seg, int tr,
                                             float* __restrict__ lds_phi, float* __restrict__ lds_varphi) {
  __shared__ double red[64 * kSweepWaves];
  const int t = threadIdx.x;
  // Everything below is latency: issue every load that does not depend on another one first
  // (tile totals, column partials, row partials, p, q, a, b, theta), then synchronise.
  double acc = 0.0;
  const int ntiles = F.nseg * F.ntr;
  for (int e = t; e < ntiles; e += 64 * kSweepWaves) acc += (double)F.tilesum_prev[e];
  // columns: 4 groups of 256 threads split the row tiles.  The partials are summed in the order
  // reduce_kernel uses (16 interleaved subsequences, then a fixed tree), so that both ways of
  // doing the update give the same bits.
  const int sub = t >> 8, cidx = t & 255;
  const int j = seg * kSegCols + cidx;
  double sj = 0.0;
  if (j < A.n) {
    double q4[4] = {0.0, 0.0, 0.0, 0.0};
    float v[16];  // at most 64 row tiles on this path: all 16 loads in flight (clamped; the excess ones add +0)
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = F.colpart_prev[(size_t)min(sub + 4 * u, F.ntr - 1) * A.np + j];
#pragma unroll
    for (int u = 0; u < 16; ++u) q4[u & 3] += (sub + 4 * u < F.ntr) ? (double)v[u] : 0.0;
    sj = (q4[0] + q4[2]) + (q4[1] + q4[3]);  // residues sub, sub+8 | sub+4, sub+12
  }
  // rows: one thread per row of the tile (threads 256 .. 287)
  const int l = t - kSegCols;
  const int i = tr * kTileRows + l;
  const bool row_thread = l >= 0 && l < kTileRows && i < A.m;
  double ri = 0.0, ai = 0.0;
  if (row_thread) {
    ri = sum_partials_16(F.rowpart_prev + i, (size_t)A.mp, F.nseg) - (double)F.p[i];
    ai = F.a_in[i];
  }
  const bool col_thread = t < kSegCols && j < A.n;
  double qj = 0.0, bj = 0.0;
  if (col_thread) {
    qj = (double)F.q[j];
    bj = F.b_in[j];
  }
  const double sum_p = *F.sum_p;
  const double theta = *F.theta_in;

  const double sum_x = block_sum_f64(acc, red);
  const double mn = (double)A.m + (double)A.n;
  const double eta = (sum_x - sum_p) / mn;
  const double cst = 2.0 * eta - theta;
  __syncthreads();  // every thread has read the wave sums of block_sum_f64
  red[t] = sj;
  __syncthreads();
  if (t < kSegCols) {
    float out = kMaskedOut;
    if (col_thread) {
      const double res = (red[t] + red[512 + t]) + (red[256 + t] + red[768 + t]) - qj;
      out = (float)((bj - 2.0 * res + cst) / (double)A.m);
      if (tr == 0) {
        F.b_out[j] = bj - res;
        F.varphi_out[j] = out;
      }
    }
    lds_varphi[t] = out;
  } else if (l < kTileRows) {
    float out = 0.f;
    if (row_thread) {
      out = (float)((ai - 2.0 * ri + cst) / (double)A.n);
      if (seg == 0) {
        F.a_out[i] = ai - ri;
        F.phi_out[i] = out;
      }
    }
    lds_phi[l] = out;
  }
  if (seg == 0 && tr == 0 && t == 0) *F.theta_out = theta - eta;
  __syncthreads();
}

template <bool FIRST, bool EDGE, bool NT, bool PRO, int MODE, int U, int NW>
__device__ __forceinline__ void sweep_body(const SweepArgs& A, const FusedUpdateArgs& F, int lane, int wave, int seg,
                                           int tr, float* __restrict__ lds_phi, float* __restrict__ lds_varphi) {
  static_assert(!PRO || (U == kSweepRows && NW == kSweepWaves), "the fused update is written for 32-row tiles");
  const int j0 = seg * kSegCols + lane * 4;
  // columns of this lane that may be accessed (the plain sums of MODE 3 have no mask: existing columns only)
  const int nmem = EDGE ? min(max((MODE == 3 ? A.n : A.n_mem) - j0, 0), 4) : 4;
  const int r0 = (tr * NW + wave) * U;  // a tile has NW * U rows
  const int nrows = min(max(A.m - r0, 0), U);
  const size_t ldx = (size_t)A.ldx, ldc = (size_t)A.ldc;
  const float* __restrict__ Cp = A.C + (size_t)r0 * ldc + j0;
  float* __restrict__ Xp = A.X + (size_t)r0 * ldx + j0;
  const float rho = A.rho, scale = A.scale;

  // X >= 0, so a row segment whose sum after the previous sweep was zero holds nothing but zeros:
  // it need not be read (lane u fetches the old sum of row r0 + u; rows read it with a scalar lane read)
  bool readx[U];
#pragma unroll
  for (int u = 0; u < U; ++u) readx[u] = true;
  if (MODE == 0 && !FIRST && !PRO && A.rowpart_prev) {
    float prev = 1.f;
    if (lane < nrows) prev = A.rowpart_prev[(size_t)seg * A.mp + r0 + lane];
#pragma unroll
    for (int u = 0; u < U; ++u)
      readx[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, prev), u)) != 0.f;
  }

  // the one batch of loads of this wave
  f4v x[U], c[U];
  if (nrows == U) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      c[u] = MODE >= 2 ? f4v{0.f, 0.f, 0.f, 0.f} : ld4<EDGE, NT>(Cp + u * ldc, nmem);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      x[u] = f4v{0.f, 0.f, 0.f, 0.f};
      if (MODE == 3) x[u] = load4(Xp + u * ldx, nmem);  // (any number of a lane's columns may exist there)
      else if (!FIRST && readx[u]) x[u] = ld4<EDGE, NT>(Xp + u * ldx, nmem);
    }
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      c[u] = f4v{0.f, 0.f, 0.f, 0.f};
      x[u] = f4v{0.f, 0.f, 0.f, 0.f};
      if (u < nrows) {
        if (MODE < 2) c[u] = ld4<EDGE, NT>(Cp + u * ldc, nmem);
        if (MODE == 3) x[u] = load4(Xp + u * ldx, nmem);
        else if (!FIRST && readx[u]) x[u] = ld4<EDGE, NT>(Xp + u * ldx, nmem);
      }
    }
  }
  // with the fused update (PRO) phi and varphi of this tile are computed into LDS while the loads fly
  if (PRO) fused_update(A, F, seg, tr, lds_phi, lds_varphi);

  f4v colacc = {0.f, 0.f, 0.f, 0.f};
  float wave_total = 0.f;
  {
    const f4v vp = PRO ? *reinterpret_cast<const f4v*>(lds_varphi + lane * 4) : load_varphi_padded(A.varphi, j0);
    // lane u holds phi of row r0 + u; rows read it back with a scalar lane read.  Rows past the end of
    // the matrix get the huge negative value: with x = c = 0 they come out as exact zeros, so the loop
    // below needs no per-row branches (only the stores are guarded).
    const float phi_lane = (lane < nrows) ? (PRO ? lds_phi[wave * U + lane] : A.phi[r0 + lane]) : kMaskedOut;
    float rowkeep = 0.f;  // lane u keeps the sum of row r0 + u
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float ph = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, phi_lane), u));
      // (in MODE 2 the stored value already carries - rho*C and c is zero)
      const f4v v = MODE == 3 ? x[u] : xbar4(x[u], c[u], vp + ph, rho) * scale;
      if (MODE == 3) {
        // sums only
      } else if (MODE == 1) {
        f4v sh;
        sh.x = fmaf(-rho, c[u].x, v.x);
        sh.y = fmaf(-rho, c[u].y, v.y);
        sh.z = fmaf(-rho, c[u].z, v.z);
        sh.w = fmaf(-rho, c[u].w, v.w);
        if (u < nrows) st4<EDGE, NT>(Xp + u * ldx, sh, nmem);
      } else if (MODE == 0 && !FIRST && !PRO) {
        // a row segment that was all zero (known from its old sum) and stays all zero is not written
        // back: plans are sparse, so once the support has settled that is nearly every segment
        const bool nonzero = ((fbits(v.x) | fbits(v.y)) | (fbits(v.z) | fbits(v.w))) != 0;
        if (u < nrows && (readx[u] || __builtin_amdgcn_ballot_w64(nonzero) != 0)) st4<EDGE, NT>(Xp + u * ldx, v, nmem);
      } else {
        if (u < nrows) st4<EDGE, NT>(Xp + u * ldx, v, nmem);
      }
      colacc += v;
      const float tot = wave_sum((v.x + v.y) + (v.z + v.w));
      rowkeep = (lane == u) ? tot : rowkeep;
      wave_total += tot;
    }
    if (lane < nrows) A.rowpart[(size_t)seg * A.mp + r0 + lane] = rowkeep;
  }
  write_col_partials<NW>(colacc, lane, wave, seg, tr, A.n, A.np, A.colpart);
  // total of the tile, for the vector update that forms eta from these
  if (A.tilesum) write_tile_total<NW>(wave_total, lane, wave, seg, tr, A.tilesum);
}

// NW waves of U rows each: 16 x 2 (32-row tiles) everywhere except the plain sweep of large problems,
// which takes 8 x 8 (64-row tiles): with most of X known to be zero that sweep is a read-only stream
// of C, which runs best with more loads in flight per wave, and the smaller workgroups let two or
// three of them share a compute unit so that one computes while another waits for memory.
template <bool FIRST, bool NT, bool PRO, int MODE = 0, int U = kSweepRows, int NW = kSweepWaves>
// (the register budget is that of 1024 threads for every NW: given more, the compiler's scheduler
// stretches live ranges until it spills)
__global__ __launch_bounds__(64 * kSweepWaves) void sweep_kernel(SweepArgs A, FusedUpdateArgs F) {
  static_assert(NW <= kSweepWaves, "launch bound");
  if (*A.done) return;
  __shared__ float lds_phi[kTileRows];
  __shared__ float lds_varphi[kSegCols];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y;
  if ((seg + 1) * kSegCols <= A.n) sweep_body<FIRST, false, NT, PRO, MODE, U, NW>(A, F, lane, wave, seg, tr, lds_phi, lds_varphi);
  else sweep_body<FIRST, true, NT, PRO, MODE, U, NW>(A, F, lane, wave, seg, tr, lds_phi, lds_varphi);
}
