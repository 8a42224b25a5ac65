// Group-lasso sweeps: the two-pass kernels and the group-resident slab kernel.
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

// ------------------------------------------------------------------------------------------
// Group lasso, general labels, two passes (Section "Group-lasso Regularized DROT": when a
// group does not fit one workgroup the reduction goes through global memory and a second
// kernel applies the scale).  Pass 1 accumulates sum_{i in class} Xbar_ij^2 per (class, column), in a
// fixed order: the rows of a class in chunks, then the chunks (the paper's kernel uses atomics here).
// ------------------------------------------------------------------------------------------
struct GroupArgs {
  SweepArgs S;
  const int* row_class;
  float* gsq;   // [num_classes][n]
  float thr;    // rho * mu
};

__device__ __forceinline__ void flush_group(float* __restrict__ g, f4v acc, int nvalid) {
  if (nvalid > 0) atomicAdd(g + 0, acc.x);
  if (nvalid > 1) atomicAdd(g + 1, acc.y);
  if (nvalid > 2) atomicAdd(g + 2, acc.z);
  if (nvalid > 3) atomicAdd(g + 3, acc.w);
}

// Pass 1: one wave adds up Xbar_ij^2 over the (at most 16) rows of one chunk of one class, for its 256
// columns, and stores the sums as row `chunk` of gpart.  grid = (nseg, ceil(nchunks / 4)).
struct ChunkArgs {
  const int* perm;         // [m] rows sorted by (class, row)
  const int* chunk_start;  // [nchunks + 1] offsets into perm
  const int* class_first;  // [num_classes + 1] first chunk of every class
  float* gpart;            // [nchunks][n]
  int nchunks;
};

template <bool FIRST>
__global__ __launch_bounds__(kBlock) void gl_norm_kernel(GroupArgs G, ChunkArgs K) {
  const SweepArgs& A = G.S;
  if (*A.done) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int chunk = blockIdx.y * kWavesPerBlock + wave;
  if (chunk >= K.nchunks) return;
  const int j0 = blockIdx.x * kSegCols + lane * 4;
  const int nvalid = min(max(A.n - j0, 0), 4);
  const f4v vp = load_varphi(A.varphi, j0, nvalid);
  const int beg = K.chunk_start[chunk], end = K.chunk_start[chunk + 1];
  f4v acc = {0.f, 0.f, 0.f, 0.f};
  for (int e = beg; e < end; ++e) {
    const int i = K.perm[e];
    const f4v c = load4(A.C + (size_t)i * A.ldc + j0, nvalid);
    const f4v x = FIRST ? f4v{0.f, 0.f, 0.f, 0.f} : load4(A.X + (size_t)i * A.ldx + j0, nvalid);
    const f4v v = xbar4(x, c, vp + A.phi[i], A.rho);
    acc += v * v;
  }
  store4(K.gpart + (size_t)chunk * A.n + j0, acc, nvalid);
}

// Between the passes: the chunks of every class added up in order, one thread per (class, column).
// grid = (ceil(n / 256), min(num_classes, 65535)).
__global__ __launch_bounds__(kBlock) void gl_norm_finish_kernel(ChunkArgs K, float* __restrict__ gsq, int n, int num_classes,
                                                                const int* done) {
  if (*done) return;
  const int j = blockIdx.x * kBlock + threadIdx.x;
  if (j >= n) return;
  for (int cls = blockIdx.y; cls < num_classes; cls += gridDim.y) {
    float t = 0.f;
    for (int k = K.class_first[cls]; k < K.class_first[cls + 1]; ++k) t += K.gpart[(size_t)k * n + j];
    gsq[(size_t)cls * n + j] = t;
  }
}

// scale of one group from its squared norm t: [1 - rho mu / sqrt(t)]_+ / (1 + rho lambda), 0 at t = 0
__device__ __forceinline__ float group_scale(float t, float thr, float qscale) {
  if (!(t > 0.f)) return 0.f;
  return fmaxf(1.f - thr / sqrtf(t), 0.f) * qscale;
}

template <bool FIRST>
__global__ __launch_bounds__(kBlock) void gl_apply_kernel(GroupArgs G) {
  const SweepArgs& A = G.S;
  if (*A.done) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y;
  const int j0 = seg * kSegCols + lane * 4;
  const int nvalid = min(max(A.n - j0, 0), 4);
  const f4v vp = load_varphi(A.varphi, j0, nvalid);
  const int rbeg = tr * kTileRows + wave * kLoopRows;
  const int rend = min(rbeg + kLoopRows, A.m);
  f4v colacc = {0.f, 0.f, 0.f, 0.f};
  float rowkeep = 0.f;
  int cur = -1;
  f4v sc = {0.f, 0.f, 0.f, 0.f};
  for (int i = rbeg; i < rend; ++i) {
    const int cls = G.row_class[i];
    if (cls != cur) {
      cur = cls;
      const f4v t = load4(G.gsq + (size_t)cls * A.n + j0, nvalid);
      sc.x = group_scale(t.x, G.thr, A.scale);
      sc.y = group_scale(t.y, G.thr, A.scale);
      sc.z = group_scale(t.z, G.thr, A.scale);
      sc.w = group_scale(t.w, G.thr, A.scale);
    }
    const f4v c = load4(A.C + (size_t)i * A.ldc + j0, nvalid);
    const f4v x = FIRST ? f4v{0.f, 0.f, 0.f, 0.f} : load4(A.X + (size_t)i * A.ldx + j0, nvalid);
    const f4v v = xbar4(x, c, vp + A.phi[i], A.rho) * sc;
    store4(A.X + (size_t)i * A.ldx + j0, v, nvalid);
    colacc += v;
    const float tot = wave_sum((v.x + v.y) + (v.z + v.w));
    rowkeep = (lane == i - rbeg) ? tot : rowkeep;
  }
  if (lane < rend - rbeg) A.rowpart[(size_t)seg * A.mp + rbeg + lane] = rowkeep;
  write_col_partials<kWavesPerBlock>(colacc, lane, wave, seg, tr, A.n, A.np, A.colpart);
}

// ------------------------------------------------------------------------------------------
// Group lasso, group-resident variant (Section "Group-lasso Regularized DROT", small-group case:
// reduce and broadcast inside one thread block).  Needs every class to be one run of rows.  A
// workgroup of 1024 threads owns one class (a run of up to 128*K consecutive rows) x 32 columns and
// keeps the whole slab of Xbar in registers: 8 lanes x 128-bit along the columns (one 128-byte line
// per row), 128 row lanes, K <= 8 rows per thread, all loads in flight at once.  Squared norms per
// column are folded through LDS, the scale is broadcast, X is stored once: 12 bytes per element like
// the plain sweep.  (Measured at 5000 x 5000, 10 classes: 46 us per sweep; 16 lanes x 64 row lanes
// with 64-column strips: 52 us.)
// Row sums: rowpart[strip][i] with 32-column strips; column sums: colpart[class run][j].
// ------------------------------------------------------------------------------------------
constexpr int kSlabThreads = 1024;
constexpr int kSlabLanes = 8;                               // lanes along the columns: strips of 32 columns
constexpr int kSlabCols = 4 * kSlabLanes;
constexpr int kSlabRowLanes = kSlabThreads / kSlabLanes;    // 128 row lanes
constexpr int kSlabMaxRows = kSlabRowLanes * 8;             // longest class the registers hold (8 rows per thread)

struct SlabArgs {
  SweepArgs S;
  const int* run_start;  // [nruns] first row of every run of equal labels
  const int* run_len;    // [nruns]
  float thr;             // rho * mu
};

// sum over the CX (8 or 16) adjacent lanes that share one matrix row; every lane gets the total
template <int CX>
__device__ __forceinline__ float rowlanes_sum(float v) {
  v += dpp_mov<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
  v += dpp_mov<0x141, 0xF>(v);  // row_half_mirror: the other quad of the 8-lane half
  if (CX == 16) v += dpp_mov<0x140, 0xF>(v);  // row_mirror: the other half of the 16-lane row
  return v;
}

// CX lanes x 128-bit along the columns (strip of 4*CX columns), 1024/CX row lanes, K rows per thread.
// PRO: the eq. (6) update of the previous sweep is computed here first (small problems), as in
// fused_update: every workgroup derives phi of the rows of its run (one thread per row) and varphi
// of its own 32 columns from the previous sweep's partial sums, in the summation order of
// reduce_kernel, and hands them to the lanes through LDS.
template <bool FIRST, int K, int CX, bool PRO>
__global__ __launch_bounds__(kSlabThreads) void gl_slab_kernel(SlabArgs G, FusedUpdateArgs F) {
  constexpr int COLS = 4 * CX, RL = kSlabThreads / CX;
  static_assert(kSlabMaxRows <= kSlabThreads, "the fused update gives every row of a run a thread");
  const SweepArgs& A = G.S;
  __shared__ float red[RL][COLS];  // 16 KiB either way
  __shared__ float part[16][COLS];
  __shared__ float bcast[COLS];
  __shared__ float lds_varphi[COLS];
  __shared__ float lds_phi[kSlabThreads];
  __shared__ double dred[kSlabThreads / 64];
  const int t = threadIdx.x;
  const int cx = t % CX, ry = t / CX;
  const int strip = blockIdx.x, run = blockIdx.y;
  // (the stop flag is asked for together with the run's place and length, one trip to memory instead of two, and
  // tested once the loads below are on their way; nothing is stored before that)
  const int stop = *A.done;
  const int start = G.run_start[run], len = G.run_len[run];
  const int j0 = strip * COLS + cx * 4;
  const int nvalid = min(max(A.n - j0, 0), 4);
  const size_t ldx = (size_t)A.ldx, ldc = (size_t)A.ldc;
  const float* __restrict__ Cp = A.C + (size_t)(start + ry) * ldc + j0;
  float* __restrict__ Xp = A.X + (size_t)(start + ry) * ldx + j0;

  f4v x[K], c[K];
  float ph[K];
  // X >= 0: a row's 32 columns of this strip (one 128-byte line, the 8 lanes of a row) are all zero
  // exactly when their sum after the previous sweep was zero; such a line is not read, and not
  // written back if it comes out as zero again (the memory contents are the same either way)
  bool held[K];
  const bool flags = !FIRST && !PRO && A.rowpart_prev != nullptr;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int r = ry + RL * k;
    held[k] = true;
    if (flags && r < len) held[k] = fbits(A.rowpart_prev[(size_t)strip * A.mp + start + r]) != 0;
  }
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int r = ry + RL * k;
    c[k] = f4v{0.f, 0.f, 0.f, 0.f};
    x[k] = f4v{0.f, 0.f, 0.f, 0.f};
    ph[k] = kMaskedOut;  // rows past the run: the clamp zeroes them
    if (r < len) {
      if (!PRO) ph[k] = A.phi[start + r];  // (first: what follows a fetch of X waits for everything asked for before it)
      c[k] = load4(Cp + (size_t)(RL * k) * ldc, nvalid);
      if (!FIRST && held[k]) x[k] = load4(Xp + (size_t)(RL * k) * ldx, nvalid);
    }
  }
  if (stop) return;
  f4v vp;
  if (PRO) {
    // ---- eq. (6) from the previous sweep's sums (F.nseg = number of strips, F.ntr = number of runs) ----
    double acc = 0.0;
    const int ntiles = F.nseg * F.ntr;
    for (int e = t; e < ntiles; e += kSlabThreads) acc += (double)F.tilesum_prev[e];
    // rows: thread t owns row t of the run; columns: the last 32 threads own the strip's columns
    const bool row_thread = t < len;
    const int i = start + t;
    double ri = 0.0, ai = 0.0;
    if (row_thread) {
      ri = sum_partials_16(F.rowpart_prev + i, (size_t)A.mp, F.nseg) - (double)F.p[i];
      ai = F.a_in[i];
    }
    const int cidx = t - (kSlabThreads - COLS);
    const int jc = strip * COLS + cidx;
    const bool col_thread = cidx >= 0 && jc < A.n;
    double sres = 0.0, bold = 0.0;
    if (col_thread) {
      sres = sum_partials_16(F.colpart_prev + jc, (size_t)A.np, F.ntr) - (double)F.q[jc];
      bold = F.b_in[jc];
    }
    const double sum_p = *F.sum_p;
    const double theta = *F.theta_in;
    const double sum_x = block_sum_f64(acc, dred);
    const double mn = (double)A.m + (double)A.n;
    const double eta = (sum_x - sum_p) / mn;
    const double cst = 2.0 * eta - theta;
    {
      float out = kMaskedOut;  // rows past the run: the clamp zeroes them
      if (row_thread) {
        out = (float)((ai - 2.0 * ri + cst) / (double)A.n);
        if (strip == 0) {
          F.a_out[i] = ai - ri;
          F.phi_out[i] = out;
        }
      }
      lds_phi[t] = out;
    }
    if (cidx >= 0) {
      float out = kMaskedOut;
      if (col_thread) {
        out = (float)((bold - 2.0 * sres + cst) / (double)A.m);
        if (run == 0) {
          F.b_out[jc] = bold - sres;
          F.varphi_out[jc] = out;
        }
      }
      lds_varphi[cidx] = out;
    }
    if (strip == 0 && run == 0 && t == 0) *F.theta_out = theta - eta;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < K; ++k) ph[k] = lds_phi[ry + RL * k];
    vp = *reinterpret_cast<const f4v*>(&lds_varphi[cx * 4]);
  } else {
    vp = load_varphi(A.varphi, j0, nvalid);
  }
  f4v sq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < K; ++k) {
    x[k] = xbar4(x[k], c[k], vp + ph[k], A.rho);
    sq += x[k] * x[k];
  }
  // Fold over the row lanes through LDS in two steps (16 threads per column, then one), fixed order.
  auto fold = [&](f4v mine) -> float {  // returns the column total in threads t < COLS
    *reinterpret_cast<f4v*>(&red[ry][cx * 4]) = mine;
    __syncthreads();
    if (t < 16 * COLS) {
      const int col = t % COLS, g = t / COLS;
      float acc = 0.f;
#pragma unroll 8
      for (int k = g; k < RL; k += 16) acc += red[k][col];
      part[g][col] = acc;
    }
    __syncthreads();
    float tot = 0.f;
    if (t < COLS) {
#pragma unroll
      for (int g = 0; g < 16; ++g) tot += part[g][t];
    }
    return tot;
  };
  const float tsum = fold(sq);
  if (t < COLS) bcast[t] = group_scale(tsum, G.thr, A.scale);
  __syncthreads();
  const f4v sc = *reinterpret_cast<const f4v*>(&bcast[cx * 4]);
  f4v colacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int r = ry + RL * k;
    const f4v v = x[k] * sc;
    const float rs = rowlanes_sum<CX>((v.x + v.y) + (v.z + v.w));
    colacc += v;
    if (r < len) {
      if (held[k] || fbits(rs) != 0) store4(Xp + (size_t)(RL * k) * ldx, v, nvalid);
      if (cx == 0) A.rowpart[(size_t)strip * A.mp + start + r] = rs;
    }
  }
  const float csum = fold(colacc);  // (the barrier inside orders it after every read of the first fold)
  if (t < COLS) {
    const int j = strip * COLS + t;
    if (j < A.n) A.colpart[(size_t)run * A.np + j] = csum;
  }
  if (A.tilesum && t < 64) {  // total of the slab, for the fused update of the next sweep (wave 0)
    const float tot = wave_sum(t < COLS ? csum : 0.f);
    if (t == 0) A.tilesum[run * gridDim.x + strip] = tot;
  }
}

// Copy of an m x n matrix between two row pitches (the caller's arrays and the padded working copies):
// 128-bit accesses that need no more than 4-byte alignment, one row of workgroups per 16 rows.
__global__ __launch_bounds__(256) void copy_rows_kernel(float* __restrict__ dst, size_t dpitch, const float* __restrict__ src,
                                                        size_t spitch, int m, int n) {
  const int j0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (j0 >= n) return;
  const int nvalid = min(n - j0, 4);
  for (int i0 = blockIdx.y * 16; i0 < m; i0 += gridDim.y * 16) {
    const int i1 = min(i0 + 16, m);
    f4v v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (i0 + u < i1) v[u] = load4(src + (size_t)(i0 + u) * spitch + j0, nvalid);
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (i0 + u < i1) store4(dst + (size_t)(i0 + u) * dpitch + j0, v[u], nvalid);
  }
}

__global__ void fill_kernel(float* __restrict__ dst, size_t count, float value, const int* done) {
  if (done && *done) return;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (size_t)gridDim.x * blockDim.x)
    dst[e] = value;
}
