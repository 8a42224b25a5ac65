// Sweep with the cost recomputed from two point clouds on the matrix cores.
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

// ------------------------------------------------------------------------------------------
// On-the-fly cost: C_ij = cost_scale * ||xs_i - xt_j||^2 recomputed from the two point clouds in
// every sweep instead of being read (8 bytes per element of HBM traffic instead of 12, plus
// 2d flops per element).  The inner products xs_i . xt_j of a 32 x 256 tile are a dense
// contraction, so they go to the matrix cores: each of the 16 waves forms a 16 x 32 block with
// v_mfma_f32_16x16x4_f32 (fp32 in, fp32 accumulate), writes it to LDS, and after a barrier every
// wave reads its two row segments back in the sweep's own layout (4 columns per lane), turns them
// into costs with the precomputed squared norms and proceeds exactly as the stored-cost sweep.
// The loads of X are issued before the matrix phase so that their latency is hidden behind it.
//
// Packed point layout (made once per solve by pack_points_kernel): P[row][kk][t] = pts[row][4t + kk],
// kk = 0..3, t = 0..dq-1 with dq = ceil(d/16)*4 (zero padded): in MFMA step t lane (r, kk) needs
// element k = 4t + kk of row r, so its operands for 4 consecutive steps are one 128-bit load.
// ------------------------------------------------------------------------------------------
struct PointArgs {
  const float* xs_pack;  // [m][4][dq]
  const float* xt_pack;  // [n][4][dq]
  const float* xs_sq;    // [m] squared norms
  const float* xt_sq;    // [n]
  int dq;
  float cost_scale;
};

__global__ void pack_points_kernel(const float* __restrict__ pts, int rows, int d, int dq, float* __restrict__ pack,
                                   float* __restrict__ sq) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= rows) return;
  double acc = 0.0;
  for (int k = 0; k < 4 * dq; ++k) {
    const float v = k < d ? pts[(size_t)row * d + k] : 0.f;
    acc += (double)v * (double)v;
    pack[((size_t)row * 4 + (k & 3)) * dq + (k >> 2)] = v;
  }
  sq[row] = (float)acc;
}

constexpr int kDotPitch = kSegCols + 4;  // LDS row pitch of the inner-product tile (keeps rows 16-byte aligned)

template <bool FIRST, bool NT>
__global__ __launch_bounds__(64 * kSweepWaves) void sweep_points_kernel(SweepArgs A, PointArgs Pt) {
  if (*A.done) return;
  __shared__ float dots[kTileRows][kDotPitch];
  constexpr int U = kSweepRows;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y;
  const int j0 = seg * kSegCols + lane * 4;
  const int nvalid = min(max(A.n - j0, 0), 4);
  const int r0 = tr * kTileRows + wave * U;
  const int nrows = min(max(A.m - r0, 0), U);
  const size_t ldx = (size_t)A.ldx;
  float* __restrict__ Xp = A.X + (size_t)r0 * ldx + j0;

  // sweep layout: start the loads of X and of the per-row / per-column vectors.  With the old row
  // sums at hand (X >= 0: a zero sum is an all-zero segment) the flags are fetched here and the few
  // segments of X that hold something after the matrix phase, which hides the flags' latency.
  const bool flags = !FIRST && A.rowpart_prev != nullptr;
  float prev = 1.f;
  if (flags && lane < nrows) prev = A.rowpart_prev[(size_t)seg * A.m + r0 + lane];
  f4v x[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    x[u] = f4v{0.f, 0.f, 0.f, 0.f};
    if (!FIRST && !flags && u < nrows) {
      if (NT && nvalid == 4) x[u] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(Xp + u * ldx));
      else x[u] = load4(Xp + u * ldx, nvalid);
    }
  }
  const f4v vp = load_varphi(A.varphi, j0, nvalid);
  const f4v ysq = load4(Pt.xt_sq + j0, nvalid);
  const float phi_lane = (lane < nrows) ? A.phi[r0 + lane] : 0.f;
  const float xsq_lane = (lane < nrows) ? Pt.xs_sq[r0 + lane] : 0.f;

  // matrix phase: this wave's 16 x 32 block of inner products
  {
    const int r = lane & 15, kk = lane >> 4;
    const int R0 = (wave >> 3) * 16, cb = (wave & 7) * 32;
    const int row = tr * kTileRows + R0 + r;
    const int col0 = seg * kSegCols + cb + r, col1 = col0 + 16;
    const int dq = Pt.dq;
    const float* __restrict__ ap = Pt.xs_pack + ((size_t)min(row, A.m - 1) * 4 + kk) * dq;
    const float* __restrict__ bp0 = Pt.xt_pack + ((size_t)min(col0, A.n - 1) * 4 + kk) * dq;
    const float* __restrict__ bp1 = Pt.xt_pack + ((size_t)min(col1, A.n - 1) * 4 + kk) * dq;
    f4v acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    for (int t = 0; t < dq; t += 4) {
      // rows / columns past the edge reuse the last valid one: their products are never read
      const f4v a = *reinterpret_cast<const f4v*>(ap + t);
      const f4v b0 = *reinterpret_cast<const f4v*>(bp0 + t);
      const f4v b1 = *reinterpret_cast<const f4v*>(bp1 + t);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b0.x, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b1.x, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b0.y, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b1.y, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b0.z, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b1.z, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b0.w, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b1.w, acc1, 0, 0, 0);
    }
    // accumulator i of lane (r, kk) is element (row 4*kk + i, column r) of the 16 x 16 block
    dots[R0 + 4 * kk + 0][cb + r] = acc0.x;
    dots[R0 + 4 * kk + 1][cb + r] = acc0.y;
    dots[R0 + 4 * kk + 2][cb + r] = acc0.z;
    dots[R0 + 4 * kk + 3][cb + r] = acc0.w;
    dots[R0 + 4 * kk + 0][cb + 16 + r] = acc1.x;
    dots[R0 + 4 * kk + 1][cb + 16 + r] = acc1.y;
    dots[R0 + 4 * kk + 2][cb + 16 + r] = acc1.z;
    dots[R0 + 4 * kk + 3][cb + 16 + r] = acc1.w;
  }
  bool readx[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    readx[u] = __builtin_amdgcn_readlane(fbits(prev), u) != 0;
    if (flags && u < nrows && readx[u]) {
      if (NT && nvalid == 4) x[u] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(Xp + u * ldx));
      else x[u] = load4(Xp + u * ldx, nvalid);
    }
  }
  __syncthreads();

  // sweep phase, as in sweep_body with the cost taken from the tile of inner products
  f4v colacc = {0.f, 0.f, 0.f, 0.f};
  if (nrows > 0) {
    const float rho = A.rho, scale = A.scale, cs = Pt.cost_scale;
    float rowkeep = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u < nrows) {
        const float ph = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, phi_lane), u));
        const float xsq = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, xsq_lane), u));
        const f4v dv = *reinterpret_cast<const f4v*>(&dots[wave * U + u][lane * 4]);
        f4v c;
        c.x = cs * fmaxf(fmaf(-2.f, dv.x, xsq + ysq.x), 0.f);
        c.y = cs * fmaxf(fmaf(-2.f, dv.y, xsq + ysq.y), 0.f);
        c.z = cs * fmaxf(fmaf(-2.f, dv.z, xsq + ysq.z), 0.f);
        c.w = cs * fmaxf(fmaf(-2.f, dv.w, xsq + ysq.w), 0.f);
        const f4v v = xbar4(x[u], c, vp + ph, rho) * scale;
        // (a segment that was all zero and comes out all zero again is not written back)
        const bool nonzero = ((fbits(v.x) | fbits(v.y)) | (fbits(v.z) | fbits(v.w))) != 0;
        if (readx[u] || __builtin_amdgcn_ballot_w64(nonzero) != 0) {
          if (NT && nvalid == 4) __builtin_nontemporal_store(v, reinterpret_cast<f4u*>(Xp + u * ldx));
          else store4(Xp + u * ldx, v, nvalid);
        }
        colacc += v;
        const float tot = wave_sum((v.x + v.y) + (v.z + v.w));
        rowkeep = (lane == u) ? tot : rowkeep;
      }
    }
    if (lane < nrows) A.rowpart[(size_t)seg * A.m + r0 + lane] = rowkeep;
  }
  write_col_partials<kSweepWaves>(colacc, lane, wave, seg, tr, A.n, A.colpart);
}

// The same cost for the kernels off the hot path (gap evaluation): plain fp32 FMAs over the packed points.
__device__ __forceinline__ f4v cost4_from_points(const PointArgs& Pt, int i, int j0, int nvalid) {
  f4v c = {0.f, 0.f, 0.f, 0.f};
  const float xsq = Pt.xs_sq[i];
  const float* __restrict__ a = Pt.xs_pack + (size_t)i * 4 * Pt.dq;
  float out[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < 4; ++k) {
    if (k < nvalid) {
      const float* __restrict__ b = Pt.xt_pack + (size_t)(j0 + k) * 4 * Pt.dq;
      float dot = 0.f;
      for (int e = 0; e < 4 * Pt.dq; ++e) dot = fmaf(a[e], b[e], dot);
      out[k] = Pt.cost_scale * fmaxf(fmaf(-2.f, dot, xsq + Pt.xt_sq[j0 + k]), 0.f);
    }
  }
  c.x = out[0]; c.y = out[1]; c.z = out[2]; c.w = out[3];
  return c;
}
