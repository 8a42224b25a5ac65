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
// Packed point layouts (made once per solve by pack_points_kernel), d padded with zeros to 4 dq = 16 ceil(d/16).
// In MFMA step t lane (r, kk) supplies element k = 4t + kk of row (or column) r, so its operands for the four
// steps of a group g = t/4 are the four floats k = 16g + 4i + kk, i = 0..3: one 128-bit load.
//   source points  S[row][g][kk][i]: the four lanes of a row read 64 contiguous bytes per group; rows can be
//                  gathered in any order (the screened sweep does)
//   target points  T[cb][g][kk][r][i], cb = column / 16, r = column % 16: the 64 lanes of a wave read 1 KiB
//                  contiguous per 16-column block and group, lane kk*16 + r at offset 16 * lane bytes; columns up
//                  to the next multiple of 16 hold zeros
// (With operands strided across lanes the sweeps were bound by the tag lookups of the vector L1, not by the
// matrix cores.)
// ------------------------------------------------------------------------------------------
struct PointArgs {
  const float* xs_pack;  // S above, [m][4 dq]
  const float* xt_pack;  // T above, [ceil(n/16)][dq/4][64][4]
  const float* xs_sq;    // [m] squared norms
  const float* xt_sq;    // [n]
  int dq;
  float cost_scale;
  int ncb;               // ceil(n / 16): 16-column blocks of T
};

// One thread per point.  cols = 0: the row layout S; cols = 1: the blocked layout T.
__global__ void pack_points_kernel(const float* __restrict__ pts, int rows, int d, int dq, float* __restrict__ pack,
                                   float* __restrict__ sq, int cols) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  const int padded = cols ? (rows + 15) / 16 * 16 : rows;
  if (row >= padded) return;
  const int ng = dq / 4;
  double acc = 0.0;
  for (int k = 0; k < 4 * dq; ++k) {
    const float v = (row < rows && k < d) ? pts[(size_t)row * d + k] : 0.f;
    acc += (double)v * (double)v;
    const int g = k >> 4, i = (k >> 2) & 3, kk = k & 3;
    if (cols) pack[((((size_t)(row >> 4) * ng + g) * 4 + kk) * 16 + (row & 15)) * 4 + i] = v;
    else pack[(size_t)row * 4 * dq + (g * 4 + kk) * 4 + i] = v;
  }
  if (row < rows) sq[row] = (float)acc;
}

constexpr int kDotPitch = kSegCols + 4;  // LDS row pitch of the inner-product tile (keeps rows 16-byte aligned)

// REFRESH: the sweep also records, per row segment, the largest of varphi_j - rho C_ij, a column that attains
// it and the largest of the others, and stores its varphi as the epoch's varphi0: the bounds the screened sweep
// below certifies zero row segments with (same definition and use as in the stored-cost screening).
// mprime, mprime2, jstar: [nseg][m]; varphi0: padded like varphi.
template <bool FIRST, bool NT, bool REFRESH = false>
__global__ __launch_bounds__(64 * kSweepWaves) void sweep_points_kernel(SweepArgs A, PointArgs Pt, float* __restrict__ mprime,
                                                                        float* __restrict__ mprime2,
                                                                        unsigned char* __restrict__ jstar,
                                                                        float* __restrict__ varphi0) {
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
  if (flags && lane < nrows) prev = A.rowpart_prev[(size_t)seg * A.mp + r0 + lane];
  f4v x[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    x[u] = f4v{0.f, 0.f, 0.f, 0.f};
    if (!FIRST && !flags && u < nrows) {
      if (NT && nvalid == 4) x[u] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(Xp + u * ldx));
      else x[u] = load4(Xp + u * ldx, nvalid);
    }
  }
  const f4v vp = load_varphi_padded(A.varphi, j0);
  const f4v ysq = load4(Pt.xt_sq + j0, nvalid);
  const float phi_lane = (lane < nrows) ? A.phi[r0 + lane] : 0.f;
  const float xsq_lane = (lane < nrows) ? Pt.xs_sq[r0 + lane] : 0.f;

  // matrix phase: this wave's 16 x 32 block of inner products
  {
    const int r = lane & 15, kk = lane >> 4;
    const int R0 = (wave >> 3) * 16, cb = (wave & 7) * 32;
    const int row = tr * kTileRows + R0 + r;
    const int dq = Pt.dq, ng = dq >> 2;
    // rows / column blocks past the edge reuse the last valid one: their products are never read
    const float* __restrict__ ap = Pt.xs_pack + (size_t)min(row, A.m - 1) * 4 * dq + kk * 4;
    const int cb0 = min((seg * kSegCols + cb) >> 4, Pt.ncb - 1), cb1 = min(cb0 + 1, Pt.ncb - 1);
    const float* __restrict__ bp0 = Pt.xt_pack + ((size_t)cb0 * ng * 64 + lane) * 4;
    const float* __restrict__ bp1 = Pt.xt_pack + ((size_t)cb1 * ng * 64 + lane) * 4;
    f4v acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    for (int g = 0; g < ng; ++g) {
      const f4v a = *reinterpret_cast<const f4v*>(ap + g * 16);
      const f4v b0 = *reinterpret_cast<const f4v*>(bp0 + g * 256);
      const f4v b1 = *reinterpret_cast<const f4v*>(bp1 + g * 256);
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
  float wave_total = 0.f;  // the total of this wave's rows (the tile's total gives eta to the one-launch vector update)
  if (nrows > 0) {
    const float rho = A.rho, scale = A.scale, cs = Pt.cost_scale;
    float rowkeep = 0.f, mkeep = 0.f, m2keep = 0.f;
    int jkeep = 0;
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
        wave_total += tot;
        if (REFRESH) {  // (columns past n carry the mask value in vp: they never win the maximum)
          const f4v t = {fmaf(-rho, c.x, vp.x), fmaf(-rho, c.y, vp.y), fmaf(-rho, c.z, vp.z), fmaf(-rho, c.w, vp.w)};
          float mm, mm2;
          int jj;
          segment_top2(t, lane, mm, jj, mm2);
          mkeep = (lane == u) ? mm : mkeep;
          m2keep = (lane == u) ? mm2 : m2keep;
          jkeep = (lane == u) ? jj : jkeep;
        }
      }
    }
    if (lane < nrows) {
      A.rowpart[(size_t)seg * A.mp + r0 + lane] = rowkeep;
      if (REFRESH) {
        mprime[(size_t)seg * A.mp + r0 + lane] = mkeep;
        mprime2[(size_t)seg * A.mp + r0 + lane] = m2keep;
        jstar[(size_t)seg * A.mp + r0 + lane] = (unsigned char)jkeep;
      }
    }
  }
  if (REFRESH && tr == 0 && wave == 0) *reinterpret_cast<f4u*>(varphi0 + j0) = vp;  // (past n both hold the mask value)
  write_col_partials<kSweepWaves>(colacc, lane, wave, seg, tr, A.n, A.np, A.colpart);
  if (A.tilesum) write_tile_total<kSweepWaves>(wave_total, lane, wave, seg, tr, A.tilesum);
}

// ------------------------------------------------------------------------------------------
// The screened sweep of the point-cloud variant, for plans known to be sparse.  A row segment whose X
// is zero and whose bound max(M + drift of its own column, M2 + largest drift) + phi_i is not positive stays
// zero (the certificate of the stored-cost screening, to the letter); for the few that are left the cost has to be formed, and
// to come out with the bits of the full sweep it is formed the same way, on the matrix cores: a
// workgroup of four waves owns a strip of 256 rows x 256 columns, gathers the rows that are left (in
// ascending order) into blocks of 16, computes each block's 16 x 256 inner products with the same
// instruction sequence per element as sweep_points_kernel (an element of an MFMA result depends on its
// own row and column operands only), and then every wave updates those rows of the block that lie in
// its own 64 rows.  Sums come out as in the full sweep: rows through the same wave reduction; columns
// added up per pair of rows, the pairs of a 32-row tile in order, then the strip's eight tiles in order
// (the reduction adds the full sweep's eight rows of column sums per strip in that order first).
// grid = (nseg, ceil(m / 256)), 256 threads.
// ------------------------------------------------------------------------------------------
constexpr int kStripRows = 256;
constexpr int kPointsColGroup = kStripRows / kTileRows;  // rows of the full sweep's column sums per strip

// Which (column segment, strip) a workgroup takes.  Workgroups go to the eight XCDs in turn (linear id modulo 8),
// and each XCD has its own L2: the target points of a column segment (32 KiB at d = 32) are fetched by every strip
// of that segment, so the segments are dealt out by their number modulo 8 and an XCD keeps meeting the same ones.
// A bijection of [0, nseg x nstrips): XCD x takes a contiguous run of the pairs ordered by (seg % 8, seg / 8, strip).
__device__ __forceinline__ void xcd_strip(int nseg, int nstrips, int& seg, int& strip) {
  const int nwg = nseg * nstrips;
  const int id = blockIdx.x + gridDim.x * blockIdx.y;
  const int x = id & 7, q = id >> 3;
  // position in the ordered list: the workgroups of the XCDs before x come first (XCD x' has ceil((nwg - x') / 8))
  int pos = q;
  for (int xb = 0; xb < x; ++xb) pos += (nwg - xb + 7) >> 3;
  for (int r = 0; r < 8; ++r) {
    const int here = ((nseg - r + 7) >> 3) * nstrips;  // pairs whose segment is r modulo 8
    if (pos < here) {
      seg = r + 8 * (pos / nstrips);
      strip = pos % nstrips;
      return;
    }
    pos -= here;
  }
  seg = 0;  // (not reached: the counts add up to nwg)
  strip = 0;
}

template <bool NT>
__global__ __launch_bounds__(256, 6) void lean_points_kernel(SweepArgs A, PointArgs Pt, ScreenArgs SC) {
  __shared__ float ctile[16][kDotPitch];  // a block's costs-to-be (inner products); the column fold at the very end
  __shared__ unsigned long long masks[4];
  __shared__ unsigned char list[kStripRows];
  __shared__ float totals[kPointsColGroup];
  static_assert(sizeof(ctile) >= sizeof(float) * kPointsColGroup * kSegCols, "the column fold reuses the tile");
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int seg, strip;
  xcd_strip(gridDim.x, gridDim.y, seg, strip);
  const int j0 = seg * kSegCols + lane * 4;
  const int nvalid = min(max(A.n - j0, 0), 4);
  const int r0 = strip * kStripRows + wave * 64;  // this wave's 64 rows: lane l holds the state of row r0 + l
  const int nrows = min(max(A.m - r0, 0), 64);
  const size_t ldx = (size_t)A.ldx;
  const float rho = A.rho, scale = A.scale, cs = Pt.cost_scale;

  const f4v vp = load_varphi_padded(A.varphi, j0);
  const f4v vp0 = load_varphi_padded(SC.varphi0, j0);
  const f4v ysq = load4(Pt.xt_sq + j0, nvalid);
  float prev = 0.f, ph = kMaskedOut, mpr = 0.f, mpr2 = 0.f, xsq_lane = 0.f;
  unsigned js = 0;
  const size_t ridx = (size_t)seg * A.mp + r0 + lane;
  if (lane < nrows) {
    prev = A.rowpart_prev[ridx];
    ph = A.phi[r0 + lane];
    mpr = SC.mprime_in[ridx];
    mpr2 = SC.m2_in[ridx];
    js = SC.jstar_in[ridx];
    xsq_lane = Pt.xs_sq[r0 + lane];
  }
  // (the stop flag travels with the loads above: asked for before them, a wave would sit out its latency with
  // nothing of its own in flight; it is tested before the first store)
  __builtin_amdgcn_sched_barrier(0);
  const int stop = *A.done;
  __builtin_amdgcn_sched_barrier(0);
  const f4v dv = vp - vp0;
  const float d = fmaxf(fmaxf(dv.x, dv.y), fmaxf(dv.z, dv.w));
  const float a = fmaxf(fmaxf(unmasked_abs(vp.x), unmasked_abs(vp.y)), fmaxf(unmasked_abs(vp.z), unmasked_abs(vp.w)));
  const float delta = wave_max(d), mag = wave_max(a);
  const bool below = certified_zero(mpr, mpr2, js, dv, delta, mag, ph);  // (the certificate of screened_body)
  const bool certified = lane >= nrows || (fbits(prev) == 0 && below);
  if (stop) return;  // (the flag arrived with the loads above; nothing has been stored yet)
  const unsigned long long todo = ~__builtin_amdgcn_ballot_w64(certified);
  if (lane == 0) masks[wave] = todo;
  __syncthreads();
  int before = 0, total = 0;  // rows left in the waves before this one, and in the whole strip
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int cnt = __builtin_popcountll(masks[w]);
    before += w < wave ? cnt : 0;
    total += cnt;
  }
  if ((todo >> lane) & 1ull) list[before + __builtin_popcountll(todo & ((1ull << lane) - 1ull))] = (unsigned char)(wave * 64 + lane);
  __syncthreads();

  // the first two of this wave's rows that hold something are fetched now, ahead of the matrix phase (a wave has
  // one or two of them as a rule; any further ones are fetched when their turn comes)
  const unsigned long long xmask = todo & __builtin_amdgcn_ballot_w64(fbits(prev) != 0);
  const int u0 = xmask ? __builtin_ctzll(xmask) : -1;
  const unsigned long long xrest = xmask & (xmask - 1ull);
  const int u1 = xrest ? __builtin_ctzll(xrest) : -1;
  f4v xpre0 = {0.f, 0.f, 0.f, 0.f}, xpre1 = {0.f, 0.f, 0.f, 0.f};
  if (u0 >= 0) {
    const float* __restrict__ Xq = A.X + (size_t)(r0 + u0) * ldx + j0;
    if (NT && nvalid == 4) xpre0 = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(Xq));
    else xpre0 = load4(Xq, nvalid);
  }
  if (u1 >= 0) {
    const float* __restrict__ Xq = A.X + (size_t)(r0 + u1) * ldx + j0;
    if (NT && nvalid == 4) xpre1 = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(Xq));
    else xpre1 = load4(Xq, nvalid);
  }
  f4v tile_acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, pair_acc = {0.f, 0.f, 0.f, 0.f};
  float tile_tot[2] = {0.f, 0.f}, pair_tot = 0.f;  // the totals, added up as the full sweep adds them: rows of a pair, pairs of a tile
  int cur_pair = -1;  // pair of rows (0 .. 31 within this wave's 64 rows) pair_acc belongs to
  float rowkeep = 0.f;
  for (int b0 = 0; b0 < total; b0 += 16) {
    {  // matrix phase: this wave's 16 x 64 share of the block's inner products (four 16 x 16 results)
      const int r = lane & 15, kk = lane >> 4;
      const int local = list[min(b0 + r, total - 1)];  // (slots past the end repeat the last row: never read back)
      const int row = strip * kStripRows + local;
      const int dq = Pt.dq, ng = dq >> 2;
      const float* __restrict__ ap = Pt.xs_pack + (size_t)row * 4 * dq + kk * 4;
      // (two column blocks at a time: half the registers, and occupancy is what hides this kernel's trips to memory)
#pragma unroll 1
      for (int half = 0; half < 2; ++half) {
        const float* __restrict__ bp[2];
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
          const int cb = min(seg * (kSegCols / 16) + 4 * wave + 2 * half + cbi, Pt.ncb - 1);  // (past the edge: never read back)
          bp[cbi] = Pt.xt_pack + ((size_t)cb * ng * 64 + lane) * 4;
        }
        f4v acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        for (int gq = 0; gq < ng; ++gq) {
          const f4v av = *reinterpret_cast<const f4v*>(ap + gq * 16);
          f4v bv[2];
#pragma unroll
          for (int cbi = 0; cbi < 2; ++cbi) bv[cbi] = *reinterpret_cast<const f4v*>(bp[cbi] + gq * 256);
#pragma unroll
          for (int cbi = 0; cbi < 2; ++cbi) acc[cbi] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv[cbi].x, acc[cbi], 0, 0, 0);
#pragma unroll
          for (int cbi = 0; cbi < 2; ++cbi) acc[cbi] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv[cbi].y, acc[cbi], 0, 0, 0);
#pragma unroll
          for (int cbi = 0; cbi < 2; ++cbi) acc[cbi] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bv[cbi].z, acc[cbi], 0, 0, 0);
#pragma unroll
          for (int cbi = 0; cbi < 2; ++cbi) acc[cbi] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bv[cbi].w, acc[cbi], 0, 0, 0);
        }
        // accumulator i of lane (r, kk) is element (row 4*kk + i, column r) of the 16 x 16 result
#pragma unroll
        for (int cbi = 0; cbi < 2; ++cbi) {
          const int col = (4 * wave + 2 * half + cbi) * 16 + r;
          ctile[4 * kk + 0][col] = acc[cbi].x;
          ctile[4 * kk + 1][col] = acc[cbi].y;
          ctile[4 * kk + 2][col] = acc[cbi].z;
          ctile[4 * kk + 3][col] = acc[cbi].w;
        }
      }
    }
    __syncthreads();
    // sweep phase: the rows of the block that lie in this wave's 64 rows, in ascending order
    const int bend = min(b0 + 16, total);
    for (int g = b0; g < bend; ++g) {
      const int local = __builtin_amdgcn_readfirstlane((int)list[g]);
      if ((local >> 6) != wave) continue;
      const int u = local & 63;
      const float phu = __builtin_bit_cast(float, __builtin_amdgcn_readlane(fbits(ph), u));
      const float xsq = __builtin_bit_cast(float, __builtin_amdgcn_readlane(fbits(xsq_lane), u));
      const bool readx = __builtin_amdgcn_readlane(fbits(prev), u) != 0;
      float* __restrict__ Xp = A.X + (size_t)(r0 + u) * ldx + j0;
      f4v x = {0.f, 0.f, 0.f, 0.f};
      if (u == u0) x = xpre0;
      else if (u == u1) x = xpre1;
      else if (readx) {
        if (NT && nvalid == 4) x = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(Xp));
        else x = load4(Xp, nvalid);
      }
      const f4v dv = *reinterpret_cast<const f4v*>(&ctile[g - b0][lane * 4]);
      f4v c;
      c.x = cs * fmaxf(fmaf(-2.f, dv.x, xsq + ysq.x), 0.f);
      c.y = cs * fmaxf(fmaf(-2.f, dv.y, xsq + ysq.y), 0.f);
      c.z = cs * fmaxf(fmaf(-2.f, dv.z, xsq + ysq.z), 0.f);
      c.w = cs * fmaxf(fmaf(-2.f, dv.w, xsq + ysq.w), 0.f);
      const f4v v = xbar4(x, c, vp + phu, rho) * scale;
      const bool nonzero = ((fbits(v.x) | fbits(v.y)) | (fbits(v.z) | fbits(v.w))) != 0;
      if (readx || __builtin_amdgcn_ballot_w64(nonzero) != 0) {
        if (NT && nvalid == 4) __builtin_nontemporal_store(v, reinterpret_cast<f4u*>(Xp));
        else store4(Xp, v, nvalid);
      }
      if ((u >> 1) != cur_pair) {  // a new pair of rows: the finished one joins its tile's sum
        if (cur_pair >= 0) {
          tile_acc[cur_pair >> 4] += pair_acc;
          tile_tot[cur_pair >> 4] += pair_tot;
        }
        pair_acc = f4v{0.f, 0.f, 0.f, 0.f};
        pair_tot = 0.f;
        cur_pair = u >> 1;
      }
      pair_acc += v;
      const float tot = wave_sum((v.x + v.y) + (v.z + v.w));
      pair_tot += tot;
      rowkeep = (lane == u) ? tot : rowkeep;
    }
    __syncthreads();  // (the tile is overwritten by the next block, and by the fold below)
  }
  if (cur_pair >= 0) {
    tile_acc[cur_pair >> 4] += pair_acc;
    tile_tot[cur_pair >> 4] += pair_tot;
  }
  // (the sums are kept in place: a row segment certified to stay all zero has a zero there already)
  if (lane < nrows && !certified) A.rowpart[ridx] = rowkeep;
  if (threadIdx.x == 0) SC.wg_reads[strip * gridDim.x + seg] = total;  // (row segments whose cost was formed)
  // the strip's column sums: its eight 32-row tiles in order
  float* __restrict__ fold = &ctile[0][0];
  *reinterpret_cast<f4v*>(fold + (2 * wave + 0) * kSegCols + lane * 4) = tile_acc[0];
  *reinterpret_cast<f4v*>(fold + (2 * wave + 1) * kSegCols + lane * 4) = tile_acc[1];
  if (lane == 0) {
    totals[2 * wave + 0] = tile_tot[0];
    totals[2 * wave + 1] = tile_tot[1];
  }
  __syncthreads();
  if (A.tilesum && threadIdx.x == 0) {  // the strip's total: its eight tiles in order
    float tot = totals[0];
#pragma unroll
    for (int k = 1; k < kPointsColGroup; ++k) tot += totals[k];
    A.tilesum[strip * gridDim.x + seg] = tot;
  }
  const int t = threadIdx.x, j = seg * kSegCols + t;
  if (j < A.n) {
    float sum = fold[t];
#pragma unroll
    for (int k = 1; k < kPointsColGroup; ++k) sum += fold[k * kSegCols + t];
    A.colpart[(size_t)strip * A.np + j] = sum;
  }
}

// The same cost for the kernels off the hot path (gap evaluation): plain fp32 FMAs over the packed points.
__device__ __forceinline__ f4v cost4_from_points(const PointArgs& Pt, int i, int j0, int nvalid) {
  f4v c = {0.f, 0.f, 0.f, 0.f};
  const float xsq = Pt.xs_sq[i];
  const int ng = Pt.dq >> 2;
  const float* __restrict__ a = Pt.xs_pack + (size_t)i * 4 * Pt.dq;
  float out[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < 4; ++k) {
    if (k < nvalid) {
      const int col = j0 + k;
      const float* __restrict__ b = Pt.xt_pack + ((size_t)(col >> 4) * ng * 64 + (col & 15)) * 4;
      float dot = 0.f;
      for (int g = 0; g < ng; ++g)
        for (int kk = 0; kk < 4; ++kk)
          for (int e = 0; e < 4; ++e) dot = fmaf(a[(g * 4 + kk) * 4 + e], b[(g * 64 + kk * 16) * 4 + e], dot);
      out[k] = Pt.cost_scale * fmaxf(fmaf(-2.f, dot, xsq + Pt.xt_sq[col]), 0.f);
    }
  }
  c.x = out[0]; c.y = out[1]; c.z = out[2]; c.w = out[3];
  return c;
}
