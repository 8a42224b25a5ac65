// Screened sweeps: the 8-wave tile and the lean one-wave-per-tile kernel.
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

// ------------------------------------------------------------------------------------------
// Screened sweep (large sparse problems).  On top of skipping the all-zero row segments of X, most
// of C need not be read either: a row segment with x = 0 comes out as zero again whenever
// phi_i + varphi_j - rho C_ij <= 0 for its 256 columns, and that can be certified from three numbers.
// A "refresh" sweep, which reads all of C, records for every row segment, with t_j = varphi0_j - rho C_ij
// (varphi0 = the varphi of that sweep),
//     M  = max_j t_j,   j* = a column that attains it,   M2 = max_{j != j*} t_j.
// Later sweeps form, per column segment, the drifts d_j = varphi_j - varphi0_j and delta = max_j d_j.
// Column j* has moved by exactly d_j*, every other column by at most delta, so
//     max_j ( phi_i + varphi_j - rho C_ij )  <=  max( M + d_j*, M2 + delta ) + phi_i  =:  S.
// If S plus a rounding margin is <= 0 and the segment of X is zero, the segment stays zero: its C is
// not read, nothing is computed, its row sum is 0.  The result is the one the plain sweep would
// produce (the margin dominates the handful of fp32 roundings between the two evaluations).  The
// row's own maximiser is what comes close to zero first, and it is tracked exactly; the second
// largest lies far enough below it, as a rule, for the cruder term to stay harmless ten times longer
// than M + delta alone would.  Still, as varphi drifts away from varphi0 fewer segments certify, so the
// bounds are renewed now and then: on the host's schedule while this kernel is in use, on the
// device's own in the lean kernel below.
// Tiles: 8 waves x 8 rows x 256 columns, as the unscreened sweep for sparse plans.
// ------------------------------------------------------------------------------------------
struct ScreenArgs {
  const float* mprime_in;   // [nseg][m] M of the current epoch (screening sweeps)
  float* mprime_out;        // [nseg][m] written by a refresh sweep
  const float* varphi0;     // [n] varphi of the epoch
  int* wave_reads;          // 8-wave tiles, profiling only (else null): [workgroup][wave] row segments of C this wave read
  float* varphi0_out;       // [n] written by a refresh sweep, and by the lean sweep when it renews its bounds
  // lean sweep only: it renews the bounds by itself when the vector update before it has raised ctl[0]
  const int* ctl;           // the control words below (kCtlRenew ...)
  int* wg_reads;            // [workgroup] row segments of C the workgroup read (always written)
  // lean sweep only: which of the eight 128-byte lines of a row segment of X hold a nonzero
  const unsigned char* lines_in;  // [nseg][m] as left by the previous sweep if that was a lean one, else null
  unsigned char* lines_out;       // [nseg][m]
  // the rest of the bounds: M2 and j* (column within the segment), read and written like mprime
  const float* m2_in;
  float* m2_out;
  const unsigned char* jstar_in;
  unsigned char* jstar_out;
};

// What a refresh records for one row segment from the wave's 256 values t (four per lane): the largest, a
// column that attains it (0 .. 255), and the largest of the others.  All three wave-uniform.
__device__ __forceinline__ void segment_top2(f4v t, int lane, float& M, int& jstar, float& M2) {
  // within the lane: largest, its position, largest of the other three
  const float hi01 = fmaxf(t.x, t.y), lo01 = fminf(t.x, t.y), hi23 = fmaxf(t.z, t.w), lo23 = fminf(t.z, t.w);
  const float m1 = fmaxf(hi01, hi23);
  const int a = m1 == t.x ? 0 : m1 == t.y ? 1 : m1 == t.z ? 2 : 3;
  const float m2l = a < 2 ? fmaxf(lo01, hi23) : fmaxf(hi01, lo23);
  M = wave_max(m1);
  const unsigned long long hit = __builtin_amdgcn_ballot_w64(m1 == M);
  const int L = hit ? (int)__builtin_ctzll(hit) : 0;
  jstar = L * 4 + __builtin_amdgcn_readlane(a, L);
  M2 = wave_max(lane == L ? m2l : m1);  // (a tie between lanes leaves M2 = M)
}

// The certificate, evaluated by lane l for row l from its record (m1, m2, j) and phi_l; dv: this lane's
// four drifts; delta, mag: their maximum over the wave and the largest |varphi_j| of the segment.  Each of
// the two candidates carries its own margin, 8 units in the last place of its terms (2^-21), which covers
// the roundings of the record, of the drifts, of the sums here and of the sweep's own evaluation (each at
// most half a unit of a term no larger than these); so does the last sum.
__device__ __forceinline__ bool certified_zero(float m1, float m2, unsigned j, f4v dv, float delta, float mag, float ph) {
  constexpr float kEps = 4.76837158e-7f;  // 2^-21
  // the drift of the row's own maximiser: lane j / 4, component j % 4
  const int src = (int)(j >> 2) << 2;
  const float d0 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, fbits(dv.x)));
  const float d1 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, fbits(dv.y)));
  const float d2 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, fbits(dv.z)));
  const float d3 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, fbits(dv.w)));
  const unsigned c = j & 3u;
  const float dstar = c == 0 ? d0 : c == 1 ? d1 : c == 2 ? d2 : d3;
  if (m1 == -INFINITY) return true;  // every pair of the segment is forbidden
  const float s1 = (m1 + dstar) + kEps * (fabsf(m1) + fabsf(dstar));
  const float s2 = m2 == -INFINITY ? -INFINITY : (m2 + delta) + kEps * (fabsf(m2) + fabsf(delta));
  const float bound = fmaxf(s1, s2) + ph;
  return bound + kEps * (fabsf(ph) + mag + fabsf(bound)) <= 0.f;
}

// Control words of the lean sweep's own refresh schedule (device memory, updated by
// reduce_update_kernel after every lean sweep): the classic rent-or-buy rule.  Reading the C of a
// row segment the bounds fail to certify is the rent, renewing the bounds (all of C once) the
// purchase: renew when the rent paid since the last renewal, counted from the level right after
// it, has reached the price.  That stays within a factor 2 of the best schedule in hindsight,
// whatever the drift of varphi does, and needs no model of it.
constexpr int kCtlRenew = 0;   // the next lean sweep renews the bounds
constexpr int kCtlSince = 1;   // lean sweeps since the last renewal
constexpr int kCtlFloor = 2;   // row segments of C read by the first sweep after it (-1: not known yet)
constexpr int kCtlPaid = 3;    // reads above that floor accumulated since
constexpr int kCtlWords = 4;

constexpr int kScreenRows = 8, kScreenWaves = 8;

template <bool EDGE, bool NT, bool REFRESH>
__device__ __forceinline__ void screened_body(const SweepArgs& A, const ScreenArgs& SC, int lane, int wave, int seg, int tr) {
  constexpr int U = kScreenRows, NW = kScreenWaves;
  const int j0 = seg * kSegCols + lane * 4;
  const int nmem = EDGE ? min(max(A.n_mem - j0, 0), 4) : 4;
  const int r0 = (tr * NW + wave) * U;
  const int nrows = min(max(A.m - r0, 0), U);
  const size_t ldx = (size_t)A.ldx, ldc = (size_t)A.ldc;
  const float* __restrict__ Cp = A.C + (size_t)r0 * ldc + j0;
  float* __restrict__ Xp = A.X + (size_t)r0 * ldx + j0;
  const float rho = A.rho, scale = A.scale;
  const size_t ridx = (size_t)seg * A.mp + r0 + lane;  // this lane's row in the per-row-segment arrays (lane < nrows)

  // lane u: old sum, phi and the bounds of row r0 + u
  const f4v vp = load_varphi_padded(A.varphi, j0);
  float prev = 0.f, ph = kMaskedOut, mpr = 0.f, mpr2 = 0.f;
  unsigned js = 0;
  if (lane < nrows) {
    prev = A.rowpart_prev ? A.rowpart_prev[ridx] : 1.f;
    ph = A.phi[r0 + lane];
    if (!REFRESH) {
      mpr = SC.mprime_in[ridx];
      mpr2 = SC.m2_in[ridx];
      js = SC.jstar_in[ridx];
    }
  }
  bool certified = lane >= nrows;  // rows past the end of the matrix: nothing to do
  if (!REFRESH) {
    const f4v vp0 = load_varphi_padded(SC.varphi0, j0);
    // drift of varphi since the epoch and its magnitude over this wave's columns (columns past n: both
    // carry the same mask value, their difference is 0; they are left out of the magnitude)
    const f4v dv = vp - vp0;
    const float d = fmaxf(fmaxf(dv.x, dv.y), fmaxf(dv.z, dv.w));
    const float a = fmaxf(fmaxf(unmasked_abs(vp.x), unmasked_abs(vp.y)), fmaxf(unmasked_abs(vp.z), unmasked_abs(vp.w)));
    const float delta = wave_max(d), mag = wave_max(a);
    const bool below = certified_zero(mpr, mpr2, js, dv, delta, mag, ph);
    certified = certified || (fbits(prev) == 0 && below);
  }
  const unsigned skipmask = (unsigned)__builtin_amdgcn_ballot_w64(certified) & 0xffu;
  const unsigned nzmask = (unsigned)__builtin_amdgcn_ballot_w64(fbits(prev) != 0) & 0xffu;
  if (REFRESH && tr == 0 && wave == 0) {
    // the first wave of every column segment stores the varphi the new bounds are recorded against
    // (here, behind the stop flag, so that bounds and epoch always belong together; nobody reads
    // varphi0 in a refresh sweep)
    *reinterpret_cast<f4u*>(SC.varphi0_out + j0) = vp;  // (past n both buffers hold the mask value)
  }

  f4v x[U], c[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    x[u] = f4v{0.f, 0.f, 0.f, 0.f};
    c[u] = f4v{0.f, 0.f, 0.f, 0.f};
  }
  if (nrows == U && skipmask == 0) {
    // nothing certified (always so in a refresh sweep, and while the plan is dense): straight-line loads
#pragma unroll
    for (int u = 0; u < U; ++u) c[u] = ld4<EDGE, NT>(Cp + u * ldc, nmem);
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (!((skipmask >> u) & 1)) c[u] = ld4<EDGE, NT>(Cp + u * ldc, nmem);
  }
  if (nzmask != 0) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if ((nzmask >> u) & 1) x[u] = ld4<EDGE, NT>(Xp + u * ldx, nmem);
  }

  f4v colacc = {0.f, 0.f, 0.f, 0.f};
  float rowkeep = 0.f, mkeep = 0.f, m2keep = 0.f, wave_total = 0.f;
  int jkeep = 0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (!((skipmask >> u) & 1)) {
      const float phu = __builtin_bit_cast(float, __builtin_amdgcn_readlane(fbits(ph), u));
      const f4v v = xbar4(x[u], c[u], vp + phu, rho) * scale;
      const bool nonzero = ((fbits(v.x) | fbits(v.y)) | (fbits(v.z) | fbits(v.w))) != 0;
      if (((nzmask >> u) & 1) || __builtin_amdgcn_ballot_w64(nonzero) != 0) st4<EDGE, NT>(Xp + u * ldx, v, nmem);
      colacc += v;
      const float tot = wave_sum((v.x + v.y) + (v.z + v.w));
      rowkeep = (lane == u) ? tot : rowkeep;
      wave_total += tot;
      if (REFRESH) {  // (columns past n carry the mask value in vp: they never win)
        const f4v t = {fmaf(-rho, c[u].x, vp.x), fmaf(-rho, c[u].y, vp.y), fmaf(-rho, c[u].z, vp.z), fmaf(-rho, c[u].w, vp.w)};
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
    A.rowpart[ridx] = rowkeep;
    if (REFRESH) {
      SC.mprime_out[ridx] = mkeep;
      SC.m2_out[ridx] = m2keep;
      SC.jstar_out[ridx] = (unsigned char)jkeep;
    }
  }
  if (SC.wave_reads && lane == 0)
    SC.wave_reads[(tr * gridDim.x + seg) * NW + wave] = __builtin_popcount(~skipmask & 0xffu);
  write_col_partials<NW>(colacc, lane, wave, seg, tr, A.n, A.np, A.colpart);
  write_tile_total<NW>(wave_total, lane, wave, seg, tr, A.tilesum);
}

// Profiling: total of `count` per-wave or per-workgroup counters (ints or doubles) into one double.
template <typename T>
__global__ __launch_bounds__(1024) void sum_counts_kernel(const T* __restrict__ counts, int count, double* out) {
  __shared__ double red[1024 / 64];
  double acc = 0.0;
  for (int e = threadIdx.x; e < count; e += 1024) acc += (double)counts[e];
  const double tot = block_sum_f64(acc, red);
  if (threadIdx.x == 0) *out = tot;
}

template <bool NT, bool REFRESH>
__global__ __launch_bounds__(64 * kSweepWaves) void screened_sweep_kernel(SweepArgs A, ScreenArgs SC) {
  if (*A.done) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y;
  if ((seg + 1) * kSegCols <= A.n) screened_body<false, NT, REFRESH>(A, SC, lane, wave, seg, tr);
  else screened_body<true, NT, REFRESH>(A, SC, lane, wave, seg, tr);
}

// The screened sweep for plans known to be sparse (a few percent of the row segments left to
// process): one wave owns a whole 64 x 256 tile, lane l holding the line flags, phi and the bounds of row l.
// It decides all 64 rows at once and then walks through the rows left over, three at a time (their
// loads overlap; the arithmetic stays in row order).  The waves of a workgroup work on their own
// and meet once, at the end (screened_lean_kernel).  8 times fewer waves than the tile of 8 waves x
// 8 rows, and the same bits: the rows of every group of 8 are added up in order and the 8 groups in
// order, which is what that tile's waves and its LDS fold do (rows and groups that contribute
// nothing add +0).  Returns the tile's column sums; tile_total: its total, added up the same way;
// reads: how many row segments of C it fetched.
template <bool EDGE, bool NT>
__device__ __forceinline__ f4v screened_lean_body(const SweepArgs& A, const ScreenArgs& SC, int lane, int seg, int tr,
                                                  int& stop, float& tile_total, int& reads) {
  const int j0 = seg * kSegCols + lane * 4;
  const int nmem = EDGE ? min(max(A.n_mem - j0, 0), 4) : 4;
  const int r0 = tr * 64;
  const int nrows = min(A.m - r0, 64);
  const size_t ldx = (size_t)A.ldx, ldc = (size_t)A.ldc;
  const float* __restrict__ Cp = A.C + (size_t)r0 * ldc + j0;
  float* __restrict__ Xp = A.X + (size_t)r0 * ldx + j0;
  const float rho = A.rho, scale = A.scale;
  const size_t ridx = (size_t)seg * A.mp + r0 + lane;

  const f4v vp = load_varphi_padded(A.varphi, j0);
  const f4v vp0 = load_varphi_padded(SC.varphi0, j0);
  float ph = kMaskedOut, mpr = 0.f, mpr2 = 0.f;
  unsigned js = 0;
  // lane u: the lines of row u's segment of X that hold a nonzero (bit g: columns 32g .. 32g+31).  From
  // the flags the previous lean sweep left; after any other sweep from the row sums (nonzero sum:
  // any line may hold something)
  unsigned oldlines = 0;
  if (lane < nrows) {
    ph = A.phi[r0 + lane];
    mpr = SC.mprime_in[ridx];
    mpr2 = SC.m2_in[ridx];
    js = SC.jstar_in[ridx];
    if (SC.lines_in) oldlines = SC.lines_in[ridx];
    else oldlines = (A.rowpart_prev == nullptr || fbits(A.rowpart_prev[ridx]) != 0) ? 0xffu : 0u;
  }
  // The stop flag and the renewal word travel with the loads above (asked for before them, a wave would
  // sit out their latency with nothing of its own in flight); both are tested before the first store.
  __builtin_amdgcn_sched_barrier(0);
  stop = *A.done;
  const bool renew = SC.ctl[kCtlRenew] != 0;
  __builtin_amdgcn_sched_barrier(0);
  // (renew, wave-uniform: this sweep records new bounds against the varphi of now; it certifies
  // nothing, walks through all its rows and takes the maximum of varphi_j - rho C_ij of each)
  const f4v dv = vp - vp0;
  const float d = fmaxf(fmaxf(dv.x, dv.y), fmaxf(dv.z, dv.w));
  const float a = fmaxf(fmaxf(unmasked_abs(vp.x), unmasked_abs(vp.y)), fmaxf(unmasked_abs(vp.z), unmasked_abs(vp.w)));
  const float delta = wave_max(d), mag = wave_max(a);
  const bool below = certified_zero(mpr, mpr2, js, dv, delta, mag, ph);  // (the same certificate as in screened_body)
  // (unchanged: the row segment was all zero and stays so; its sum and its line flags in memory are zeros already)
  const bool unchanged = !renew && oldlines == 0 && below;
  const bool certified = lane >= nrows || unchanged;
  tile_total = 0.f;
  reads = 0;
  if (stop) return f4v{0.f, 0.f, 0.f, 0.f};
  unsigned long long todo = ~__builtin_amdgcn_ballot_w64(certified);
  reads = __builtin_popcountll(todo);
  float mkeep = 0.f, m2keep = 0.f;  // renew: lane u keeps the new bounds of row u
  int jkeep = 0;
  unsigned newlines = 0;  // lane u keeps the nonzero lines of the new row u
  const unsigned myline = (unsigned)lane >> 3;  // 8 lanes x 16 bytes: one 128-byte line

  f4v tile_acc = {0.f, 0.f, 0.f, 0.f}, group_acc = {0.f, 0.f, 0.f, 0.f};
  float tile_tot = 0.f, group_tot = 0.f;  // the total of the tile, added up in the same order
  int group = -1;
  float rowkeep = 0.f;
  constexpr int kWalk = 3;  // rows fetched together: their loads overlap, the arithmetic stays in row order
  while (todo != 0) {
    int row[kWalk];
    unsigned wl[kWalk];  // the lines of the new row to write
    f4v c[kWalk], x[kWalk];
#pragma unroll
    for (int b = 0; b < kWalk; ++b) {
      row[b] = -1;
      wl[b] = 0;
      c[b] = f4v{0.f, 0.f, 0.f, 0.f};
      x[b] = f4v{0.f, 0.f, 0.f, 0.f};
      if (todo != 0) {
        row[b] = __builtin_ctzll(todo);
        todo &= todo - 1;
        c[b] = ld4<EDGE, NT>(Cp + row[b] * ldc, nmem);
        // of X only the lines that hold something (a plan has about one nonzero per nonzero row segment)
        const unsigned ol = (unsigned)__builtin_amdgcn_readlane((int)oldlines, row[b]);
        if ((ol >> myline) & 1) x[b] = ld4<EDGE, NT>(Xp + row[b] * ldx, nmem);
      }
    }
    // (everything fetched has arrived from here on: said once, for all the rows, so that no row's arithmetic and
    // no store below waits again, which on this counter would mean waiting for the stores issued before it)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
#pragma unroll
    for (int b = 0; b < kWalk; ++b) {
      const int u = row[b];
      if (u >= 0) {
        if ((u >> 3) != group) {
          if (group >= 0) {
            tile_acc += group_acc;
            tile_tot += group_tot;
          }
          group_acc = f4v{0.f, 0.f, 0.f, 0.f};
          group_tot = 0.f;
          group = u >> 3;
        }
        const float phu = __builtin_bit_cast(float, __builtin_amdgcn_readlane(fbits(ph), u));
        const f4v v = xbar4(x[b], c[b], vp + phu, rho) * scale;
        const bool nonzero = ((fbits(v.x) | fbits(v.y)) | (fbits(v.z) | fbits(v.w))) != 0;
        // lines with a nonzero now (bit g: any of lanes 8g .. 8g+7); those and the ones that held one
        // before are written, the others are zero in memory and stay so
        unsigned long long nzb = __builtin_amdgcn_ballot_w64(nonzero);
        nzb |= nzb >> 4;
        nzb |= nzb >> 2;
        nzb |= nzb >> 1;
        const unsigned nl = (unsigned)(((nzb & 0x0101010101010101ull) * 0x0102040810204080ull) >> 56);
        const unsigned ol = (unsigned)__builtin_amdgcn_readlane((int)oldlines, u);
        x[b] = v;
        wl[b] = ol | nl;
        newlines = (lane == u) ? nl : newlines;
        group_acc += v;
        const float tot = wave_sum((v.x + v.y) + (v.z + v.w));
        rowkeep = (lane == u) ? tot : rowkeep;
        group_tot += tot;
        if (renew) {
          const f4v t = {fmaf(-rho, c[b].x, vp.x), fmaf(-rho, c[b].y, vp.y), fmaf(-rho, c[b].z, vp.z), fmaf(-rho, c[b].w, vp.w)};
          float mm, mm2;
          int jj;
          segment_top2(t, lane, mm, jj, mm2);
          mkeep = (lane == u) ? mm : mkeep;
          m2keep = (lane == u) ? mm2 : m2keep;
          jkeep = (lane == u) ? jj : jkeep;
        }
      }
    }
    // the stores leave together, after the arithmetic of all the rows fetched together: the one counter for loads
    // and stores cannot tell a store still on its way from a load, so a row worked on after another row's store
    // would wait for that store to come back
#pragma unroll
    for (int b = 0; b < kWalk; ++b)
      if (row[b] >= 0 && ((wl[b] >> myline) & 1)) st4<EDGE, NT>(Xp + row[b] * ldx, x[b], nmem);
  }
  if (group >= 0) {
    tile_acc += group_acc;
    tile_tot += group_tot;
  }
  if (lane < nrows) {
    // (the sums are kept in place, and the flags too when the previous sweep left them: what has not changed is
    // not written again, which is nearly everything)
    if (!unchanged) A.rowpart[ridx] = rowkeep;
    if (SC.lines_in == nullptr || newlines != oldlines) SC.lines_out[ridx] = (unsigned char)newlines;
  }
  if (renew) {
    if (lane < nrows) {
      SC.mprime_out[ridx] = mkeep;
      SC.m2_out[ridx] = m2keep;
      SC.jstar_out[ridx] = (unsigned char)jkeep;
    }
    if (tr == 0) {  // the first tile of the column segment also stores the epoch's varphi
      *reinterpret_cast<f4u*>(SC.varphi0_out + j0) = vp;  // (past n both buffers hold the mask value)
    }
  }
  tile_total = tile_tot;
  return tile_acc;  // column sums of the tile (columns past n: 0)
}

// Four waves per workgroup, stacked along the rows.  They work independently; each leaves its tile's column sums
// in LDS, counts itself in and ends, and the one that finds itself the last adds the four tiles' sums in the
// order tile 0, 1, 2, 3 (kColGroup in the reduction: the sweeps that store one row of column sums per 64-row
// tile are added up in that order too) and stores them.  No wave waits for another: a wave that has little to
// do gives its place on the SIMD to the next workgroup's at once.  (LDS serves a wave's operations in the order
// it issued them, so a wave's sums are in place before its count is; the count starts at zero behind the one
// barrier at the start, where nobody has anything to wait for yet.)
constexpr int kLeanWaves = 4;
constexpr int kColGroup = kLeanWaves;
static_assert(64 * kLeanWaves == kSegCols, "four columns per lane of the wave that does the final fold");

template <bool NT>
__global__ __launch_bounds__(64 * kLeanWaves, 8) void screened_lean_kernel(SweepArgs A, ScreenArgs SC, int ntiles_rows) {
  __shared__ float fold[kLeanWaves][kSegCols];
  __shared__ float totals[kLeanWaves];
  __shared__ int nreads[kLeanWaves];
  __shared__ int arrived;
  if (threadIdx.x == 0) arrived = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y * kLeanWaves + wave;
  f4v acc = {0.f, 0.f, 0.f, 0.f};
  float total = 0.f;
  int reads = 0, stop;
  if (tr < ntiles_rows) {
    if ((seg + 1) * kSegCols <= A.n) acc = screened_lean_body<false, NT>(A, SC, lane, seg, tr, stop, total, reads);
    else acc = screened_lean_body<true, NT>(A, SC, lane, seg, tr, stop, total, reads);
  } else {
    stop = *A.done;
  }
  if (stop) return;
  *reinterpret_cast<f4v*>(&fold[wave][lane * 4]) = acc;
  if (lane == 0) {
    totals[wave] = total;
    nreads[wave] = reads;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  int before = 0;
  if (lane == 0) before = __hip_atomic_fetch_add(&arrived, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  before = __builtin_amdgcn_readfirstlane(before);
  if (before != kLeanWaves - 1) return;  // (somebody is still at work: they will do the rest)
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  const int c0 = lane * 4, j0 = seg * kSegCols + c0;
  const f4v f0 = *reinterpret_cast<const f4v*>(&fold[0][c0]), f1 = *reinterpret_cast<const f4v*>(&fold[1][c0]);
  const f4v f2 = *reinterpret_cast<const f4v*>(&fold[2][c0]), f3 = *reinterpret_cast<const f4v*>(&fold[3][c0]);
  const f4v sum = ((f0 + f1) + f2) + f3;
  float* __restrict__ dst = A.colpart + (size_t)blockIdx.y * A.np + j0;
  if (j0 + 3 < A.n) {
    *reinterpret_cast<f4v*>(dst) = sum;  // (np is a multiple of 64: 16-byte aligned)
  } else {
    if (j0 < A.n) dst[0] = sum.x;
    if (j0 + 1 < A.n) dst[1] = sum.y;
    if (j0 + 2 < A.n) dst[2] = sum.z;
  }
  if (lane == 0) {
    A.tilesum[blockIdx.y * gridDim.x + seg] = ((totals[0] + totals[1]) + totals[2]) + totals[3];
    SC.wg_reads[blockIdx.y * gridDim.x + seg] = (nreads[0] + nreads[1]) + (nreads[2] + nreads[3]);
  }
}
