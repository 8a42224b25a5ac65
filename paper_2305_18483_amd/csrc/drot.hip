// Douglas-Rachford splitting for regularized discrete optimal transport on MI355X (gfx950).
//
// One iteration = one sweep over the m x n plan (eq. (8): X <- prox_{rho h}([X + phi 1^T +
// 1 varphi^T - rho C]_+), fused with the row sums, column sums and grand total the marginal
// projection needs) followed by the O(m+n) recursion of eq. (6).  Y is never formed (Section
// 2.1: "Y_k can be eliminated").  The sweep is HBM bound (12 bytes per element: read X, read C,
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
// This file is the whole product path: kernels, host loop and the C ABI of include/drot.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "drot.h"

namespace {

typedef float f4v __attribute__((ext_vector_type(4)));
typedef f4v f4u __attribute__((aligned(4)));  // 128-bit access that only needs 4-byte alignment

constexpr int kBlock = 256;          // threads per workgroup in the group-lasso and gap kernels (4 waves)
constexpr int kWavesPerBlock = 4;
constexpr int kSegCols = 256;        // columns per tile: 64 lanes x 4
constexpr int kTileRows = 32;        // rows per tile, the same in every matrix kernel
constexpr int kAlignElems = 32;      // rows of X and C are kept on 128-byte lines (padded working copies otherwise)
constexpr int kSweepWaves = 16;      // sweep: waves per workgroup, stacked along the rows
constexpr int kSweepRows = kTileRows / kSweepWaves;   // sweep: rows per wave (one batch, no loop)
constexpr int kLoopRows = kTileRows / kWavesPerBlock; // looping kernels: rows per wave
constexpr float kMaskedOut = -1.0e30f;  // added to columns past n so that [.]_+ yields exactly 0

// ------------------------------------------------------------------------------------------
// device helpers
// ------------------------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}

// Bits of a float.  (By value on purpose: __builtin_bit_cast applied directly to an element of a
// vector, as in bit_cast(int, v.y), reads the vector's first element.)
__device__ __forceinline__ int fbits(float f) { return __builtin_bit_cast(int, f); }

// Sum over the 64 lanes of a wave; the result is wave-uniform (read back from lane 63).
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_mov<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
  v += dpp_mov<0x141, 0xF>(v);  // row_half_mirror
  v += dpp_mov<0x140, 0xF>(v);  // row_mirror: every lane of a 16-lane row holds the row total
  v += dpp_mov<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
  v += dpp_mov<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// The same for a double (each step moves the two halves separately).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_mov_f64(double v) {
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)b, CTRL, ROW_MASK, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(b >> 32), CTRL, ROW_MASK, 0xF, false);
  return __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi << 32) | (unsigned long long)(unsigned)lo);
}
__device__ __forceinline__ double wave_sum_f64(double v) {
  v += dpp_mov_f64<0xB1, 0xF>(v);
  v += dpp_mov_f64<0x4E, 0xF>(v);
  v += dpp_mov_f64<0x141, 0xF>(v);
  v += dpp_mov_f64<0x140, 0xF>(v);
  v += dpp_mov_f64<0x142, 0xA>(v);
  v += dpp_mov_f64<0x143, 0xC>(v);
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, 63);
  const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), 63);
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | (unsigned long long)lo);
}

// Maximum over the 64 lanes of a wave, wave-uniform: the steps of wave_sum with max in place of +.
// (The two broadcast steps hand 0 to the lanes they do not reach; lane 63, the one read back, is
// reached by both, and the lanes it reads are read before they are touched: the result is exact
// whatever the signs.)
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1, 0xF>(v));
  v = fmaxf(v, dpp_mov<0x4E, 0xF>(v));
  v = fmaxf(v, dpp_mov<0x141, 0xF>(v));
  v = fmaxf(v, dpp_mov<0x140, 0xF>(v));
  v = fmaxf(v, dpp_mov<0x142, 0xA>(v));
  v = fmaxf(v, dpp_mov<0x143, 0xC>(v));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__device__ __forceinline__ f4v load4(const float* __restrict__ ptr, int nvalid) {
  if (nvalid == 4) return *reinterpret_cast<const f4u*>(ptr);
  f4v v = {0.f, 0.f, 0.f, 0.f};
  if (nvalid > 0) v.x = ptr[0];
  if (nvalid > 1) v.y = ptr[1];
  if (nvalid > 2) v.z = ptr[2];
  return v;
}

__device__ __forceinline__ void store4(float* __restrict__ ptr, f4v v, int nvalid) {
  if (nvalid == 4) {
    *reinterpret_cast<f4u*>(ptr) = v;
    return;
  }
  if (nvalid > 0) ptr[0] = v.x;
  if (nvalid > 1) ptr[1] = v.y;
  if (nvalid > 2) ptr[2] = v.z;
}

// varphi of this lane's four columns; columns past n get a huge negative value so that the
// nonnegativity clamp zeroes them and they drop out of every sum.
__device__ __forceinline__ f4v load_varphi(const float* __restrict__ varphi, int j0, int nvalid) {
  f4v v = {kMaskedOut, kMaskedOut, kMaskedOut, kMaskedOut};
  if (nvalid == 4) return *reinterpret_cast<const f4u*>(varphi + j0);
  if (nvalid > 0) v.x = varphi[j0];
  if (nvalid > 1) v.y = varphi[j0 + 1];
  if (nvalid > 2) v.z = varphi[j0 + 2];
  return v;
}

// [x + phi_i + varphi_j - rho c]_+   (first half of eq. (8))
__device__ __forceinline__ f4v xbar4(f4v x, f4v c, f4v pv, float rho) {
  f4v v;
  v.x = fmaxf(fmaf(-rho, c.x, x.x + pv.x), 0.f);
  v.y = fmaxf(fmaf(-rho, c.y, x.y + pv.y), 0.f);
  v.z = fmaxf(fmaf(-rho, c.z, x.z + pv.z), 0.f);
  v.w = fmaxf(fmaf(-rho, c.w, x.w + pv.w), 0.f);
  return v;
}

// Sum of one double per thread over the workgroup, the same value (same bits) in every thread:
// butterfly inside each wave, then the wave sums added in wave order.  red: >= blockDim.x/64 doubles.
__device__ __forceinline__ double block_sum_f64(double v, double* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  const int t = threadIdx.x;
  const int nw = (blockDim.x + 63) >> 6;
  __syncthreads();  // red may still be read by the previous use
  if ((t & 63) == 0) red[t >> 6] = v;
  __syncthreads();
  double out = 0.0;
  for (int w = 0; w < nw; ++w) out += red[w];
  return out;
}

// ------------------------------------------------------------------------------------------
// device-side state shared by the kernels of one solve
// ------------------------------------------------------------------------------------------
struct DeviceStatus {
  double r2, s2;                 // ||X1-p||^2, ||X^T1-q||^2 of the last checked iterate
  double cost, h, dual_lin, h_conj, gap, dual_res;
  double nz_segments;            // row partial sums of the last reduction that were not zero (density of the plan)
  int iters;                     // iteration the residuals belong to
  int converged;
};

struct SweepArgs {
  float* X;
  const float* C;
  const float* phi;
  const float* varphi;
  float* rowpart;
  float* colpart;
  float* tilesum;        // [ntr*nseg] total of every tile (only read by the fused vector update)
  const int* done;
  int m, n;
  int ldx, ldc;          // row pitch of X and of C in elements (n, or the padded working copies' pitch)
  float rho, scale;
  int n_mem;             // columns the sweep may touch in memory: n, or the pitch when X and C are both the
                         // library's padded copies (their pad columns are kept at zero), so that the last
                         // lanes of a row can use full 128-bit accesses
  const float* rowpart_prev;  // plain sweep: the row-segment sums of the X in memory (layout of rowpart), or null
                              // when they are not known or not to be used; a segment whose sum is zero is all
                              // zero: it is not read, and not written back if it stays zero
};

// Inputs of the vector update when it is fused into the head of the next sweep (small problems):
// the partial sums the previous sweep left and the eq. (6) state before / after the update.
struct FusedUpdateArgs {
  const float* rowpart_prev;
  const float* colpart_prev;
  const float* tilesum_prev;
  const float* p;
  const float* q;
  const double* a_in;
  const double* b_in;
  double* a_out;
  double* b_out;
  const double* theta_in;
  double* theta_out;
  const double* sum_p;
  float* phi_out;
  float* varphi_out;
  int nseg, ntr;
};

// ------------------------------------------------------------------------------------------
// S1-S4: the sweep for h = 0 and h = (lambda/2)||X||^2 (a constant scale, Section 3).
// grid = (nseg, ntr); a workgroup owns 32 rows x 256 columns; each of its 16 waves loads its
// 2 row segments of 1 KiB of X and C, updates, stores and is done.  EDGE marks the last column
// segment when n is not a multiple of 256: only there do lanes check how many of their 4
// columns exist.  NT marks the accesses non-temporal (used when X and C cannot stay in cache).
//
// Alignment (what the paper's "shifted work areas" of Section "General Optimization" are for):
// row segments that straddle 128-byte lines cost 10-28 % here, so the host hands this kernel
// rows that start on a line: the caller's arrays when n % 32 == 0 and the base is aligned, else
// working copies with the pitch rounded up to 32 elements (ldx, ldc).
// ------------------------------------------------------------------------------------------
template <bool EDGE, bool NT>
__device__ __forceinline__ f4v ld4(const float* __restrict__ ptr, int nvalid) {
  if (EDGE) return load4(ptr, nvalid);
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f4u*>(ptr));
  return *reinterpret_cast<const f4u*>(ptr);
}
template <bool EDGE, bool NT>
__device__ __forceinline__ void st4(float* __restrict__ ptr, f4v v, int nvalid) {
  if (EDGE) store4(ptr, v, nvalid);
  else if (NT) __builtin_nontemporal_store(v, reinterpret_cast<f4u*>(ptr));
  else *reinterpret_cast<f4u*>(ptr) = v;
}

// Folds the column partials of the NW waves of a workgroup through LDS and writes the tile's
// column sums (fixed order: deterministic).
template <int NW>
__device__ __forceinline__ void write_col_partials(f4v colacc, int lane, int wave, int seg, int tr, int n,
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
    if (j < n) colpart[(size_t)tr * n + j] = sum;
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
    for (int u = 0; u < 16; ++u) v[u] = F.colpart_prev[(size_t)min(sub + 4 * u, F.ntr - 1) * A.n + j];
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
    ri = sum_partials_16(F.rowpart_prev + i, (size_t)A.m, F.nseg) - (double)F.p[i];
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
  const int nvalid = EDGE ? min(max(A.n - j0, 0), 4) : 4;      // columns of this lane that exist
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
    if (lane < nrows) prev = A.rowpart_prev[(size_t)seg * A.m + r0 + lane];
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
      if (!FIRST && readx[u]) x[u] = ld4<EDGE, NT>(Xp + u * ldx, nmem);
    }
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      c[u] = f4v{0.f, 0.f, 0.f, 0.f};
      x[u] = f4v{0.f, 0.f, 0.f, 0.f};
      if (u < nrows) {
        if (MODE < 2) c[u] = ld4<EDGE, NT>(Cp + u * ldc, nmem);
        if (!FIRST && readx[u]) x[u] = ld4<EDGE, NT>(Xp + u * ldx, nmem);
      }
    }
  }
  // with the fused update (PRO) phi and varphi of this tile are computed into LDS while the loads fly
  if (PRO) fused_update(A, F, seg, tr, lds_phi, lds_varphi);

  f4v colacc = {0.f, 0.f, 0.f, 0.f};
  float wave_total = 0.f;
  {
    const f4v vp = PRO ? *reinterpret_cast<const f4v*>(lds_varphi + lane * 4) : load_varphi(A.varphi, j0, nvalid);
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
    if (lane < nrows) A.rowpart[(size_t)seg * A.m + r0 + lane] = rowkeep;
  }
  write_col_partials<NW>(colacc, lane, wave, seg, tr, A.n, A.colpart);
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
  else sweep_body<FIRST, true, false, PRO, MODE, U, NW>(A, F, lane, wave, seg, tr, lds_phi, lds_varphi);
}

// ------------------------------------------------------------------------------------------
// Screened sweep (large sparse problems).  On top of skipping the all-zero row segments of X, most
// of C need not be read either: a row segment with x = 0 comes out as zero again whenever
// phi_i + varphi_j - rho C_ij <= 0 for its 256 columns, and that can be certified from one number.
// A "refresh" sweep, which reads all of C, records for every row segment
//     M_is = max_j ( varphi0_j - rho C_ij )            (varphi0 = the varphi of that sweep).
// Later sweeps form, per column segment, delta_s = max_j (varphi_j - varphi0_j) and, per row,
//     S = M_is + delta_s + phi_i  >=  max_j ( phi_i + varphi_j - rho C_ij ).
// If S plus a rounding margin is <= 0 and the segment of X is zero, the segment stays zero: its C is
// not read, nothing is computed, its row sum is 0.  The result is the one the plain sweep would
// produce (the margin dominates the handful of fp32 roundings between the two evaluations).  As
// varphi drifts away from varphi0 fewer segments certify; the host refreshes every so many sweeps.
// Tiles: 8 waves x 8 rows x 256 columns, as the unscreened sweep for sparse plans.
// ------------------------------------------------------------------------------------------
struct ScreenArgs {
  const float* mprime_in;   // [nseg][m] M_is of the current epoch (screening sweeps)
  float* mprime_out;        // [nseg][m] written by a refresh sweep
  const float* varphi0;     // [n] varphi of the epoch
  int* wave_reads;          // 8-wave tiles, profiling only (else null): [workgroup][wave] row segments of C this wave read
  // lean sweep only: it renews the bounds by itself when the vector update before it has raised ctl[0]
  float* varphi0_out;       // [n]
  const int* ctl;           // kCtl... words, see ScreenCtl
  int* wg_reads;            // [workgroup] row segments of C the workgroup read (always written)
  // lean sweep only: which of the eight 128-byte lines of a row segment of X hold a nonzero
  const unsigned char* lines_in;  // [nseg][m] as left by the previous sweep if that was a lean one, else null
  unsigned char* lines_out;       // [nseg][m]
};

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
  const int nvalid = EDGE ? min(max(A.n - j0, 0), 4) : 4;
  const int nmem = EDGE ? min(max(A.n_mem - j0, 0), 4) : 4;
  const int r0 = (tr * NW + wave) * U;
  const int nrows = min(max(A.m - r0, 0), U);
  const size_t ldx = (size_t)A.ldx, ldc = (size_t)A.ldc;
  const float* __restrict__ Cp = A.C + (size_t)r0 * ldc + j0;
  float* __restrict__ Xp = A.X + (size_t)r0 * ldx + j0;
  const float rho = A.rho, scale = A.scale;
  const size_t ridx = (size_t)seg * A.m + r0 + lane;  // this lane's row in the per-row-segment arrays (lane < nrows)

  // lane u: old sum, phi and M of row r0 + u
  const f4v vp = load_varphi(A.varphi, j0, nvalid);
  float prev = 0.f, ph = kMaskedOut, mpr = 0.f;
  if (lane < nrows) {
    prev = A.rowpart_prev ? A.rowpart_prev[ridx] : 1.f;
    ph = A.phi[r0 + lane];
    if (!REFRESH) mpr = SC.mprime_in[ridx];
  }
  bool certified = lane >= nrows;  // rows past the end of the matrix: nothing to do
  if (!REFRESH) {
    const f4v vp0 = load_varphi(SC.varphi0, j0, nvalid);
    // drift of varphi since the epoch and its magnitude over this wave's columns (columns past n: both
    // carry the same mask value, their difference is 0; they are left out of the magnitude)
    float d = fmaxf(fmaxf(vp.x - vp0.x, vp.y - vp0.y), fmaxf(vp.z - vp0.z, vp.w - vp0.w));
    float a = 0.f;
    if (nvalid > 0) a = fabsf(vp.x);
    if (nvalid > 1) a = fmaxf(a, fabsf(vp.y));
    if (nvalid > 2) a = fmaxf(a, fabsf(vp.z));
    if (nvalid > 3) a = fmaxf(a, fabsf(vp.w));
    const float delta = wave_max(d), mag = wave_max(a);
    // S bounds every phi_i + varphi_j - rho C_ij of the row segment from above; the margin, 8 units in
    // the last place of the largest term, covers the roundings of M, of delta, of this sum and of the
    // sweep's own evaluation (each at most half a unit of a term no larger than these)
    const float bound = (mpr + delta) + ph;
    const float margin = 4.76837158e-7f * (fabsf(mpr) + fabsf(delta) + fabsf(ph) + mag);  // 2^-21
    const bool below = (bound + margin <= 0.f) || mpr == -INFINITY;  // (-inf: every pair of the segment is forbidden)
    certified = certified || (fbits(prev) == 0 && below);
  }
  const unsigned skipmask = (unsigned)__builtin_amdgcn_ballot_w64(certified) & 0xffu;
  const unsigned nzmask = (unsigned)__builtin_amdgcn_ballot_w64(fbits(prev) != 0) & 0xffu;

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
  float rowkeep = 0.f, mkeep = 0.f, wave_total = 0.f;
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
      if (REFRESH) {
        const float mx = fmaxf(fmaxf(fmaf(-rho, c[u].x, vp.x), fmaf(-rho, c[u].y, vp.y)),
                               fmaxf(fmaf(-rho, c[u].z, vp.z), fmaf(-rho, c[u].w, vp.w)));
        const float mm = wave_max(mx);
        mkeep = (lane == u) ? mm : mkeep;
      }
    }
  }
  if (lane < nrows) {
    A.rowpart[ridx] = rowkeep;
    if (REFRESH) SC.mprime_out[ridx] = mkeep;
  }
  if (SC.wave_reads && lane == 0)
    SC.wave_reads[(tr * gridDim.x + seg) * NW + wave] = __builtin_popcount(~skipmask & 0xffu);
  write_col_partials<NW>(colacc, lane, wave, seg, tr, A.n, A.colpart);
  write_tile_total<NW>(wave_total, lane, wave, seg, tr, A.tilesum);
}

// Profiling: total of the per-wave read counts of one screened sweep.
__global__ __launch_bounds__(1024) void sum_reads_kernel(const int* __restrict__ wave_reads, int count, double* out) {
  __shared__ double red[1024 / 64];
  double acc = 0.0;
  for (int e = threadIdx.x; e < count; e += 1024) acc += (double)wave_reads[e];
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
  else screened_body<true, false, REFRESH>(A, SC, lane, wave, seg, tr);
}

// The screened sweep for plans known to be sparse (a few percent of the row segments left to
// process): one wave owns a whole 64 x 256 tile, lane l holding the old sum, phi and M of row l.
// It decides all 64 rows at once and then walks through the rows left over, one at a time.  No
// LDS, no barrier; 8 times fewer waves than the tile of 8 waves x 8 rows, and the same bits: the
// rows of every group of 8 are added up in order and the 8 groups in order, which is what that
// tile's waves and its LDS fold do (rows and groups that contribute nothing add +0).
template <bool EDGE, bool NT>
__device__ __forceinline__ f4v screened_lean_body(const SweepArgs& A, const ScreenArgs& SC, int lane, int seg, int tr,
                                                  int stop, bool renew, float& tile_total, int& reads) {
  const int j0 = seg * kSegCols + lane * 4;
  const int nvalid = EDGE ? min(max(A.n - j0, 0), 4) : 4;
  const int nmem = EDGE ? min(max(A.n_mem - j0, 0), 4) : 4;
  const int r0 = tr * 64;
  const int nrows = min(A.m - r0, 64);
  const size_t ldx = (size_t)A.ldx, ldc = (size_t)A.ldc;
  const float* __restrict__ Cp = A.C + (size_t)r0 * ldc + j0;
  float* __restrict__ Xp = A.X + (size_t)r0 * ldx + j0;
  const float rho = A.rho, scale = A.scale;
  const size_t ridx = (size_t)seg * A.m + r0 + lane;

  const f4v vp = load_varphi(A.varphi, j0, nvalid);
  const f4v vp0 = load_varphi(SC.varphi0, j0, nvalid);
  float prev = 0.f, ph = kMaskedOut, mpr = 0.f;
  unsigned oldlines = 0;  // lane u: the lines of row u's segment of X that hold a nonzero (bit g: columns 32g .. 32g+31)
  if (lane < nrows) {
    prev = A.rowpart_prev ? A.rowpart_prev[ridx] : 1.f;
    ph = A.phi[r0 + lane];
    mpr = SC.mprime_in[ridx];
    oldlines = SC.lines_in ? SC.lines_in[ridx] : 0xffu;
  }
  if (fbits(prev) == 0) oldlines = 0;
  // (renew, wave-uniform: this sweep records new bounds against the varphi of now; it certifies
  // nothing, walks through all its rows and takes the maximum of varphi_j - rho C_ij of each)
  float d = fmaxf(fmaxf(vp.x - vp0.x, vp.y - vp0.y), fmaxf(vp.z - vp0.z, vp.w - vp0.w));
  float a = 0.f;
  if (nvalid > 0) a = fabsf(vp.x);
  if (nvalid > 1) a = fmaxf(a, fabsf(vp.y));
  if (nvalid > 2) a = fmaxf(a, fabsf(vp.z));
  if (nvalid > 3) a = fmaxf(a, fabsf(vp.w));
  const float delta = wave_max(d), mag = wave_max(a);
  const float bound = (mpr + delta) + ph;  // (the same certificate, to the letter, as in screened_body)
  const float margin = 4.76837158e-7f * (fabsf(mpr) + fabsf(delta) + fabsf(ph) + mag);
  const bool below = (bound + margin <= 0.f) || mpr == -INFINITY;
  const bool certified = lane >= nrows || (!renew && fbits(prev) == 0 && below);
  tile_total = 0.f;
  reads = 0;
  if (stop) return f4v{0.f, 0.f, 0.f, 0.f};
  unsigned long long todo = ~__builtin_amdgcn_ballot_w64(certified);
  reads = __builtin_popcountll(todo);
  float mkeep = 0.f;  // renew: lane u keeps the new bound of row u
  unsigned newlines = 0;  // lane u keeps the nonzero lines of the new row u
  const unsigned myline = (unsigned)lane >> 3;  // 8 lanes x 16 bytes: one 128-byte line

  f4v tile_acc = {0.f, 0.f, 0.f, 0.f}, group_acc = {0.f, 0.f, 0.f, 0.f};
  float tile_tot = 0.f, group_tot = 0.f;  // the total of the tile, added up in the same order
  int group = -1;
  float rowkeep = 0.f;
  constexpr int kWalk = 4;  // rows fetched together: their loads overlap, the arithmetic stays in row order
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
        c[b] = ld4<EDGE, NT>(Cp + row[b] * ldc, nmem);
        // of X only the lines that hold something (a plan has about one nonzero per nonzero row segment)
        const unsigned ol = (unsigned)__builtin_amdgcn_readlane((int)oldlines, row[b]);
        if ((ol >> myline) & 1) x[b] = ld4<EDGE, NT>(Xp + row[b] * ldx, nmem);
      }
    }
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
        if (((ol | nl) >> myline) & 1) st4<EDGE, NT>(Xp + u * ldx, v, nmem);
        newlines = (lane == u) ? nl : newlines;
        group_acc += v;
        const float tot = wave_sum((v.x + v.y) + (v.z + v.w));
        rowkeep = (lane == u) ? tot : rowkeep;
        group_tot += tot;
        if (renew) {
          const float mx = fmaxf(fmaxf(fmaf(-rho, c[b].x, vp.x), fmaf(-rho, c[b].y, vp.y)),
                                 fmaxf(fmaf(-rho, c[b].z, vp.z), fmaf(-rho, c[b].w, vp.w)));
          const float mm = wave_max(mx);
          mkeep = (lane == u) ? mm : mkeep;
        }
      }
    }
  }
  if (group >= 0) {
    tile_acc += group_acc;
    tile_tot += group_tot;
  }
  if (lane < nrows) {
    A.rowpart[ridx] = rowkeep;
    SC.lines_out[ridx] = (unsigned char)newlines;
  }
  if (renew) {
    if (lane < nrows) SC.mprime_out[ridx] = mkeep;
    if (tr == 0) {  // the first tile of the column segment also stores the epoch's varphi
      float* __restrict__ v0 = SC.varphi0_out + j0;
      if (nvalid == 4) *reinterpret_cast<f4u*>(v0) = vp;
      else {
        if (nvalid > 0) v0[0] = vp.x;
        if (nvalid > 1) v0[1] = vp.y;
        if (nvalid > 2) v0[2] = vp.z;
      }
    }
  }
  tile_total = tile_tot;
  return tile_acc;  // column sums of the tile (columns past n: 0)
}

// Four waves per workgroup, stacked along the rows: they work independently and meet once, at the
// end, to add their tiles' column sums in the order tile 0, 1, 2, 3 (kColGroup in the reduction:
// the sweeps that store one row of column sums per 64-row tile are added up in that order too).
constexpr int kLeanWaves = 4;
constexpr int kColGroup = kLeanWaves;
static_assert(64 * kLeanWaves == kSegCols, "one thread per column of the segment in the final fold");

template <bool NT>
__global__ __launch_bounds__(64 * kLeanWaves) void screened_lean_kernel(SweepArgs A, ScreenArgs SC, int ntiles_rows) {
  // (the stop flag is fetched along with a wave's first loads and tested before its first store)
  const int stop = *A.done;
  const bool renew = SC.ctl[kCtlRenew] != 0;
  __shared__ float fold[kLeanWaves][kSegCols];
  __shared__ float totals[kLeanWaves];
  __shared__ int nreads[kLeanWaves];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int seg = blockIdx.x, tr = blockIdx.y * kLeanWaves + wave;
  f4v acc = {0.f, 0.f, 0.f, 0.f};
  float total = 0.f;
  int reads = 0;
  if (tr < ntiles_rows) {
    if ((seg + 1) * kSegCols <= A.n) acc = screened_lean_body<false, NT>(A, SC, lane, seg, tr, stop, renew, total, reads);
    else acc = screened_lean_body<true, false>(A, SC, lane, seg, tr, stop, renew, total, reads);
  }
  if (stop) return;
  *reinterpret_cast<f4v*>(&fold[wave][lane * 4]) = acc;
  if (lane == 0) {
    totals[wave] = total;
    nreads[wave] = reads;
  }
  __syncthreads();
  const int t = threadIdx.x, j = seg * kSegCols + t;
  if (j < A.n) A.colpart[(size_t)blockIdx.y * A.n + j] = ((fold[0][t] + fold[1][t]) + fold[2][t]) + fold[3][t];
  if (t == 0) {
    A.tilesum[blockIdx.y * gridDim.x + seg] = ((totals[0] + totals[1]) + totals[2]) + totals[3];
    SC.wg_reads[blockIdx.y * gridDim.x + seg] = (nreads[0] + nreads[1]) + (nreads[2] + nreads[3]);
  }
}

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

  // sweep layout: start the loads of X and of the per-row / per-column vectors
  f4v x[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    x[u] = f4v{0.f, 0.f, 0.f, 0.f};
    if (!FIRST && u < nrows) {
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
        if (NT && nvalid == 4) __builtin_nontemporal_store(v, reinterpret_cast<f4u*>(Xp + u * ldx));
        else store4(Xp + u * ldx, v, nvalid);
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

// ------------------------------------------------------------------------------------------
// Group lasso, general labels, two passes (Section "Group-lasso Regularized DROT": when a
// group does not fit one workgroup the reduction goes through global memory and a second
// kernel applies the scale).  Pass 1 accumulates sum_{i in class} Xbar_ij^2 per (class, column).
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

template <bool FIRST>
__global__ __launch_bounds__(kBlock) void gl_norm_kernel(GroupArgs G) {
  const SweepArgs& A = G.S;
  if (*A.done) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j0 = blockIdx.x * kSegCols + lane * 4;
  const int nvalid = min(max(A.n - j0, 0), 4);
  const f4v vp = load_varphi(A.varphi, j0, nvalid);
  const int rbeg = blockIdx.y * kTileRows + wave * kLoopRows;
  const int rend = min(rbeg + kLoopRows, A.m);
  int cur = -1;
  f4v acc = {0.f, 0.f, 0.f, 0.f};
  for (int i = rbeg; i < rend; ++i) {
    const int cls = G.row_class[i];
    if (cls != cur) {
      if (cur >= 0) flush_group(G.gsq + (size_t)cur * A.n + j0, acc, nvalid);
      cur = cls;
      acc = f4v{0.f, 0.f, 0.f, 0.f};
    }
    const f4v c = load4(A.C + (size_t)i * A.ldc + j0, nvalid);
    const f4v x = FIRST ? f4v{0.f, 0.f, 0.f, 0.f} : load4(A.X + (size_t)i * A.ldx + j0, nvalid);
    const f4v v = xbar4(x, c, vp + A.phi[i], A.rho);
    acc += v * v;
  }
  if (cur >= 0) flush_group(G.gsq + (size_t)cur * A.n + j0, acc, nvalid);
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
  if (lane < rend - rbeg) A.rowpart[(size_t)seg * A.m + rbeg + lane] = rowkeep;
  write_col_partials<kWavesPerBlock>(colacc, lane, wave, seg, tr, A.n, A.colpart);
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
  if (*A.done) return;
  __shared__ float red[RL][COLS];  // 16 KiB either way
  __shared__ float part[16][COLS];
  __shared__ float bcast[COLS];
  __shared__ float lds_varphi[COLS];
  __shared__ float lds_phi[kSlabThreads];
  __shared__ double dred[kSlabThreads / 64];
  const int t = threadIdx.x;
  const int cx = t % CX, ry = t / CX;
  const int strip = blockIdx.x, run = blockIdx.y;
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
    if (flags && r < len) held[k] = fbits(A.rowpart_prev[(size_t)strip * A.m + start + r]) != 0;
  }
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int r = ry + RL * k;
    c[k] = f4v{0.f, 0.f, 0.f, 0.f};
    x[k] = f4v{0.f, 0.f, 0.f, 0.f};
    ph[k] = kMaskedOut;  // rows past the run: the clamp zeroes them
    if (r < len) {
      c[k] = load4(Cp + (size_t)(RL * k) * ldc, nvalid);
      if (!FIRST && held[k]) x[k] = load4(Xp + (size_t)(RL * k) * ldx, nvalid);
      if (!PRO) ph[k] = A.phi[start + r];
    }
  }
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
      ri = sum_partials_16(F.rowpart_prev + i, (size_t)A.m, F.nseg) - (double)F.p[i];
      ai = F.a_in[i];
    }
    const int cidx = t - (kSlabThreads - COLS);
    const int jc = strip * COLS + cidx;
    const bool col_thread = cidx >= 0 && jc < A.n;
    double sres = 0.0, bold = 0.0;
    if (col_thread) {
      sres = sum_partials_16(F.colpart_prev + jc, (size_t)A.n, F.ntr) - (double)F.q[jc];
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
      if (cx == 0) A.rowpart[(size_t)strip * A.m + start + r] = rs;
    }
  }
  const float csum = fold(colacc);  // (the barrier inside orders it after every read of the first fold)
  if (t < COLS) {
    const int j = strip * COLS + t;
    if (j < A.n) A.colpart[(size_t)run * A.n + j] = csum;
  }
  if (A.tilesum && t < 64) {  // total of the slab, for the fused update of the next sweep (wave 0)
    const float tot = wave_sum(t < COLS ? csum : 0.f);
    if (t == 0) A.tilesum[run * gridDim.x + strip] = tot;
  }
}

__global__ void fill_kernel(float* __restrict__ dst, size_t count, float value, const int* done) {
  if (done && *done) return;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (size_t)gridDim.x * blockDim.x)
    dst[e] = value;
}

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
  int cgroup;  // 1, or kColGroup: consecutive rows of colpart are first added up in fp32, in groups of that many
};

constexpr int kReduceThreads = 1024;

// First part: the partial sums of 64 entries split 16 ways (share c takes the partials c, c + 16,
// ...), each share added up in order.  NW waves: wave w forms the shares w, w + NW, ... of entry
// idx and leaves them in red[share][lane]; nz_out counts the nonzero partials this wave saw.
template <int NW>
__device__ __forceinline__ void reduce_gather(const ReduceArgs& A, double* red, int& nz_out) {
  static_assert(16 % NW == 0, "the 16 shares are dealt out to the waves");
  const int t = threadIdx.x;
  const int sub = t >> 6, l = t & 63;
  const bool rows = (int)blockIdx.x < A.nbm;
  const int idx = (rows ? (int)blockIdx.x : (int)blockIdx.x - A.nbm) * 64 + l;
  const int len = rows ? A.m : A.n;
  const bool grouped = !rows && A.cgroup == kColGroup;
  const int nparts = rows ? A.nseg : grouped ? (A.ntr + kColGroup - 1) / kColGroup : A.ntr;
  const float* __restrict__ part = rows ? A.rowpart : A.colpart;
  int nz = 0;
  constexpr int kStride = 16, kBatch = 8;
#pragma unroll
  for (int share = sub; share < 16; share += NW) {
    double acc = 0.0;
    if (grouped) {
      // column sums stored per 64-row tile: tiles 4k .. 4k+3 are added first, in fp32 and in order, as
      // the workgroups of the lean sweep do before they store (a tile past the end adds +0)
      constexpr int kGroups = kBatch / 2;
      for (int k0 = share; k0 < nparts; k0 += kStride * kGroups) {
        float v[kGroups][kColGroup];
#pragma unroll
        for (int b = 0; b < kGroups; ++b)
#pragma unroll
          for (int g = 0; g < kColGroup; ++g) {
            const int k = (k0 + b * kStride) * kColGroup + g;
            v[b][g] = (idx < len && k < A.ntr) ? part[(size_t)k * len + idx] : 0.f;
          }
#pragma unroll
        for (int b = 0; b < kGroups; ++b)
          if (k0 + b * kStride < nparts) acc += (double)(((v[b][0] + v[b][1]) + v[b][2]) + v[b][3]);
      }
    }
    for (int k0 = share; !grouped && k0 < nparts; k0 += kStride * kBatch) {  // (nparts and share are wave-uniform)
      // a batch of independent loads, then the additions in the order k0, k0 + 16, ... (one load per
      // trip would wait for memory once per partial sum)
      float v[kBatch];
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        const int k = k0 + b * kStride;
        v[b] = (idx < len && k < nparts) ? part[(size_t)k * len + idx] : 0.f;
      }
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        if (k0 + b * kStride < nparts) acc += (double)v[b];
        nz += __builtin_popcountll(__builtin_amdgcn_ballot_w64(v[b] != 0.f));
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
// sums (a few hundred doubles); workgroup 0 also stores theta+ and the squared residual norms.
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

// The update for all m + n entries by one workgroup (all = true: it strides over them) or for the
// 1024 entries of workgroup `vb` (all = false); the arithmetic per entry is the same either way.
__device__ __forceinline__ void update_body(const UpdateArgs& A, int vb, bool all, double* red) {
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
  const long long total = (long long)A.m + A.n;
  const long long first = all ? t : (long long)vb * kReduceThreads + t;
  const long long step = all ? kReduceThreads : total;  // (all = false: one entry per thread)
  for (long long g = first; g < total; g += step) {
    if (g < A.m) {
      const double r = A.V.r[g], ai = A.a_in[g];
      A.V.phi[g] = (float)((ai - 2.0 * r + cst) / (double)A.n);
      A.a_out[g] = ai - r;
    } else {
      const long long j = g - A.m;
      const double sj = A.V.s[j], bj = A.b_in[j];
      A.V.varphi[j] = (float)((bj - 2.0 * sj + cst) / (double)A.m);
      A.b_out[j] = bj - sj;
    }
  }
  if ((all || vb == 0) && t == 0) A.V.theta[A.par ^ 1] = theta - eta;
}

__global__ __launch_bounds__(kReduceThreads) void update_kernel(UpdateArgs A) {
  if (*A.V.done) return;
  __shared__ double red[kReduceThreads];
  update_body(A, (int)blockIdx.x, false, red);
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
  int tgroup;            // kColGroup: add tile rows 4k .. 4k+3 first; 1: stored that way
};

// The lean sweep's refresh schedule rides along (last workgroup): see ScreenCtl above.
struct ScreenCtlArgs {
  int* ctl;              // the control words
  const int* wg_reads;   // [nwg] what the lean sweep's workgroups read
  int nwg;
  int mode;              // 0: nothing; 1: the sweep was a refresh ordered by the host: start afresh; 2: account for a lean sweep
  int price;             // rent that buys a renewal, in row segments of C
  int max_since;         // renew after this many lean sweeps at the latest
};

// (8 waves: every workgroup of a 40000-entry problem is resident at once.  The tile totals are dealt
// out to 1024 shares whatever the number of threads, share v taking the entries v, v + 1024, ...)
constexpr int kMergedWaves = 8;

__global__ __launch_bounds__(64 * kMergedWaves) void reduce_update_kernel(ReduceArgs A, UpdateArgs U, TileTotals T,
                                                                          ScreenCtlArgs K) {
  // (the stop flag travels with the other loads and is tested before the first store: a test up
  // front would put one more trip to memory ahead of everything)
  const int stop = *A.V.done;
  constexpr int NW = kMergedWaves, kShares = 1024, kPerThread = kShares / (64 * NW);
  __shared__ double red[16 * 64];
  __shared__ double eta_part[kShares / 64];
  __shared__ int nzw[NW];
  __shared__ int readw[NW];
  const int t = threadIdx.x;
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
  // eq. (6) inputs of this thread's entry, fetched early
  const bool rows = (int)blockIdx.x < A.nbm;
  const int idx = (rows ? (int)blockIdx.x : (int)blockIdx.x - A.nbm) * 64 + t;
  const bool owner = t < 64 && idx < (rows ? A.m : A.n);
  const double ab_in = owner ? (rows ? U.a_in[idx] : U.b_in[idx]) : 0.0;
  const double theta = A.V.theta[U.par], sum_p = *A.V.sum_p;
  const float pq = reduce_entry_pq(A);
  // the shares of the tile totals: batches of independent loads, added in index order
  double acc[kPerThread];
#pragma unroll
  for (int s = 0; s < kPerThread; ++s) {
    acc[s] = 0.0;
    const int v0 = t + s * 64 * NW;
    if (T.tgroup == kColGroup) {
      constexpr int kGroups = 4;
      const int ngroups = ((T.tile_rows + kColGroup - 1) / kColGroup) * T.nseg;
      for (int e0 = v0; e0 < ngroups; e0 += kShares * kGroups) {
        float v[kGroups][kColGroup];
#pragma unroll
        for (int b = 0; b < kGroups; ++b) {
          const int e = e0 + b * kShares;
          const int k = e / T.nseg, sg = e - k * T.nseg;
#pragma unroll
          for (int g = 0; g < kColGroup; ++g) {
            const int tr = k * kColGroup + g;
            v[b][g] = (e < ngroups && tr < T.tile_rows) ? T.tilesum[tr * T.nseg + sg] : 0.f;
          }
        }
#pragma unroll
        for (int b = 0; b < kGroups; ++b) acc[s] += (double)(((v[b][0] + v[b][1]) + v[b][2]) + v[b][3]);
      }
    } else {
      constexpr int kBatch = 8;
      const int ngroups = T.tile_rows * T.nseg;
      for (int e0 = v0; e0 < ngroups; e0 += kShares * kBatch) {
        float v[kBatch];
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
          const int e = e0 + b * kShares;
          v[b] = e < ngroups ? T.tilesum[e] : 0.f;
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) acc[s] += (double)v[b];
      }
    }
  }
  int nz;
  reduce_gather<NW>(A, red, nz);
#pragma unroll
  for (int s = 0; s < kPerThread; ++s) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc[s] += __shfl_xor(acc[s], off, 64);
    if ((t & 63) == 0) eta_part[(t >> 6) + s * NW] = acc[s];
  }
  if (keeper) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nread += __shfl_xor(nread, off, 64);
  }
  if ((t & 63) == 0) {
    nzw[t >> 6] = nz;
    readw[t >> 6] = nread;
  }
  __syncthreads();
  if (stop) return;
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
  const double res = reduce_finish<NW>(A, red, nzw, pq);
  if (t >= 64) return;
  double total = 0.0;
  for (int k = 0; k < kShares / 64; ++k) total += eta_part[k];
  const double eta = (total - sum_p) / ((double)A.m + (double)A.n);
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
  if (blockIdx.x == 0 && t == 0) A.V.theta[U.par ^ 1] = theta - eta;
}

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
void launch_resident(const ResidentArgs& RS, hipStream_t stream) {
  const int m = RS.m;
  if (m <= 16) hipLaunchKernelGGL((resident_kernel<1, 16, CPL>), dim3(1), dim3(1024), 0, stream, RS);
  else if (m <= 32) hipLaunchKernelGGL((resident_kernel<2, 16, CPL>), dim3(1), dim3(1024), 0, stream, RS);
  else if (m <= 64) hipLaunchKernelGGL((resident_kernel<4, 16, CPL>), dim3(1), dim3(1024), 0, stream, RS);
  else if constexpr (CPL < 4) hipLaunchKernelGGL((resident_kernel<8, 16, CPL>), dim3(1), dim3(1024), 0, stream, RS);
  else hipLaunchKernelGGL((resident_kernel<16, 8, CPL>), dim3(1), dim3(512), 0, stream, RS);
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
// later kernel of the solve returns at once.
__global__ void status_kernel(VecState V, int iters, double tol) {
  if (*V.done) return;
  const double r2 = V.resid[0], s2 = V.resid[1];
  V.status->r2 = r2;
  V.status->s2 = s2;
  V.status->nz_segments = V.resid[2];
  V.status->iters = iters;
  if (tol > 0.0 && r2 <= tol * tol && s2 <= tol * tol) {
    V.status->converged = 1;
    __threadfence();
    *V.done = 1;
  }
}

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
};

__global__ __launch_bounds__(kBlock) void gap_kernel(GapArgs A) {
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
                                                         int reg_kind, double lambda, double mu) {
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
                            // of 16 M entries and more, 1 always, k >= 2 always and with the bounds renewed at
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
  if (enable)
    for (auto& e : h->prof_ev)
      if (!e && hipEventCreate(&e) != hipSuccess) {
        e = nullptr;
        return DROT_ERR_HIP;
      }
  if (enable)
    for (auto& e : h->cal_ev)
      if (!e && hipEventCreate(&e) != hipSuccess) {
        e = nullptr;
        return DROT_ERR_HIP;
      }
  if (enable && !h->prof_reads) {
    // read counts of the screened sweeps: one int per wave of the largest grid, one total per timed sweep
    const size_t waves = (size_t)ceil_div(h->max_n, kSegCols) * (size_t)ceil_div(h->max_m, kScreenRows * kScreenWaves) * kScreenWaves;
    if (hipMalloc(reinterpret_cast<void**>(&h->wave_reads), sizeof(int) * waves) != hipSuccess) return DROT_ERR_ALLOC;
    h->wave_reads_len = waves;
    if (hipMalloc(reinterpret_cast<void**>(&h->prof_reads), sizeof(double) * kMaxProfiled) != hipSuccess) return DROT_ERR_ALLOC;
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
  const bool adaptive = can_pair && !small && h->skip_cost == -1 && h->skip_unchanged != 0;
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
  if (max_iters == 0 && !resume && !warm)
    hipLaunchKernelGGL(fill_kernel, dim3(1024), dim3(256), 0, stream, X_out, (size_t)m * n, 0.f, (const int*)nullptr);

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
      if (adaptive && !(plan_density >= 0.0 && plan_density < 0.25)) {
        // how sparse the plan is decides the sweep: until it is known to be sparse, have a look after
        // 16, 32 and 64 iterations too (a plan is dense in its first iterations, whatever it becomes:
        // these early readings can move the solver to the lean sweep, never to the even/odd pairs)
        const int next = k < 16 ? 16 : k < 32 ? 32 : k < 64 ? 64 : 0;
        if (next > 0 && next - k < chunk) {
          chunk = next - k;
          probe = true;
        }
      }
    }
    const bool skip_cost = can_pair && (h->skip_cost == 1 || (adaptive && dense_plan));
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
        // (automatic: from 16 M entries up; below that the whole of C streams from the caches as fast)
        const bool screened = mode == 0 && tall && !first &&
                              (h->screening > 0 || (h->screening == -1 && (size_t)m * (size_t)n >= ((size_t)1 << 24)));
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
          if (refresh) {
            DROT_HIP(hipMemcpyAsync(h->varphi0, h->varphi, sizeof(float) * (size_t)n, hipMemcpyDeviceToDevice, stream));
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
          if (density > 0.7 && !was_probe[slot ^ 1]) dense_plan = true;
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
  h->epoch_gen = epoch_gen;
  h->refresh_period = refresh_period;
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
