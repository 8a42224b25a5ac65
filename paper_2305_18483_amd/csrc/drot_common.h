// Constants, wave-level helpers and the device-side state shared by all kernels.
// Part of drot.hip (included there, inside its anonymous namespace, in this order); not a stand-alone header.

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

// A word every lane needs, fetched through the vector memory path (an atomic load is never made a scalar one).
// Scalar loads share their counter with the LDS operations and the kernel arguments, and waiting on that counter
// waits for all of them: a flag fetched that way sits in front of the first wait for an argument, one trip to
// memory ahead of every other load.  These count with the vector loads and arrive with them.
__device__ __forceinline__ int vector_load_uniform(const int* p) {
  return __builtin_amdgcn_readfirstlane(__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
}
__device__ __forceinline__ double vector_load_uniform(const double* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

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

// The same from the solver's own varphi buffers (workspace and the screening epoch's copy), which are
// allocated up to the end of the last 256-column segment and hold the mask value past n (set at the
// start of every solve): one 128-bit load, no edge case.
__device__ __forceinline__ f4v load_varphi_padded(const float* __restrict__ varphi, int j0) {
  return *reinterpret_cast<const f4u*>(varphi + j0);
}

// |v| of a varphi entry, 0 for the mask value of the columns past n.
__device__ __forceinline__ float unmasked_abs(float v) { return v == kMaskedOut ? 0.f : fabsf(v); }

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
  int gap_iters;                 // iteration the objective / gap / dual residual above belong to (0: none yet)
  int pad_;
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
  int mp, np;            // pitches of the arrays kept per row segment ([segment][mp]: sums, bounds, line flags) and of
                         // the rows of column sums ([tile row][np]): m and n rounded up to 64, so that a wave's 64
                         // consecutive entries never straddle one 128-byte line more than they must
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

// Launch with, in profile mode, a pair of events that take the kernel's own start and end as the hardware stamps
// them (the HIP extension launch); without events the plain launch, which is also what a stream capture accepts.
template <typename... KArgs, typename... Args>
inline void launch_timed(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream, hipEvent_t e0, hipEvent_t e1,
                         Args&&... args) {
  if (e0 || e1) hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, e0, e1, 0, static_cast<KArgs>(args)...);
  else hipLaunchKernelGGL(kernel, grid, block, 0, stream, static_cast<KArgs>(args)...);
}
