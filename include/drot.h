/*
 * drot.h -- C ABI of the MI355X (gfx950) Douglas-Rachford solver for regularized discrete
 * optimal transport
 *
 *        minimise  <C,X> + h(X)   subject to  X 1_n = p,  X^T 1_m = q,  X >= 0      (problem (1))
 *
 * with h in {0, (lambda/2)||X||_F^2, mu*sum_g ||X_g||_2 + (lambda/2)||X||_F^2} (Section 3:
 * quadratic and group-lasso regularization; groups g = (class of source row, target column)).
 *
 * Every iteration is one sweep over the m x n plan (eq. (8): X <- prox_{rho h}([X + phi 1^T +
 * 1 varphi^T - rho C]_+), fused with the row and column sums) followed by the O(m+n) vector
 * recursion of eq. (6).  All of it runs in hand-written HIP kernels on the caller's stream.
 *
 * Conventions
 *   - All matrix pointers are DEVICE pointers to row-major fp32 arrays with pitch n (no padding).
 *     Any m, n >= 1 and any 4-byte-aligned base address are accepted; 16-byte alignment and
 *     n % 4 == 0 are not required.
 *   - The caller owns C, p, q, X_out, row_class and the point clouds; the library never frees or
 *     reallocates them and never writes C, p, q, row_class.  The handle owns only workspace
 *     (including, for unaligned problems, padded working copies of C and X: 8*m*ceil32(n) bytes).
 *   - Preconditions that are NOT checked (they would need a pass over the data): p, q >= 0 with
 *     sum(p) = sum(q) = 1, C >= 0 and finite, labels in range.  The stepsize default assumes
 *     max(C) = 1 ("Stepsize selection").
 *   - Return value: 0 = DROT_OK, 1 = DROT_MAX_ITERS (ran out of iterations before reaching tol;
 *     a status, the outputs are valid), negative = error, nothing was computed.  No exceptions
 *     cross the boundary.  One solve at a time per handle; different handles are independent.
 *   - drot_solve* return after the stream work they enqueued has completed (they synchronise
 *     with `stream` only), so X_out and drot_get_info are valid on return.
 */
#ifndef DROT_H_
#define DROT_H_

#ifdef __cplusplus
extern "C" {
#endif

typedef struct drot_handle_s* drot_handle;

typedef enum {
  DROT_REG_NONE = 0,        /* h = 0                                   (eq. (5))            */
  DROT_REG_QUADRATIC = 1,   /* h = (lambda/2)||X||_F^2                 (Quadratic Regularization) */
  DROT_REG_GROUP_LASSO = 2  /* h = mu sum_g ||X_g||_2 + (lambda/2)||X||_F^2 (Group Lasso Regularization) */
} drot_reg_kind;

enum {
  DROT_OK = 0,
  DROT_MAX_ITERS = 1,
  DROT_ERR_INVALID_ARG = -1,
  DROT_ERR_ALLOC = -2,
  DROT_ERR_HIP = -3,
  DROT_ERR_NOT_INITIALIZED = -4,
  DROT_ERR_TOO_LARGE = -5
};

/* Regularizer parameters; HOST struct, read during the call. */
typedef struct {
  float lambda;          /* weight of (lambda/2)||X||_F^2, >= 0; used by QUADRATIC and GROUP_LASSO */
  float mu;              /* group-lasso weight, >= 0; GROUP_LASSO only                              */
  int num_classes;       /* GROUP_LASSO only: number of row classes, >= 1                           */
  const int* row_class;  /* GROUP_LASSO only: DEVICE pointer, m labels in [0, num_classes)          */
  const float* weights;  /* any kind (stored cost only): NULL, or DEVICE pointer to m*n weights
                            w_ij >= 0, row-major, of an added weighted l1 term sum w_ij |X_ij|
                            (Section 2, list of sparsity promoting regularizers)                     */
} drot_reg_params;

/*
 * Constrained OT (same list: h = indicator{X_ij = 0 for (i,j) in S}) needs no parameter: set
 * C_ij = +INFINITY for the pairs of S.  Every sweep then leaves X_ij = 0 there, the pair adds
 * nothing to <C,X>, and its dual constraint is vacuous.  Combines with every regularizer kind.
 * Weighted l1: on X >= 0 the term equals <W,X>, so the solve runs on a working copy C + W that the
 * library forms once per call (one extra pass, m*n floats of workspace); drot_info.objective
 * counts <W,X> as part of h.  Not available with drot_solve_points.
 */

/* Result of the last solve on a handle (host struct). */
typedef struct {
  int iters;         /* iterations performed (index of the returned iterate X_iters)             */
  int converged;     /* 1 if the residual test passed, else 0                                    */
  float r_row;       /* ||X 1_n - p||_2 of the returned iterate (Appendix C, r_primal)           */
  float r_col;       /* ||X^T 1_m - q||_2                                                        */
  double objective;  /* <C,X> + h(X)                        (filled when the gap was requested)  */
  double gap;        /* duality gap of (X, phi, varphi), Appendix C                              */
  double dual_res;   /* dual constraint violation where h* is an indicator, else 0               */
} drot_info;

/*
 * Create a solver for problems up to max_m x max_n on the current HIP device.  Allocates the
 * O(m+n) vectors, the partial-sum buffers of the fused reductions and a pinned status block.
 * Errors: INVALID_ARG (null out, sizes < 1), ALLOC, HIP.
 */
int drot_create(drot_handle* out, int max_m, int max_n);

/* Free the workspace.  A null handle is DROT_ERR_INVALID_ARG. */
int drot_destroy(drot_handle h);

/*
 * Options: drot_set_option(h, option, value); defaults in brackets.  INVALID_ARG for a null handle, an
 * unknown option or a value outside the stated range.
 *
 * How the solve is run
 *   DROT_OPT_CHECK_EVERY [100], >= 1: the residual test of Appendix C (r_primal) is evaluated on the
 *       device every this many iterations; the solve stops at the first test that passes.
 *   DROT_OPT_COMPUTE_GAP [1], 0/1: evaluate objective, duality gap and dual residual of the returned
 *       iterate (Appendix C; one read-only pass over X and C at the end of the solve, or, where screening
 *       bounds certify that a row segment adds nothing to any of the sums, over the other row segments
 *       only: the same numbers, bit for bit).
 *   DROT_OPT_GAP_EVERY [0], >= 0: k >= 1 evaluates objective, duality gap and dual residual also during
 *       the solve, at every k-th residual check (iterations that are multiples of k * check_every), and
 *       records them (drot_get_checks); 0: only at the end.  See drot_set_gap_tolerance.
 *   DROT_OPT_CONTINUE [0], 0/1: the next drot_solve / drot_solve_points does not restart from X_0 = 0: it
 *       resumes the iteration from the state the previous solve on this handle left (phi, varphi and the
 *       running sums of eq. (6) in the workspace, the plan in X_out, which must still hold that solve's
 *       output; same m, n, C, p, q and regularizer are the caller's responsibility).  Running K1 then K2
 *       iterations this way gives bit for bit the iterate of one K1+K2 solve, unless the automatic
 *       even/odd scheme (DROT_OPT_SKIP_COST) comes into play: when it starts depends on where the calls
 *       and their stretches of check_every iterations begin.  INVALID_ARG at the next solve if no solve
 *       has run or the sizes differ.  drot_info.iters counts the iterations of the call.
 *   DROT_OPT_PROFILE [0], 0/1: take the start and the end of every sweep kernel (the first 256 of a solve),
 *       as the hardware stamps them, through a pair of HIP events attached to the launch, and count what the
 *       sweep read; see drot_get_profile.  Costs a few tiny kernels per iteration, so leave it off when
 *       timing a solve.
 *
 * Which kernels run (tuning; the iterates do not depend on these unless stated)
 *   DROT_OPT_SKIP_UNCHANGED [-1 = on], -1/0/1: X >= 0, so a row segment (256 consecutive columns of a
 *       row) whose sum after the previous sweep was zero holds only zeros; the sweep then does not read
 *       that segment of X, and does not write it back if it stays zero.  Transport plans are sparse: once
 *       the support has settled the sweep is a read-only stream of C (4 instead of 12 bytes per element).
 *       Beyond the fused small-problem path these sweeps run on 64-row tiles.  The group-resident
 *       group-lasso sweep does the same with 128-byte lines, the sweep of drot_solve_points with row
 *       segments.  Same memory contents either way.  0 reads and stores everything.
 *   DROT_OPT_SCREENING [-1], -1 .. 100000: with the skipping on, sweeps over large sparse plans also leave
 *       out most reads of C.  Now and then a sweep records, per row segment, the largest of
 *       varphi_j - rho C_ij, a column that attains it and the largest over the other columns; until the next
 *       such sweep these bound phi_i + varphi_j - rho C_ij over the segment from above (the recorded column
 *       moves by its own drift of varphi since then, the others by at most the largest drift), and a row
 *       segment whose X is zero and whose bound, plus a margin for the fp32 roundings involved, is not
 *       positive is known to stay zero: nothing of it is read, computed or written.  The iterates are those
 *       of the unscreened sweeps, bit for bit.  The bounds are renewed after 8, 16, 32, ... sweeps at first,
 *       at most 1024 apart; once the plan is known to be sparse the sweep itself decides, on the device,
 *       when the reads that weakened bounds cost it have added up to the price of new ones.  -1 screens problems of 11.5 million entries
 *       and more (smaller ones stream all of C from the caches just as fast), 1 every problem the skipping
 *       applies to, k >= 2 the same with the bounds renewed at least every k-th sweep, 0 never.
 *   DROT_OPT_SKIP_COST [-1], -1/0/1: the even/odd scheme of the paper's GPU appendix (Section
 *       "Quadratically Regularized DROT"): sweeps pair up, the first of a pair stores X - rho*C, the second
 *       reads that and needs no C (20 instead of 24 bytes per element and pair).  Row and column sums are
 *       always those of X itself, and X_out is the plain plan on return and at every residual check.  The
 *       rounding differs slightly from the plain scheme (same tolerance against the fp64 iteration).
 *       Applies to the none/quadratic sweeps over a stored cost whose vector update is not fused into the
 *       sweep; the better scheme for dense plans, as the skipping is for sparse ones.  -1 follows the plan:
 *       the reduction counts the nonzero row segments, the host reads the count with the status of every
 *       stretch (one stretch late, without waiting) and switches to the pairs above 70 % nonzero segments
 *       and back below 50 %; with a switch the result depends, within rounding, on check_every and on how a
 *       solve is cut into continued calls.  1: pairs wherever they apply; 0: never.
 *   DROT_OPT_FUSED_UPDATE [-1], -1/0: small problems (at most 2048 rows and 4096 tiles of 32 x 256) compute
 *       the O(m+n) update of eq. (6) at the head of the next sweep, one launch per iteration instead of
 *       three; 0 always runs the separate kernels.  Same bits.
 *   DROT_OPT_RESIDENT [-1], -1/0: problems of at most 128 x 256 without group lasso, from a stored cost, run
 *       in a single workgroup that keeps X and C in registers: all the iterations up to the next residual
 *       check are one launch.  Agrees with the other paths to rounding (different summation order).
 *   DROT_OPT_GROUP_TWO_PASS [0], 0/1: a group-lasso solve uses the group-resident kernel (a whole class x
 *       32 columns in one workgroup's registers, 12 bytes per element) when every class is one run of at
 *       most 1024 consecutive rows, and otherwise the two-pass path (any labels, 20 bytes per element);
 *       1 forces the two-pass path.
 *   DROT_OPT_NONTEMPORAL [-1], -1/0/1: mark the sweep's loads and stores of X and C non-temporal (best when
 *       they are far larger than the caches); -1 decides from 8*m*n bytes.  Same results.
 */
typedef enum {
  DROT_OPT_CHECK_EVERY = 0,
  DROT_OPT_COMPUTE_GAP = 1,
  DROT_OPT_GAP_EVERY = 2,
  DROT_OPT_CONTINUE = 3,
  DROT_OPT_PROFILE = 4,
  DROT_OPT_SKIP_UNCHANGED = 5,
  DROT_OPT_SCREENING = 6,
  DROT_OPT_SKIP_COST = 7,
  DROT_OPT_FUSED_UPDATE = 8,
  DROT_OPT_RESIDENT = 9,
  DROT_OPT_GROUP_TWO_PASS = 10,
  DROT_OPT_NONTEMPORAL = 11
} drot_option;

int drot_set_option(drot_handle h, drot_option option, int value);

/*
 * Stopping on the duality gap as well [0 = off] (Section 3, "Stopping criteria"; Appendix C).  With
 * gap_tol > 0 a check passes only if, besides the residual test, the gap was evaluated at that check
 * (DROT_OPT_GAP_EVERY, taken as 1 if it is 0) and
 *     |gap| <= gap_tol * |objective|   and   dual_res <= gap_tol
 * (the dual residual, where the conjugate of h is an indicator, is a norm of a violation in units of
 * the cost, which the stepsize default assumes normalised to max(C) = 1; it is 0 for the quadratic
 * term).  The residual test alone says nothing about optimality: with a weak quadratic term the
 * conjugate ||W||_F^2 / (2 lambda) magnifies any dual infeasibility left.  INVALID_ARG for a negative
 * or NaN tolerance.
 */
int drot_set_gap_tolerance(drot_handle h, float gap_tol);

/*
 * The residual checks of the last solve, in order: the status block of every check, as the host read
 * it (each check once; after a stop the checks queued behind it do not run).
 */
typedef struct {
  int iters;           /* iteration of the check (counted within the call)                           */
  int gap_evaluated;   /* 1 if objective, gap and dual_res below were evaluated at this very check     */
  float r_row, r_col;  /* the two residual norms of Appendix C                                         */
  double objective, gap, dual_res;
} drot_check;
/* out [out] HOST, capacity entries; *count receives how many checks the solve made (at most
 * min(capacity, *count) entries are written; the library keeps the first 65536). */
int drot_get_checks(drot_handle h, drot_check* out, int capacity, int* count);

/*
 * Sweep timings of the last solve in profile mode, in launch order (at most the first 256 sweeps).
 *   ms          duration of the sweep kernel: from its start to its end as the hardware stamps them, read
 *               through a pair of HIP events attached to the launch (the group-lasso sweep of three
 *               launches: from the start of the first to the end of the last)
 *   kind        0 = read X and C, stored X (32-row tiles; also the group-lasso sweeps), 1 = also stored
 *               X - rho*C (first of an even/odd pair), 2 = read the shifted X and no C (second of a pair),
 *               3 = a launch of the resident kernel (its duration divided by the iterations it ran),
 *               4 = as 0 on 64-row tiles with the zero-segment skipping, 5 = the same with screening,
 *               6 = a screening sweep that reads all of C and records the bounds, 7 = the screened sweep
 *               for plans known to be sparse (one wave per tile), 8 = the screened sweep of
 *               drot_solve_points (cost formed only for the row segments no bound covers), 9 = a full
 *               sweep of drot_solve_points that also records the bounds
 *   c_fraction  fraction of the row segments of C (256 columns of one row) the sweep read (kind 8: formed):
 *               counted by the kernel for kinds 5 to 8; 1 for the kinds that take all of C, 0 for kind 2
 *   x_fraction  fraction of the row segments of X that hold a nonzero after the sweep (counted by the
 *               vector update that follows it), or -1 where that update is fused into the next sweep
 */
typedef struct {
  float ms;
  int kind;
  double c_fraction;
  double x_fraction;
} drot_sweep_timing;
int drot_get_profile(drot_handle h, drot_sweep_timing* out, int capacity, int* count);

/*
 * Solve problem (1) by the iteration of eq. (8) + eq. (6), starting from X_0 = 0 and the
 * phi_0, varphi_0 of the Initialization paragraph.
 *
 *   C [in]      DEVICE, m*n fp32 row-major, the cost
 *   p, q [in]   DEVICE, m resp. n fp32, the marginals
 *   stepsize    rho; <= 0 selects 2/(m+n) ("Stepsize selection")
 *   reg_kind, reg_params   the regularizer; reg_params may be NULL for DROT_REG_NONE
 *   max_iters   >= 0; with tol <= 0 exactly max_iters iterations are run
 *   tol         stop when max(||X1-p||_2, ||X^T1-q||_2) <= tol at a check (eq. "stopping criteria")
 *   X_out [out] DEVICE, m*n fp32 row-major; contents on entry ignored.  It is the iterate buffer
 *               itself when n % 32 == 0 and the address is a multiple of 128; otherwise the
 *               library iterates on an internal copy with padded rows (and likewise reads C
 *               from a padded copy), and writes X_out once at the end
 *   stream      hipStream_t (as void*); NULL = the default stream
 *
 * Errors: INVALID_ARG (null pointers, m/n outside [1, max], negative max_iters or weights,
 * unknown reg_kind, GROUP_LASSO without labels or with a label outside [0, num_classes): the
 * labels are copied to the host and checked at the start of a group-lasso solve), ALLOC, HIP.
 */
int drot_solve(drot_handle h, const float* C, const float* p, const float* q, int m, int n,
               float stepsize, drot_reg_kind reg_kind, const drot_reg_params* reg_params,
               int max_iters, float tol, float* X_out, void* stream);

/*
 * On-the-fly cost: like drot_solve, but the cost is C_ij = cost_scale * ||xs_i - xt_j||_2^2 for two
 * point clouds and is recomputed in every sweep instead of being read from memory (8 instead of 12
 * bytes per element of HBM traffic, 2d flops per element on the matrix cores; no m x n cost array).
 *   xs [in]  DEVICE, m*d fp32 row-major (source points), xt [in] DEVICE, n*d fp32 (target points), d >= 1
 *   cost_scale > 0; 1/max_ij ||xs_i - xt_j||^2 gives the normalisation the stepsize default assumes
 * The cost is evaluated in fp32 as cost_scale*max(|xs_i|^2 + |xt_j|^2 - 2 xs_i.xt_j, 0) (squared
 * norms accumulated in fp64), so it agrees with a stored fp32 cost to a few 1e-7 absolute, and the
 * iterates agree with the stored-cost solve to that perturbation accumulated over the iterations.
 * With DROT_OPT_SKIP_UNCHANGED on (the default) the sweeps screen as the stored-cost sweeps do: every
 * full sweep records, per row segment, the bound max_j (varphi_j - rho C_ij) in the arithmetic it
 * sweeps with, and once the plan is sparse a lean sweep forms the cost (on the matrix cores, 16
 * gathered rows at a time, operand for operand as the full sweep does) only for the row segments the
 * bound does not certify to stay zero.  Bit for bit the iterates of the sweep that forms every cost.
 * DROT_REG_NONE and DROT_REG_QUADRATIC only, and no weighted l1 term (INVALID_ARG): a weight matrix
 * is m*n floats that every sweep would have to read, which is the traffic of the stored cost this
 * entry point exists to avoid (add the weights to a stored C and call drot_solve); the group-lasso
 * sweeps keep a class's rows of one column strip in registers or make two passes over X and C, and
 * have no variant that forms the cost.  Other arguments, results and errors as drot_solve.
 */
int drot_solve_points(drot_handle h, const float* xs, const float* xt, int d, float cost_scale,
                      const float* p, const float* q, int m, int n, float stepsize,
                      drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters,
                      float tol, float* X_out, void* stream);

/*
 * Warm start: like drot_solve, but the iteration starts from a caller-supplied point instead of
 * X_0 = 0 and the constants of the Initialization paragraph (which the paper offers as one choice;
 * the iteration converges from any start).  On entry X_inout holds X_0 (m*n, entries >= 0) and
 * phi0[m], varphi0[n] (DEVICE, read only) hold phi_0, varphi_0; the iteration starts at
 * Y_0 = X_0 + phi_0 1^T + 1 varphi_0^T (eq. (5)).  On return X_inout holds the new plan.  Feeding
 * back the X_out, phi, varphi of an earlier solve continues that solve (to rounding); potentials
 * of a related problem give a head start (the paper's remark on better dual initialisations).
 * Costs one extra read of X.  Errors as drot_solve, plus INVALID_ARG for null phi0 / varphi0.
 */
int drot_solve_warm(drot_handle h, const float* C, const float* p, const float* q, int m, int n,
                    float stepsize, drot_reg_kind reg_kind, const drot_reg_params* reg_params,
                    int max_iters, float tol, float* X_inout, const float* phi0, const float* varphi0,
                    void* stream);

/*
 * Warm start with the on-the-fly cost: drot_solve_points from the point (X_0, phi_0, varphi_0), with
 * X_inout, phi0, varphi0 as in drot_solve_warm and everything else as in drot_solve_points.
 */
int drot_solve_points_warm(drot_handle h, const float* xs, const float* xt, int d, float cost_scale,
                           const float* p, const float* q, int m, int n, float stepsize,
                           drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters,
                           float tol, float* X_inout, const float* phi0, const float* varphi0,
                           void* stream);

/*
 * For callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: drot_solve without a handle.  The workspace is a fixed array inside the
 * library's code object (6 MiB, held by every GPU the library runs on until the process ends), so the call
 * allocates nothing, on the device or the host; it only enqueues kernels on `stream` and returns WITHOUT
 * waiting for them.  Results arrive in the caller's DEVICE buffers once the stream has run:
 *   X_out [out]       DEVICE, m*n, as drot_solve
 *   phi_out, varphi_out [out]  DEVICE, m resp. n floats, or NULL: phi and varphi of the returned iterate
 *   info_out [out]    DEVICE pointer to one drot_info (all fields, the gap ones included), or NULL
 * Limits: m <= DROT_STATIC_MAX_M and n <= DROT_STATIC_MAX_N, else DROT_ERR_TOO_LARGE; DROT_REG_NONE or
 * DROT_REG_QUADRATIC without weights; n % 32 == 0 and C, X_out at addresses that are multiples of 128 (the
 * padded working copies other shapes need are allocations), else DROT_ERR_INVALID_ARG.  Defaults of every
 * option of drot_set_option; residual test every 100 iterations.  The host never looks at the status block,
 * so the whole schedule is fixed when the call returns: the work enqueued is proportional to max_iters even
 * if the tolerance is reached early (the sweeps behind the stop return at once), and the sweeps are the ones
 * that need no report on the plan's density (no even/odd pairs, no lean sweep; same iterates as drot_solve
 * unless that switches to the even/odd pairs).  The return value says whether the work was enqueued (DROT_OK),
 * not whether the tolerance was reached: read info_out.
 * All calls on one GPU share the one workspace, which keeps the last call's contents (everything that must
 * start from zero is cleared by the call): calls that overlap on one GPU -- from two streams or two threads --
 * race; calls on different GPUs are independent.
 */
#define DROT_STATIC_MAX_M 4096
#define DROT_STATIC_MAX_N 4096
int drot_solve_static(const float* C, const float* p, const float* q, int m, int n, float stepsize,
                      drot_reg_kind reg_kind, const drot_reg_params* reg_params, int max_iters, float tol,
                      float* X_out, float* phi_out, float* varphi_out, drot_info* info_out, void* stream);

/* Results of the last solve (host struct).  NOT_INITIALIZED if no solve has run. */
int drot_get_info(drot_handle h, drot_info* out);

/*
 * Copy phi (m floats) and varphi (n floats) of the last solve into DEVICE buffers; u = phi/rho,
 * v = varphi/rho estimate the dual potentials (Appendix C).  Either pointer may be NULL.
 */
int drot_get_duals(drot_handle h, float* phi_out, float* varphi_out);

/* Human-readable text for a return code. */
const char* drot_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DROT_H_ */
