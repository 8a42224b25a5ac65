/*
 * drot_oracle.c -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, fp64 CPU implementation of the Douglas-Rachford iteration for regularized
 * discrete optimal transport
 *
 *        min <C,X> + h(X)   s.t.  X 1_n = p,  X^T 1_m = q,  X >= 0          (problem (1))
 *
 * written from the paper in its three-update form (eq. (4)) with explicit m x n iterates
 * X, Y and Z.  It exists to check the HIP solver; it shares no code with it.  Only tests, the
 * smoke check and the cpu_baseline leg of the benchmark may call it.
 *
 * Pins (tests/test_oracle_*.py): closed-form affine projection vs. a dense least-squares solve;
 * unregularized optimum vs. brute force over permutations and vs. an LP solver; quadratic case
 * vs. its KKT system and an L-BFGS solve of the smooth dual; group-lasso prox vs. a numerical
 * minimiser and its textbook special cases; the entrywise terms (weighted l1, constrained OT)
 * vs. a numerical minimiser of the prox objective and vs. LPs with shifted cost resp. fixed zeros; the O(m+n) vector recursion the paper prints as
 * eq. (6) vs. the explicit iteration here; feasibility, nonnegativity, duality gap -> 0.
 * The exact iterates after K steps have no printed example in the paper: that part of parity is
 * "unpinned by the paper" and rests on this file being the definition written out.
 *
 * Layout: all matrices row-major, m rows, n columns, pitch n.  C is read as fp32 (the array
 * the GPU gets) and widened per element; everything else is fp64.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_REG_NONE 0
#define ORACLE_REG_QUADRATIC 1
#define ORACLE_REG_GROUP_LASSO 2

/* Number of threads the parallel loops below use (for reporting the CPU baseline). */
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Row sums rs[i] = sum_j A_ij and column sums cs[j] = sum_i A_ij, each a left-to-right sum. */
void oracle_row_col_sums(const double* A, int m, int n, double* rs, double* cs) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < m; ++i) {
    double acc = 0.0;
    for (int j = 0; j < n; ++j) acc += A[(size_t)i * n + j];
    rs[i] = acc;
  }
  /* one thread per block of columns, rows visited in order: deterministic */
#pragma omp parallel for schedule(static)
  for (int jb = 0; jb < n; jb += 256) {
    int je = jb + 256 < n ? jb + 256 : n;
    for (int j = jb; j < je; ++j) cs[j] = 0.0;
    for (int i = 0; i < m; ++i)
      for (int j = jb; j < je; ++j) cs[j] += A[(size_t)i * n + j];
  }
}

/*
 * Projection onto the affine set {Z : Z 1_n = p, Z^T 1_m = q} (the prox of g in the split of
 * Section 2.1).  The paper uses it without printing it; minimising ||Z - V||_F under the two
 * sets of sum constraints gives a correction of the form a 1^T + 1 b^T:
 *     r = V 1_n - p,  s = V^T 1_m - q,  eta = (1^T r)/(m+n)
 *     Z = V - (1/n)(r - eta 1_m) 1_n^T - (1/m) 1_m (s - eta 1_n)^T.
 * corr_row / corr_col (optional) receive the two correction vectors -(r-eta)/n and -(s-eta)/m.
 * Z may alias V.
 */
void oracle_project_marginals(const double* V, int m, int n, const double* p, const double* q,
                              double* Z, double* corr_row, double* corr_col) {
  double* r = (double*)malloc(sizeof(double) * (size_t)m);
  double* s = (double*)malloc(sizeof(double) * (size_t)n);
  oracle_row_col_sums(V, m, n, r, s);
  double sum_r = 0.0;
  for (int i = 0; i < m; ++i) { r[i] -= p[i]; sum_r += r[i]; }
  for (int j = 0; j < n; ++j) s[j] -= q[j];
  const double eta = sum_r / (double)(m + n);
  for (int i = 0; i < m; ++i) r[i] = -(r[i] - eta) / (double)n;
  for (int j = 0; j < n; ++j) s[j] = -(s[j] - eta) / (double)m;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) Z[(size_t)i * n + j] = V[(size_t)i * n + j] + r[i] + s[j];
  if (corr_row) memcpy(corr_row, r, sizeof(double) * (size_t)m);
  if (corr_col) memcpy(corr_col, s, sizeof(double) * (size_t)n);
  free(r);
  free(s);
}

/*
 * prox_{rho h} applied to a nonnegative matrix Xbar, in place (Section 3).
 *   none:       identity
 *   quadratic:  h = (lambda/2)||X||_F^2        ->  Xbar / (1 + rho*lambda)
 *   group lasso (+ quadratic): h = mu * sum_g ||X_g||_2 + (lambda/2)||X||_F^2 with
 *       g = (class of row i, column j); block soft-threshold with threshold rho*mu, then the
 *       quadratic scaling:  X_g = max(1 - rho*mu/||Xbar_g||, 0) / (1 + rho*lambda) * Xbar_g,
 *       and X_g = 0 when ||Xbar_g|| = 0.
 * scratch: num_classes*n doubles (group lasso only).
 */
void oracle_prox_h(double* Xbar, int m, int n, double rho, int reg_kind, double lambda, double mu,
                   const int* row_class, int num_classes, double* scratch) {
  if (reg_kind == ORACLE_REG_NONE) return;
  if (reg_kind == ORACLE_REG_QUADRATIC) {
    const double denom = 1.0 + rho * lambda;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < n; ++j) Xbar[(size_t)i * n + j] /= denom;
    return;
  }
  /* group lasso: squared norm of every (class, column) group, rows visited in order */
  double* t = scratch;
#pragma omp parallel for schedule(static)
  for (int jb = 0; jb < n; jb += 256) {
    int je = jb + 256 < n ? jb + 256 : n;
    for (int c = 0; c < num_classes; ++c)
      for (int j = jb; j < je; ++j) t[(size_t)c * n + j] = 0.0;
    for (int i = 0; i < m; ++i) {
      const int c = row_class[i];
      for (int j = jb; j < je; ++j) {
        const double v = Xbar[(size_t)i * n + j];
        t[(size_t)c * n + j] += v * v;
      }
    }
  }
  const double thr = rho * mu, denom = 1.0 + rho * lambda;
  for (size_t g = 0; g < (size_t)num_classes * n; ++g) {
    const double nrm = sqrt(t[g]);
    double sc = 0.0;
    if (nrm > 0.0) {
      sc = 1.0 - thr / nrm;
      if (sc < 0.0) sc = 0.0;
    }
    t[g] = sc / denom;
  }
#pragma omp parallel for schedule(static)
  for (int i = 0; i < m; ++i) {
    const int c = row_class[i];
    for (int j = 0; j < n; ++j) Xbar[(size_t)i * n + j] *= t[(size_t)c * n + j];
  }
}

/*
 * The two further members of the class of Section 2 that act entry by entry, applied to a
 * nonnegative matrix Xbar in place, before oracle_prox_h:
 *   weighted l1, h = sum w_ij |X_ij| with w >= 0 (W != NULL): the soft-threshold
 *       sign(x) max(|x| - rho w, 0), which for x >= 0 is max(x - rho w, 0);
 *   constrained OT, h = indicator{X_ij = 0 for (i,j) in S} (forbidden != NULL, nonzero marks S):
 *       the projection, X_ij = 0 on S.
 * Both leave the matrix nonnegative, and the prox of their sum with the quadratic or the
 * group-lasso term is the composition in this order (entrywise shrinkage first, then the group
 * shrinkage and scaling); a test checks that against a numerical minimiser.
 */
void oracle_prox_entrywise(double* Xbar, int m, int n, double rho, const float* W,
                           const unsigned char* forbidden) {
  if (!W && !forbidden) return;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) {
      const size_t e = (size_t)i * n + j;
      double x = Xbar[e];
      if (W) {
        x -= rho * (double)W[e];
        if (x < 0.0) x = 0.0;
      }
      if (forbidden && forbidden[e]) x = 0.0;
      Xbar[e] = x;
    }
}

/*
 * The iteration, eq. (4) with the split of eq. (7):
 *     X_{k+1} = prox_{rho f}(Y_k) = prox_{rho h}([Y_k - rho C]_+)         (Lemma 3.1, eq. (8))
 *     Z_{k+1} = P(2 X_{k+1} - Y_k)                                         (projection above)
 *     Y_{k+1} = Y_k + Z_{k+1} - X_{k+1}.
 * Start: Y_0 = X_0 + phi_0 1^T + 1 varphi_0^T (eq. (5)); X0 == NULL means X_0 = 0.
 * Since Y_{k+1} - X_{k+1} = Z_{k+1} - (2X_{k+1} - Y_k), the vectors phi_{k+1}, varphi_{k+1}
 * of eq. (5) are the projection's two correction vectors; they are returned for the last step.
 *
 * Stopping (Section 3 "Stopping criteria", Appendix C): r = X 1 - p, s = X^T 1 - q, stop when
 * max(||r||_2, ||s||_2) <= tol, tested only at iterations that are multiples of check_every
 * (tol <= 0: never).  With gap_every >= 1 the objective, the duality gap and the dual residual of
 * (X_k, phi_k, varphi_k) are evaluated at every gap_every-th of those tests (oracle_objective_gap
 * below) and written to gap_trace (optional; 4 doubles per evaluation: k, objective, gap, dual
 * residual; capacity gap_trace_cap evaluations, *gap_trace_len receives their number); with
 * gap_tol > 0 a test then passes only if the gap was evaluated at it and
 * |gap| <= gap_tol * |objective| and dual residual <= gap_tol.
 * res_trace (optional, 2*max_iters doubles): ||r||_2, ||s||_2 of every iterate.
 * W, forbidden (optional): the entrywise terms of oracle_prox_entrywise, added to h.
 * Returns the number of iterations done, or -1 if memory ran out.
 */
void oracle_objective_gap(const float* C, const double* X, const double* p, const double* q,
                          const double* phi, const double* varphi, int m, int n, double rho,
                          int reg_kind, double lambda, double mu, const int* row_class,
                          int num_classes, const float* Wl1, const unsigned char* forbidden,
                          double* out);

int oracle_drot_solve(const float* C, const double* p, const double* q, int m, int n, double rho,
                      int reg_kind, double lambda, double mu, const int* row_class, int num_classes,
                      const float* W, const unsigned char* forbidden,
                      const double* X0, const double* phi0, const double* varphi0,
                      int max_iters, double tol, int check_every, int gap_every, double gap_tol,
                      double* X_out, double* Y_out, double* phi_out, double* varphi_out,
                      double* res_trace, double* gap_trace, int gap_trace_cap, int* gap_trace_len) {
  const size_t mn = (size_t)m * n;
  double* X = X_out;
  double* Y = (double*)malloc(sizeof(double) * mn);
  double* V = (double*)malloc(sizeof(double) * mn);
  double* rs = (double*)malloc(sizeof(double) * (size_t)m);
  double* cs = (double*)malloc(sizeof(double) * (size_t)n);
  double* gscratch = NULL;
  if (reg_kind == ORACLE_REG_GROUP_LASSO)
    gscratch = (double*)malloc(sizeof(double) * (size_t)num_classes * n);
  if (!Y || !V || !rs || !cs || (reg_kind == ORACLE_REG_GROUP_LASSO && !gscratch)) {
    free(Y); free(V); free(rs); free(cs); free(gscratch);
    return -1;
  }
  if (check_every < 1) check_every = 1;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) {
      const size_t e = (size_t)i * n + j;
      X[e] = X0 ? X0[e] : 0.0;
      Y[e] = X[e] + phi0[i] + varphi0[j];
    }
  for (int i = 0; i < m; ++i) phi_out[i] = phi0[i];
  for (int j = 0; j < n; ++j) varphi_out[j] = varphi0[j];

  int k = 0, ngap = 0;
  while (k < max_iters) {
    /* x-update */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < n; ++j) {
        const size_t e = (size_t)i * n + j;
        const double v = Y[e] - rho * (double)C[e];
        X[e] = v > 0.0 ? v : 0.0;
      }
    oracle_prox_entrywise(X, m, n, rho, W, forbidden);
    oracle_prox_h(X, m, n, rho, reg_kind, lambda, mu, row_class, num_classes, gscratch);
    /* z-update */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < n; ++j) {
        const size_t e = (size_t)i * n + j;
        V[e] = 2.0 * X[e] - Y[e];
      }
    oracle_project_marginals(V, m, n, p, q, V, phi_out, varphi_out); /* V now holds Z */
    /* y-update */
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < n; ++j) {
        const size_t e = (size_t)i * n + j;
        Y[e] = Y[e] + V[e] - X[e];
      }
    ++k;
    /* primal residuals of the iterate just produced */
    oracle_row_col_sums(X, m, n, rs, cs);
    double nr = 0.0, ns = 0.0;
    for (int i = 0; i < m; ++i) { const double d = rs[i] - p[i]; nr += d * d; }
    for (int j = 0; j < n; ++j) { const double d = cs[j] - q[j]; ns += d * d; }
    nr = sqrt(nr);
    ns = sqrt(ns);
    if (res_trace) { res_trace[2 * (size_t)(k - 1)] = nr; res_trace[2 * (size_t)(k - 1) + 1] = ns; }
    if (k % check_every == 0) {
      int gap_ok = gap_tol <= 0.0;
      if (gap_every >= 1 && (k / check_every) % gap_every == 0) {
        double t[6];
        oracle_objective_gap(C, X, p, q, phi_out, varphi_out, m, n, rho, reg_kind, lambda, mu, row_class,
                             num_classes, W, forbidden, t);
        const double objective = t[0] + t[1];
        if (gap_trace && ngap < gap_trace_cap) {
          gap_trace[4 * (size_t)ngap] = (double)k;
          gap_trace[4 * (size_t)ngap + 1] = objective;
          gap_trace[4 * (size_t)ngap + 2] = t[4];
          gap_trace[4 * (size_t)ngap + 3] = t[5];
        }
        ++ngap;
        if (gap_tol > 0.0) gap_ok = fabs(t[4]) <= gap_tol * fabs(objective) && t[5] <= gap_tol;
      }
      if (tol > 0.0 && nr <= tol && ns <= tol && gap_ok) break;
    }
  }
  if (gap_trace_len) *gap_trace_len = ngap < gap_trace_cap ? ngap : gap_trace_cap;
  if (Y_out) memcpy(Y_out, Y, sizeof(double) * mn);
  free(Y); free(V); free(rs); free(cs); free(gscratch);
  return k;
}

/*
 * Cost of the variant that takes two point clouds instead of a matrix: C_ij = scale*||xs_i - xt_j||_2^2
 * (squared Euclidean cost between the samples, normalised by `scale`, as in the paper's experiments),
 * from the fp32 points, difference form, fp64 arithmetic, rounded once to fp32.
 */
void oracle_sqdist_cost(const float* xs, const float* xt, int m, int n, int d, double scale, float* C_out) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < m; ++i)
    for (int j = 0; j < n; ++j) {
      double acc = 0.0;
      for (int k = 0; k < d; ++k) {
        const double diff = (double)xs[(size_t)i * d + k] - (double)xt[(size_t)j * d + k];
        acc += diff * diff;
      }
      C_out[(size_t)i * n + j] = (float)(scale * acc);
    }
}

/*
 * Objective and duality gap of a triple (X, phi, varphi) (Appendix C, stopping criteria).
 * With u = phi/rho, v = varphi/rho and W = [u 1^T + 1 v^T - C]_+ :
 *     gap = <C,X> + h(X) - (p^T u + q^T v) + h*(W)
 * where h* is the Fenchel conjugate of h.  Where h* is an indicator its value is dropped from
 * the gap and the constraint violation is returned as the dual residual instead:
 *   none:                 h* = indicator{W = 0}          -> dual_res = ||W||_F
 *   quadratic, lambda>0:  h*(W) = ||W||_F^2 / (2 lambda) -> dual_res = 0
 *   group lasso, lambda>0: h*(W) = sum_g max(||W_g||-mu,0)^2/(2 lambda), dual_res = 0
 *   group lasso, lambda=0: h* = indicator{||W_g|| <= mu} -> dual_res = ||(max(||W_g||-mu,0))_g||_2
 * The entrywise terms (Wl1 = weights of the l1 term, forbidden = the set S of constrained OT)
 * enter through their conjugates, which are indicators composed with h*'s argument: with them
 *   W = [u 1^T + 1 v^T - C - Wl1]_+ outside S and W = 0 on S
 * (the l1 term shifts the cost; entries of S are free in the dual), h(X) gains <Wl1, X>, and
 * entries of S are left out of <C,X> (X vanishes there, whatever C holds).
 * out[0] = <C,X>, out[1] = h(X), out[2] = p^T u + q^T v, out[3] = h*(W) term, out[4] = gap,
 * out[5] = dual_res.
 */
void oracle_objective_gap(const float* C, const double* X, const double* p, const double* q,
                          const double* phi, const double* varphi, int m, int n, double rho,
                          int reg_kind, double lambda, double mu, const int* row_class,
                          int num_classes, const float* Wl1, const unsigned char* forbidden,
                          double* out) {
  double cx = 0.0, xx = 0.0, ww = 0.0, l1 = 0.0;
  double* gx = NULL;
  double* gw = NULL;
  if (reg_kind == ORACLE_REG_GROUP_LASSO) {
    gx = (double*)calloc((size_t)num_classes * n, sizeof(double));
    gw = (double*)calloc((size_t)num_classes * n, sizeof(double));
  }
  for (int i = 0; i < m; ++i) {
    const int c = gx ? row_class[i] : 0;
    for (int j = 0; j < n; ++j) {
      const size_t e = (size_t)i * n + j;
      if (forbidden && forbidden[e]) continue; /* x = 0 and w = 0 there */
      const double x = X[e], cc = (double)C[e];
      const double wl = Wl1 ? (double)Wl1[e] : 0.0;
      double w = (phi[i] + varphi[j]) / rho - cc - wl;
      if (w < 0.0) w = 0.0;
      cx += cc * x;
      l1 += wl * x;
      xx += x * x;
      ww += w * w;
      if (gx) { gx[(size_t)c * n + j] += x * x; gw[(size_t)c * n + j] += w * w; }
    }
  }
  double dual_lin = 0.0;
  for (int i = 0; i < m; ++i) dual_lin += p[i] * phi[i] / rho;
  for (int j = 0; j < n; ++j) dual_lin += q[j] * varphi[j] / rho;
  double hX = 0.0, hstar = 0.0, dres = 0.0;
  if (reg_kind == ORACLE_REG_NONE || (reg_kind == ORACLE_REG_QUADRATIC && lambda <= 0.0)) {
    dres = sqrt(ww);
  } else if (reg_kind == ORACLE_REG_QUADRATIC) {
    hX = 0.5 * lambda * xx;
    hstar = ww / (2.0 * lambda);
  } else {
    double viol2 = 0.0, hs = 0.0, gl = 0.0;
    for (size_t g = 0; g < (size_t)num_classes * n; ++g) {
      gl += sqrt(gx[g]);
      double ex = sqrt(gw[g]) - mu;
      if (ex < 0.0) ex = 0.0;
      viol2 += ex * ex;
      hs += ex * ex;
    }
    hX = mu * gl + 0.5 * lambda * xx;
    if (lambda > 0.0) hstar = hs / (2.0 * lambda);
    else dres = sqrt(viol2);
  }
  hX += l1;
  out[0] = cx; out[1] = hX; out[2] = dual_lin; out[3] = hstar;
  out[4] = cx + hX - dual_lin + hstar;
  out[5] = dres;
  free(gx);
  free(gw);
}
