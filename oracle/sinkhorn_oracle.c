/*
 * sinkhorn_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, fp64 CPU statement of what the Sinkhorn hot path computes,
 * written from the paper's definitions so that it can be checked against the
 * paper by eye.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it.  It shares no code with the GPU library.
 *
 * What it follows:
 *   - Gibbs kernel K = exp(-C/eps) and the scaling iteration
 *       u <- a ./ (K v),  v <- b ./ (K^T u)            (Sec. 1, below Eq. 1)
 *   - one iteration = u-update then v-update, u = v = 1 at start
 *                                                      (Algorithm 1)
 *   - row-partitioned form, n = c*m, contiguous index sets I_j
 *                                                      (Sec. 3.1, Algorithm 1)
 *   - blocked iterates equal centralised iterates      (Proposition 1)
 *   - multitarget form: n x N matrices of scalings sharing K (Sec. 5.3.2)
 *   - marginal error of P = diag(u) K diag(v)          (Sec. 5.4, App. DP protocol)
 *   - the objective of Eq. 1 and the expected loss sum P_ij l(x'_j) of the finance example
 *   - damped updates, arithmetic and geometric         (Sec. 3.3 and its Remark)
 *   - bounded-delay emulation of the asynchronous schedule (Algorithm 3, assumption A3)
 *   - synchronous iteration with w local steps between collectives (Sec. 3.1 Remark,
 *     App. "Additional details on local steps")
 *   - log-domain form: the paper only names it (Sec. 1, Sec. 2.1); the
 *     formulas here are the exact logarithm of the iteration above with
 *     f = eps*log u, g = eps*log v.
 *
 * Every sum is a single left-to-right fp64 loop.  K may be handed over as
 * fp32 or fp64 storage; each entry is promoted to fp64 before use.  OpenMP is
 * used only across independent outputs (one thread owns one output element's
 * whole sum), so results do not depend on the thread count.
 *
 * Parity pins (see tests/test_oracle_*.py): exact marginals after each
 * half-step, constant-cost closed form, 2x2 and 3x3 brute-force optimum of
 * Eq. 1, dual ascent and duality gap, blocked == centralised, numpy matmul /
 * scipy logsumexp on single steps, dense == log-domain, batched column ==
 * single run, symmetric special case, resume, Hilbert-metric contraction.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void orc_set_threads(int t) {
#ifdef _OPENMP
  if (t > 0) omp_set_num_threads(t);
#else
  (void)t;
#endif
}

/* K entry (i,j) of a row-major matrix with leading dimension ld, as fp64. */
static inline double k_at(const void* K, int k_is_f32, int64_t ld, int64_t i, int64_t j) {
  return k_is_f32 ? (double)((const float*)K)[i * ld + j] : ((const double*)K)[i * ld + j];
}

/* ------------------------------------------------------------------ setup */

/* C_ij = sum_k (x_ik - y_jk)^2, x: nx x d, y: ny x d, C: nx x ny (Sec. 5.6). */
void orc_cost_sqeuclid(const double* x, const double* y, int64_t nx, int64_t ny, int d, double* C) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < nx; ++i)
    for (int64_t j = 0; j < ny; ++j) {
      double s = 0.0;
      for (int k = 0; k < d; ++k) {
        double t = x[i * d + k] - y[j * d + k];
        s += t * t;
      }
      C[i * ny + j] = s;
    }
}

double orc_max(const double* C, int64_t count) {
  double m = C[0];
  for (int64_t t = 1; t < count; ++t)
    if (C[t] > m) m = C[t];
  return m;
}

/* C <- C / s  (the "normalised by max(C)" step of the workloads). */
void orc_divide_inplace(double* C, int64_t count, double s) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < count; ++t) C[t] = C[t] / s;
}

/* K = exp(-C/eps), elementwise (Sec. 1). */
void orc_gibbs(const double* C, int64_t count, double eps, double* K) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < count; ++t) K[t] = exp(-C[t] / eps);
}

/* Same, fused for large n so that no n x n fp64 array is needed:
 * K_ij = (float) exp(-(||x_i-y_j||^2 / cmax) / eps); pass cmax = 1 for no
 * normalisation.  Written to fp32 storage (the value the fp32 GPU path is fed). */
void orc_gibbs_from_points_f32(const double* x, const double* y, int64_t nx, int64_t ny, int d,
                               double cmax, double eps, float* K) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < nx; ++i)
    for (int64_t j = 0; j < ny; ++j) {
      double s = 0.0;
      for (int k = 0; k < d; ++k) {
        double t = x[i * d + k] - y[j * d + k];
        s += t * t;
      }
      K[i * ny + j] = (float)exp(-(s / cmax) / eps);
    }
}

/* max_ij ||x_i-y_j||^2 without storing C. */
double orc_max_sqeuclid(const double* x, const double* y, int64_t nx, int64_t ny, int d) {
  double m = 0.0;
#pragma omp parallel for schedule(static) reduction(max : m)
  for (int64_t i = 0; i < nx; ++i)
    for (int64_t j = 0; j < ny; ++j) {
      double s = 0.0;
      for (int k = 0; k < d; ++k) {
        double t = x[i * d + k] - y[j * d + k];
        s += t * t;
      }
      if (s > m) m = s;
    }
  return m;
}

/* ------------------------------------------------- the two kernel products */

/* q_i = sum_j K_ij v_j for rows i in [r0, r1); q has n entries, only
 * q[r0..r1) are written.  This is x -> K_{I,:} x of Sec. 3.1. */
void orc_row_products(const void* K, int k_is_f32, int64_t n, int64_t ld, int64_t r0, int64_t r1,
                      const double* v, double* q) {
#pragma omp parallel for schedule(static)
  for (int64_t i = r0; i < r1; ++i) {
    double s = 0.0;
    for (int64_t j = 0; j < n; ++j) s += k_at(K, k_is_f32, ld, i, j) * v[j];
    q[i] = s;
  }
}

/* r_j = sum_{i in [r0,r1)} K_ij u_i for columns j in [c0, c1); only
 * r[c0..c1) are written.  With [r0,r1) = all rows this is x -> (K_{:,I})^T x
 * of Sec. 3.1; with a row range it is one row slab's contribution K_{I,:}^T u_I.
 * Threads split the columns; each r_j is summed over i in increasing order. */
void orc_col_products(const void* K, int k_is_f32, int64_t n, int64_t ld, int64_t r0, int64_t r1,
                      int64_t c0, int64_t c1, const double* u, double* r) {
  (void)n;
  const int64_t chunk = 256;
#pragma omp parallel for schedule(static)
  for (int64_t cb = c0; cb < c1; cb += chunk) {
    int64_t ce = cb + chunk < c1 ? cb + chunk : c1;
    for (int64_t j = cb; j < ce; ++j) r[j] = 0.0;
    for (int64_t i = r0; i < r1; ++i)
      for (int64_t j = cb; j < ce; ++j) r[j] += k_at(K, k_is_f32, ld, i, j) * u[i];
  }
}

/* ------------------------------------------------------ dense, centralised */

/* `iters` iterations of Algorithm 1's loop body on the whole problem; u, v are
 * in/out (the caller puts 1 there for a cold start). */
int orc_sinkhorn_dense(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                       const double* b, double* u, double* v, int iters) {
  double* q = (double*)malloc(sizeof(double) * (size_t)n);
  if (!q) return -1;
  for (int t = 0; t < iters; ++t) {
    orc_row_products(K, k_is_f32, n, ld, 0, n, v, q);
    for (int64_t i = 0; i < n; ++i) u[i] = a[i] / q[i];
    orc_col_products(K, k_is_f32, n, ld, 0, n, 0, n, u, q);
    for (int64_t j = 0; j < n; ++j) v[j] = b[j] / q[j];
  }
  free(q);
  return 0;
}

/* Row and column marginals of P = diag(u) K diag(v). */
void orc_row_marginal(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* u,
                      const double* v, double* out) {
  orc_row_products(K, k_is_f32, n, ld, 0, n, v, out);
  for (int64_t i = 0; i < n; ++i) out[i] = u[i] * out[i];
}

void orc_col_marginal(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* u,
                      const double* v, double* out) {
  orc_col_products(K, k_is_f32, n, ld, 0, n, 0, n, u, out);
  for (int64_t j = 0; j < n; ++j) out[j] = v[j] * out[j];
}

/* ||P 1 - a||_1 and ||P 1 - a||_2 with the current scalings. */
void orc_marginal_error(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                        const double* u, const double* v, double* err_l1, double* err_l2) {
  double* p = (double*)malloc(sizeof(double) * (size_t)n);
  orc_row_marginal(K, k_is_f32, n, ld, u, v, p);
  double s1 = 0.0, s2 = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double e = p[i] - a[i];
    s1 += fabs(e);
    s2 += e * e;
  }
  *err_l1 = s1;
  *err_l2 = sqrt(s2);
  free(p);
}

/* Objective of Eq. 1 and related sums at P = diag(u) K diag(v), by explicit loops over P:
 *   out[0] = <P, C>                      out[1] = sum P_ij (log P_ij - 1)   (0 log 0 = 0)
 *   out[2] = out[0] + eps * out[1]       out[3] = sum P_ij
 *   out[4] = sum_ij P_ij l_j (0 if l is NULL) -- the expected loss of the finance example. */
void orc_plan_objective(const void* K, int k_is_f32, const double* C, int64_t n, int64_t ld,
                        double eps, const double* u, const double* v, const double* l, double* out) {
  double pc = 0.0, ent = 0.0, mass = 0.0, loss = 0.0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) {
      const double p = u[i] * k_at(K, k_is_f32, ld, i, j) * v[j];
      pc += p * C[i * n + j];
      if (p > 0.0) ent += p * (log(p) - 1.0);
      mass += p;
      if (l) loss += p * l[j];
    }
  out[0] = pc; out[1] = ent; out[2] = pc + eps * ent; out[3] = mass; out[4] = loss;
}

/* Kernel of the robust-risk example (Sec. "Illustrative application"): the combined cost is
 * C_lambda,ij = lambda c_ij - l_j, so K_ij = exp(-(lambda c_ij - l_j)/eps).  l may be NULL (0).
 * as_f32: round every entry to fp32 (the value an fp32 consumer holds). */
void orc_gibbs_lambda(const double* c, int64_t n, double lambda, const double* l, double eps,
                      int as_f32, double* K) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) {
      const double k = exp(-(lambda * c[i * n + j] - (l ? l[j] : 0.0)) / eps);
      K[i * n + j] = as_f32 ? (double)(float)k : k;
    }
}

/* Radius search (App. "Enforcing the Wasserstein radius", steps 1-3) by bisection on
 * [lo, hi]: lambda = (lo + hi)/2; K from orc_gibbs_lambda; Algorithm 1 from u = v = 1 for
 * `iters` iterations; g = <P, c> - delta; stop if |g| <= gtol, else lo = lambda when g > 0
 * (the plan moves too far: raise the price of transport) and hi = lambda otherwise; at most
 * max_steps solves.  K (n*n), u, v are left as of the last solve.
 *   out[0] = lambda   out[1] = <P, c>   out[2] = sum_ij P_ij l_j   out[3] = solves done */
void orc_radius_search(const double* c, const double* l, const double* a, const double* b,
                       int64_t n, double eps, double delta, double lo, double hi, int max_steps,
                       double gtol, int iters, int as_f32, double* K, double* u, double* v,
                       double* out) {
  double lambda = 0.5 * (lo + hi), cost = NAN, loss = NAN;
  int steps = 0;
  while (steps < max_steps) {
    lambda = 0.5 * (lo + hi);
    orc_gibbs_lambda(c, n, lambda, l, eps, as_f32, K);
    for (int64_t i = 0; i < n; ++i) u[i] = v[i] = 1.0;
    orc_sinkhorn_dense(K, 0, n, n, a, b, u, v, iters);
    cost = 0.0;
    loss = 0.0;
    for (int64_t i = 0; i < n; ++i)
      for (int64_t j = 0; j < n; ++j) {
        const double p = u[i] * K[i * n + j] * v[j];
        cost += p * c[i * n + j];
        if (l) loss += p * l[j];
      }
    ++steps;
    const double g = cost - delta;
    if (fabs(g) <= gtol) break;
    if (g > 0.0) lo = lambda; else hi = lambda;
  }
  out[0] = lambda; out[1] = cost; out[2] = loss; out[3] = (double)steps;
}

/* Tolerance mode: iterate; after every `check_every`-th iteration (and after
 * the last one) evaluate err = ||P1 - a|| with the scalings just produced;
 * stop at the first such check with err < tol.  l2 == 0: the 1-norm; l2 != 0: the 2-norm,
 * the metric of the paper's convergence plots (Sec. 5.4, err_a) and of its privacy appendix
 * ("Marginal error metric").  Returns iterations done. */
int orc_sinkhorn_dense_tol(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                           const double* b, double* u, double* v, int max_iters, double tol,
                           int check_every, double* err_out, int l2) {
  int done = 0;
  double e1 = INFINITY, e2 = INFINITY;
  while (done < max_iters) {
    orc_sinkhorn_dense(K, k_is_f32, n, ld, a, b, u, v, 1);
    ++done;
    if (done % check_every == 0 || done == max_iters) {
      orc_marginal_error(K, k_is_f32, n, ld, a, u, v, &e1, &e2);
      if ((l2 ? e2 : e1) < tol) break;
    }
  }
  if (err_out) *err_out = l2 ? e2 : e1;
  return done;
}

/* --------------------------------------------------- dense, row-partitioned */

/* c workers, worker j owns I_j = [j*m, (j+1)*m), m = n/c (Sec. 3.1).
 * flow 0: Algorithm 1 as printed -- worker j forms q_{I_j} = K_{I_j,:} v and
 *         u_{I_j}; after the (here trivial) gather of u it forms
 *         r_{I_j} = (K_{:,I_j})^T u and v_{I_j}.
 * flow 1: a worker that holds only its row slab forms the slab's contribution
 *         s^(j) = K_{I_j,:}^T u_{I_j} (length n); r = s^(0) + s^(1) + ... in
 *         that order (the row-wise reduction of the 2D baseline with one
 *         block column, App. "HPC-oriented 2D baseline").
 * Returns -2 if c does not divide n. */
int orc_sinkhorn_blocked(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                         const double* b, double* u, double* v, int iters, int c, int flow) {
  if (c < 1 || n % c != 0) return -2;
  const int64_t m = n / c;
  double* q = (double*)malloc(sizeof(double) * (size_t)n);
  double* s = (double*)malloc(sizeof(double) * (size_t)n);
  if (!q || !s) return -1;
  for (int t = 0; t < iters; ++t) {
    for (int j = 0; j < c; ++j) { /* every worker, same v */
      orc_row_products(K, k_is_f32, n, ld, j * m, (j + 1) * m, v, q);
      for (int64_t i = j * m; i < (j + 1) * m; ++i) u[i] = a[i] / q[i];
    }
    /* Allgather u: all slices already sit in one array */
    if (flow == 0) {
      for (int j = 0; j < c; ++j) {
        orc_col_products(K, k_is_f32, n, ld, 0, n, j * m, (j + 1) * m, u, q);
        for (int64_t i = j * m; i < (j + 1) * m; ++i) v[i] = b[i] / q[i];
      }
    } else {
      for (int64_t i = 0; i < n; ++i) q[i] = 0.0;
      for (int j = 0; j < c; ++j) {
        orc_col_products(K, k_is_f32, n, ld, j * m, (j + 1) * m, 0, n, u, s);
        for (int64_t i = 0; i < n; ++i) q[i] += s[i];
      }
      for (int64_t i = 0; i < n; ++i) v[i] = b[i] / q[i];
    }
    /* Allgather v: likewise */
  }
  free(q);
  free(s);
  return 0;
}

/* 2D block distribution over a p_r x p_c grid (App. "HPC baseline: 2D block distribution"):
 * rank (i, j) holds K_ij (rows R_i = [i n/p_r, (i+1) n/p_r), columns J_j likewise with p_c)
 * and forms the block products K_ij v_j and K_ij^T u_i; the row-wise reduction adds the
 * p_c block products of a block row in the order j = 0, 1, ..., the column-wise one the p_r
 * block products of a block column in the order i = 0, 1, ....
 * Returns -2 if p_r or p_c does not divide n. */
int orc_sinkhorn_grid(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                      const double* b, double* u, double* v, int iters, int p_r, int p_c) {
  if (p_r < 1 || p_c < 1 || n % p_r != 0 || n % p_c != 0) return -2;
  const int64_t nr = n / p_r, nc = n / p_c;
  double* q = (double*)malloc(sizeof(double) * (size_t)n);
  if (!q) return -1;
  for (int t = 0; t < iters; ++t) {
    for (int64_t i = 0; i < n; ++i) { /* q_i = sum_j (K_ij v_j), then u = a ./ q */
      double sum = 0.0;
      for (int j = 0; j < p_c; ++j) {
        double block = 0.0;
        for (int64_t col = j * nc; col < (j + 1) * nc; ++col) block += k_at(K, k_is_f32, ld, i, col) * v[col];
        sum += block;
      }
      q[i] = sum;
    }
    for (int64_t i = 0; i < n; ++i) u[i] = a[i] / q[i];
    for (int64_t col = 0; col < n; ++col) { /* r_j = sum_i (K_ij^T u_i), then v = b ./ r */
      double sum = 0.0;
      for (int i = 0; i < p_r; ++i) {
        double block = 0.0;
        for (int64_t row = i * nr; row < (i + 1) * nr; ++row) block += k_at(K, k_is_f32, ld, row, col) * u[row];
        sum += block;
      }
      q[col] = sum;
    }
    for (int64_t col = 0; col < n; ++col) v[col] = b[col] / q[col];
  }
  free(q);
  return 0;
}

/* ------------------------------------------------------------ damped forms */

/* Relaxed updates of Sec. 3.3 in the centralised view.
 * geometric == 0:  u <- (1-eta) u + eta a./(K v),   likewise v with the new u.
 * geometric != 0:  u <- u^(1-eta) .* (a./(K v))^eta (the Remark), likewise v. */
int orc_sinkhorn_dense_damped(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                              const double* b, double* u, double* v, int iters, double eta,
                              int geometric) {
  double* q = (double*)malloc(sizeof(double) * (size_t)n);
  if (!q) return -1;
  for (int t = 0; t < iters; ++t) {
    orc_row_products(K, k_is_f32, n, ld, 0, n, v, q);
    for (int64_t i = 0; i < n; ++i) {
      double target = a[i] / q[i];
      u[i] = geometric ? pow(u[i], 1.0 - eta) * pow(target, eta) : (1.0 - eta) * u[i] + eta * target;
    }
    orc_col_products(K, k_is_f32, n, ld, 0, n, 0, n, u, q);
    for (int64_t j = 0; j < n; ++j) {
      double target = b[j] / q[j];
      v[j] = geometric ? pow(v[j], 1.0 - eta) * pow(target, eta) : (1.0 - eta) * v[j] + eta * target;
    }
  }
  free(q);
  return 0;
}

/* Bounded-delay emulation of the asynchronous All-to-All schedule (Algorithm 3; assumption
 * A3 of the convergence section) with a deterministic delay: client j (rows/columns
 * I_j = [j*m, (j+1)*m)) keeps cached global vectors whose own slice is always current and
 * whose remote slices are what the peers held at the end of iteration s(t), the last exchange
 * (every `w` iterations) that is at least `tau` iterations old:
 *     s(t) = floor((t-1-tau)/w)*w   (the initial vectors if that is <= 0).
 * Iteration t = 1, 2, ...: with v_hat = [remote: v^{s(t)}, own: v^{t-1}_{I_j}],
 *     u^t_{I_j} = (1-eta) u^{t-1}_{I_j} + eta a_j ./ (K_{I_j,:} v_hat);
 * then with u_hat = [remote: u^{s(t)}, own: u^t_{I_j}],
 *     v^t_{I_j} = (1-eta) v^{t-1}_{I_j} + eta b_j ./ ((K_{:,I_j})^T u_hat).
 * u, v in/out hold the global vectors (every client's own slice). */
int orc_sinkhorn_async_emulated(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                                const double* b, double* u, double* v, int iters, int c, double eta,
                                int tau, int w) {
  if (c < 1 || n % c != 0 || tau < 0 || w < 1) return -2;
  const int64_t m = n / c;
  /* hist_u[s], hist_v[s]: the global vectors at the end of iteration s (s = 0: the init) */
  double* hist_u = (double*)malloc(sizeof(double) * (size_t)n * (size_t)(iters + 1));
  double* hist_v = (double*)malloc(sizeof(double) * (size_t)n * (size_t)(iters + 1));
  double* view = (double*)malloc(sizeof(double) * (size_t)n);
  double* prod = (double*)malloc(sizeof(double) * (size_t)n);
  if (!hist_u || !hist_v || !view || !prod) return -1;
  memcpy(hist_u, u, sizeof(double) * (size_t)n);
  memcpy(hist_v, v, sizeof(double) * (size_t)n);
  for (int t = 1; t <= iters; ++t) {
    int s = t - 1 - tau;
    s = s <= 0 ? 0 : (s / w) * w;
    const double* su = hist_u + (size_t)s * n;       /* what the peers last sent */
    const double* sv = hist_v + (size_t)s * n;
    const double* pu = hist_u + (size_t)(t - 1) * n; /* own slices as of the previous iteration */
    const double* pv = hist_v + (size_t)(t - 1) * n;
    double* nu = hist_u + (size_t)t * n;
    double* nv = hist_v + (size_t)t * n;
    for (int j = 0; j < c; ++j) {
      const int64_t lo = j * m, hi = (j + 1) * m;
      for (int64_t i = 0; i < n; ++i) view[i] = (i >= lo && i < hi) ? pv[i] : sv[i];
      orc_row_products(K, k_is_f32, n, ld, lo, hi, view, prod);
      for (int64_t i = lo; i < hi; ++i) nu[i] = (1.0 - eta) * pu[i] + eta * (a[i] / prod[i]);
      for (int64_t i = 0; i < n; ++i) view[i] = (i >= lo && i < hi) ? nu[i] : su[i];
      orc_col_products(K, k_is_f32, n, ld, 0, n, lo, hi, view, prod);
      for (int64_t i = lo; i < hi; ++i) nv[i] = (1.0 - eta) * pv[i] + eta * (b[i] / prod[i]);
    }
  }
  memcpy(u, hist_u + (size_t)iters * n, sizeof(double) * (size_t)n);
  memcpy(v, hist_v + (size_t)iters * n, sizeof(double) * (size_t)n);
  free(hist_u); free(hist_v); free(view); free(prod);
  return 0;
}

/* Synchronous federated iteration with w local steps between collectives (Sec. 3.1, Remark
 * "Local steps before communication"; App. "Additional details on local steps"; the
 * "optional" collectives (i) and (iii) of Sec. 3.2.1).  Every client j keeps its OWN
 * full-length views uview[j], vview[j] of the global scalings (all equal to the init at the
 * start).  Iteration k = 1, 2, ..., iters, for every client j:
 *     q_{I_j} = K_{I_j,:} vview[j],        u_{I_j} = a_j ./ q_{I_j}   (stored in uview[j] only);
 *     if k is a multiple of w: Allgather u -- every view receives every client's own slice;
 *     r_{I_j} = (K_{:,I_j})^T uview[j],    v_{I_j} = b_j ./ r_{I_j}   (stored in vview[j] only);
 *     if k is a multiple of w: Allgather v.
 * So between collectives a client sees its own slices as current and the peers' slices as of
 * the last collective; w = 1 is Algorithm 1 line by line.  u, v in/out are the global vectors
 * (client j's own slice at positions I_j).  Returns -2 unless c | n and w >= 1. */
int orc_sinkhorn_local_steps(const void* K, int k_is_f32, int64_t n, int64_t ld, const double* a,
                             const double* b, double* u, double* v, int iters, int c, int w) {
  if (c < 1 || n % c != 0 || w < 1) return -2;
  const int64_t m = n / c;
  double* uview = (double*)malloc(sizeof(double) * (size_t)n * (size_t)c);
  double* vview = (double*)malloc(sizeof(double) * (size_t)n * (size_t)c);
  double* prod = (double*)malloc(sizeof(double) * (size_t)n);
  if (!uview || !vview || !prod) return -1;
  for (int j = 0; j < c; ++j) { /* "identical at all clients" */
    memcpy(uview + (size_t)j * n, u, sizeof(double) * (size_t)n);
    memcpy(vview + (size_t)j * n, v, sizeof(double) * (size_t)n);
  }
  for (int k = 1; k <= iters; ++k) {
    for (int j = 0; j < c; ++j) {
      double* uj = uview + (size_t)j * n;
      orc_row_products(K, k_is_f32, n, ld, j * m, (j + 1) * m, vview + (size_t)j * n, prod);
      for (int64_t i = j * m; i < (j + 1) * m; ++i) uj[i] = a[i] / prod[i];
    }
    if (k % w == 0) /* Allgather u: slice I_p of every view <- client p's own slice */
      for (int p = 0; p < c; ++p)
        for (int j = 0; j < c; ++j)
          if (j != p)
            memcpy(uview + (size_t)j * n + p * m, uview + (size_t)p * n + p * m, sizeof(double) * (size_t)m);
    for (int j = 0; j < c; ++j) {
      double* vj = vview + (size_t)j * n;
      orc_col_products(K, k_is_f32, n, ld, 0, n, j * m, (j + 1) * m, uview + (size_t)j * n, prod);
      for (int64_t i = j * m; i < (j + 1) * m; ++i) vj[i] = b[i] / prod[i];
    }
    if (k % w == 0) /* Allgather v */
      for (int p = 0; p < c; ++p)
        for (int j = 0; j < c; ++j)
          if (j != p)
            memcpy(vview + (size_t)j * n + p * m, vview + (size_t)p * n + p * m, sizeof(double) * (size_t)m);
  }
  for (int j = 0; j < c; ++j) {
    memcpy(u + j * m, uview + (size_t)j * n + j * m, sizeof(double) * (size_t)m);
    memcpy(v + j * m, vview + (size_t)j * n + j * m, sizeof(double) * (size_t)m);
  }
  free(uview); free(vview); free(prod);
  return 0;
}

/* ---------------------------------------------------------------- batched */

/* Multitarget form (Sec. 5.3.2): A, B, U, V are n x m row-major (ld = m), one
 * histogram pair per column, K shared.  Q = K V, U = A ./ Q, R = K^T U,
 * V = B ./ R. */
int orc_sinkhorn_batched(const void* K, int k_is_f32, int64_t n, int64_t ld, int m, const double* A,
                         const double* B, double* U, double* V, int iters) {
  double* Q = (double*)malloc(sizeof(double) * (size_t)n * (size_t)m);
  if (!Q) return -1;
  for (int t = 0; t < iters; ++t) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
      for (int k = 0; k < m; ++k) Q[i * m + k] = 0.0;
      for (int64_t j = 0; j < n; ++j) {
        double kij = k_at(K, k_is_f32, ld, i, j);
        for (int k = 0; k < m; ++k) Q[i * m + k] += kij * V[j * m + k];
      }
      for (int k = 0; k < m; ++k) U[i * m + k] = A[i * m + k] / Q[i * m + k];
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
      for (int k = 0; k < m; ++k) Q[j * m + k] = 0.0;
      for (int64_t i = 0; i < n; ++i) {
        double kij = k_at(K, k_is_f32, ld, i, j);
        for (int k = 0; k < m; ++k) Q[j * m + k] += kij * U[i * m + k];
      }
      for (int k = 0; k < m; ++k) V[j * m + k] = B[j * m + k] / Q[j * m + k];
    }
  }
  free(Q);
  return 0;
}

/* Multitarget form with the relaxed updates of Sec. 3.3 applied to every target
 * (geometric == 0: X <- (1-eta) X + eta X_new; else X <- X^(1-eta) .* X_new^eta, X = U or V). */
int orc_sinkhorn_batched_damped(const void* K, int k_is_f32, int64_t n, int64_t ld, int m,
                                const double* A, const double* B, double* U, double* V, int iters,
                                double eta, int geometric) {
  double* Q = (double*)malloc(sizeof(double) * (size_t)n * (size_t)m);
  if (!Q) return -1;
  for (int t = 0; t < iters; ++t) {
    for (int side = 0; side < 2; ++side) {
      const double* X = side == 0 ? V : U;     /* the factor the product runs over */
      double* Y = side == 0 ? U : V;           /* the factor being updated */
      const double* M = side == 0 ? A : B;
#pragma omp parallel for schedule(static)
      for (int64_t i = 0; i < n; ++i) {
        for (int k = 0; k < m; ++k) Q[i * m + k] = 0.0;
        for (int64_t j = 0; j < n; ++j) {
          double kij = side == 0 ? k_at(K, k_is_f32, ld, i, j) : k_at(K, k_is_f32, ld, j, i);
          for (int k = 0; k < m; ++k) Q[i * m + k] += kij * X[j * m + k];
        }
      }
      for (int64_t e = 0; e < n * (int64_t)m; ++e) {
        double target = M[e] / Q[e];
        Y[e] = geometric ? pow(Y[e], 1.0 - eta) * pow(target, eta) : (1.0 - eta) * Y[e] + eta * target;
      }
    }
  }
  free(Q);
  return 0;
}

/* Multitarget form with the stop rule of orc_sinkhorn_dense_tol applied to all targets at once
 * (the multitarget experiment of Sec. 5.3.2 iterates until every target meets the threshold):
 * err = max over columns k of ||P_k 1 - a_k|| (1-norm, or 2-norm with l2 != 0), P_k = diag(u_k) K
 * diag(v_k), evaluated after a V-update every check_every iterations and after the last one.
 * Returns iterations done. */
int orc_sinkhorn_batched_tol(const void* K, int k_is_f32, int64_t n, int64_t ld, int m,
                             const double* A, const double* B, double* U, double* V, int max_iters,
                             double tol, int check_every, double* err_out, int l2) {
  double* Q = (double*)malloc(sizeof(double) * (size_t)n * (size_t)m);
  double* colerr = (double*)malloc(sizeof(double) * (size_t)m);
  if (!Q || !colerr) return -1;
  int done = 0;
  double err = INFINITY;
  while (done < max_iters) {
    orc_sinkhorn_batched(K, k_is_f32, n, ld, m, A, B, U, V, 1);
    ++done;
    if (done % check_every == 0 || done == max_iters) {
#pragma omp parallel for schedule(static)
      for (int64_t i = 0; i < n; ++i) {
        for (int k = 0; k < m; ++k) Q[i * m + k] = 0.0;
        for (int64_t j = 0; j < n; ++j) {
          double kij = k_at(K, k_is_f32, ld, i, j);
          for (int k = 0; k < m; ++k) Q[i * m + k] += kij * V[j * m + k];
        }
      }
      err = 0.0;
      for (int k = 0; k < m; ++k) {
        colerr[k] = 0.0;
        for (int64_t i = 0; i < n; ++i) {
          const double dev = U[i * m + k] * Q[i * m + k] - A[i * m + k];
          colerr[k] += l2 ? dev * dev : fabs(dev);
        }
        if (l2) colerr[k] = sqrt(colerr[k]);
        if (colerr[k] > err) err = colerr[k];
      }
      if (err < tol) break;
    }
  }
  if (err_out) *err_out = err;
  free(Q);
  free(colerr);
  return done;
}

/* ------------------------------------------------- privacy layer (DP appendix) */

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11): a counter-based generator; 128-bit counter, 64-bit key, ten rounds of two
 * 32x32->64 multiplications with the key bumped by Weyl constants between rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Standard normal number `e` of release `release` under `seed`: Philox call e/4 with counter
 * (call, release) and key seed gives x0..x3; Box-Muller on (x0, x1) gives normals 0 and 1 of
 * the call, on (x2, x3) normals 2 and 3: with u1 = (xa + 1/2) 2^-32, u2 = (xb + 1/2) 2^-32,
 * z_even = sqrt(-2 ln u1) cos(2 pi u2), z_odd = sqrt(-2 ln u1) sin(2 pi u2). */
double orc_dp_normal(uint64_t seed, uint64_t release, uint64_t e) {
  const uint64_t call = e / 4;
  const uint32_t ctr[4] = {(uint32_t)call, (uint32_t)(call >> 32), (uint32_t)release, (uint32_t)(release >> 32)};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t x[4];
  orc_philox4x32_10(ctr, key, x);
  const int pair = (int)((e % 4) / 2);
  const double u1 = ((double)x[2 * pair] + 0.5) * 0x1p-32, u2 = ((double)x[2 * pair + 1] + 0.5) * 0x1p-32;
  const double r = sqrt(-2.0 * log(u1)), phi = 6.283185307179586476925286766559 * u2;
  return (e % 2 == 0) ? r * cos(phi) : r * sin(phi);
}

void orc_dp_normals(uint64_t seed, uint64_t release, uint64_t first, int64_t count, double* out) {
  for (int64_t t = 0; t < count; ++t) out[t] = orc_dp_normal(seed, release, first + (uint64_t)t);
}

/* One release of an n x m scaling matrix X (row-major, in place): L = log X; every row of L is
 * scaled by min(1, S / ||L_i||_2) (the row-wise clip across the m targets; S <= 0 or infinite:
 * no clipping, the Gaussian-only ablation); L_ik += sigma * normal number i*m + k of this
 * release; X = exp(L). */
void orc_dp_release(double* X, int64_t n, int m, double S, double sigma, uint64_t seed, uint64_t release) {
  for (int64_t i = 0; i < n; ++i) {
    double sq = 0.0;
    for (int k = 0; k < m; ++k) {
      const double l = log(X[i * m + k]);
      sq += l * l;
    }
    const double norm = sqrt(sq);
    const double scale = (S > 0.0 && isfinite(S) && norm > S) ? S / norm : 1.0;
    for (int k = 0; k < m; ++k) {
      const double l = log(X[i * m + k]) * scale + sigma * orc_dp_normal(seed, release, (uint64_t)(i * m + k));
      X[i * m + k] = exp(l);
    }
  }
}

/* Multitarget iteration with a release after every update (centralised view: the noised
 * scalings replace the held ones): U = A ./ (K V), release 2t of U, V = B ./ (K^T U), release
 * 2t + 1 of V, for t = release0/2 ...; release0 (even) numbers the first release of this call. */
int orc_sinkhorn_batched_dp(const void* K, int k_is_f32, int64_t n, int64_t ld, int m, const double* A,
                            const double* B, double* U, double* V, int iters, double S_u, double S_v,
                            double sigma_u, double sigma_v, uint64_t seed, uint64_t release0) {
  double* Q = (double*)malloc(sizeof(double) * (size_t)n * (size_t)m);
  if (!Q) return -1;
  for (int t = 0; t < iters; ++t) {
    for (int64_t i = 0; i < n; ++i) {
      for (int k = 0; k < m; ++k) Q[i * m + k] = 0.0;
      for (int64_t j = 0; j < n; ++j)
        for (int k = 0; k < m; ++k) Q[i * m + k] += k_at(K, k_is_f32, ld, i, j) * V[j * m + k];
      for (int k = 0; k < m; ++k) U[i * m + k] = A[i * m + k] / Q[i * m + k];
    }
    orc_dp_release(U, n, m, S_u, sigma_u, seed, release0 + 2 * (uint64_t)t);
    for (int64_t j = 0; j < n; ++j) {
      for (int k = 0; k < m; ++k) Q[j * m + k] = 0.0;
      for (int64_t i = 0; i < n; ++i)
        for (int k = 0; k < m; ++k) Q[j * m + k] += k_at(K, k_is_f32, ld, i, j) * U[i * m + k];
      for (int k = 0; k < m; ++k) V[j * m + k] = B[j * m + k] / Q[j * m + k];
    }
    orc_dp_release(V, n, m, S_v, sigma_v, seed, release0 + 2 * (uint64_t)t + 1);
  }
  free(Q);
  return 0;
}

/* Renyi-DP accountant: a Gaussian release with l2 sensitivity Delta = 2 S and noise sigma is
 * (p, p Delta^2 / (2 sigma^2))-RDP; `releases` of them add up; the (eps, delta) bound is the
 * minimum over the given orders p > 1 of eps_RDP(p) + log(1/delta)/(p - 1).  Returns the
 * bound and stores the minimising order. */
double orc_rdp_epsilon(double S, double sigma, int64_t releases, double delta, const double* orders,
                       int n_orders, double* best_order) {
  double best = INFINITY, arg = NAN;
  for (int t = 0; t < n_orders; ++t) {
    const double p = orders[t];
    if (!(p > 1.0)) continue;
    const double rdp = (double)releases * p * (2.0 * S) * (2.0 * S) / (2.0 * sigma * sigma);
    const double eps = rdp + log(1.0 / delta) / (p - 1.0);
    if (eps < best) { best = eps; arg = p; }
  }
  if (best_order) *best_order = arg;
  return best;
}

/* ------------------------------------------------------------- log domain */

/* LSE(z) = max z + log sum exp(z - max z). */
double orc_lse(const double* z, int64_t n) {
  double m = z[0];
  for (int64_t t = 1; t < n; ++t)
    if (z[t] > m) m = z[t];
  if (isinf(m)) return m;
  double s = 0.0;
  for (int64_t t = 0; t < n; ++t) s += exp(z[t] - m);
  return m + log(s);
}

static double sqdist(const double* p, const double* q, int d) {
  double s = 0.0;
  for (int k = 0; k < d; ++k) {
    double t = p[k] - q[k];
    s += t * t;
  }
  return s;
}

/* One potential update against a point cloud, for a list of rows:
 *   out[t] = eps*log w_i - eps*LSE_j((h_j - ||p_i - q_j||^2)/eps),  i = rows[t]
 * (rows == NULL means rows[t] = t).  With (p,w,h,q) = (x,a,g,y) this is the
 * f-update (the logarithm of u = a./(K v) times eps); with (y,b,f,x) it is the
 * g-update (cost is symmetric in the roles of the two clouds). */
void orc_log_update_points(const double* p, const double* w, const double* q, const double* h,
                           int64_t nq, int d, double eps, const int64_t* rows, int64_t n_rows,
                           double* out) {
#pragma omp parallel
  {
    double* z = (double*)malloc(sizeof(double) * (size_t)nq);
#pragma omp for schedule(static)
    for (int64_t t = 0; t < n_rows; ++t) {
      int64_t i = rows ? rows[t] : t;
      for (int64_t j = 0; j < nq; ++j) z[j] = (h[j] - sqdist(p + i * d, q + j * d, d)) / eps;
      out[t] = eps * log(w[i]) - eps * orc_lse(z, nq);
    }
    free(z);
  }
}

/* Row marginal of P_ij = exp((f_i + g_j - C_ij)/eps) for listed rows:
 * out[t] = exp(f_i/eps + LSE_j((g_j - C_ij)/eps)). */
void orc_log_row_marginal_points(const double* x, const double* f, const double* y, const double* g,
                                 int64_t ny, int d, double eps, const int64_t* rows, int64_t n_rows,
                                 double* out) {
#pragma omp parallel
  {
    double* z = (double*)malloc(sizeof(double) * (size_t)ny);
#pragma omp for schedule(static)
    for (int64_t t = 0; t < n_rows; ++t) {
      int64_t i = rows ? rows[t] : t;
      for (int64_t j = 0; j < ny; ++j) z[j] = (g[j] - sqdist(x + i * d, y + j * d, d)) / eps;
      out[t] = exp(f[i] / eps + orc_lse(z, ny));
    }
    free(z);
  }
}

/* Log-domain Sinkhorn on point clouds, cost evaluated on the fly.  f, g in/out
 * (0 for a cold start, i.e. u = v = 1).  tol <= 0: exactly max_iters
 * iterations.  tol > 0: same polling rule as orc_sinkhorn_dense_tol, with
 * err = ||P1 - a||_1 (||P1 - a||_2 with l2 != 0) evaluated after the g-update.  Returns
 * iterations done. */
int orc_sinkhorn_log_points(const double* x, const double* y, int64_t n, int d, double eps,
                            const double* a, const double* b, double* f, double* g, int max_iters,
                            double tol, int check_every, double* err_out, int l2) {
  double* t1 = (double*)malloc(sizeof(double) * (size_t)n);
  int done = 0;
  double err = INFINITY;
  while (done < max_iters) {
    orc_log_update_points(x, a, y, g, n, d, eps, NULL, n, t1);
    memcpy(f, t1, sizeof(double) * (size_t)n);
    orc_log_update_points(y, b, x, f, n, d, eps, NULL, n, t1);
    memcpy(g, t1, sizeof(double) * (size_t)n);
    ++done;
    if (tol > 0.0 && (done % check_every == 0 || done == max_iters)) {
      orc_log_row_marginal_points(x, f, y, g, n, d, eps, NULL, n, t1);
      err = 0.0;
      for (int64_t i = 0; i < n; ++i) err += l2 ? (t1[i] - a[i]) * (t1[i] - a[i]) : fabs(t1[i] - a[i]);
      if (l2) err = sqrt(err);
      if (err < tol) break;
    }
  }
  if (err_out) *err_out = err;
  free(t1);
  return done;
}

/* The relaxed updates of Sec. 3.3 in the log domain, f = eps log u, g = eps log v.
 * geometric != 0:  u <- u^(1-eta) (u_new)^eta  is  f <- (1-eta) f + eta f_new.
 * geometric == 0:  u <- (1-eta) u + eta u_new  is  f <- eps log((1-eta) e^(f/eps) + eta e^(f_new/eps)),
 *                  evaluated with the larger of the two exponents taken out.
 * Exactly max_iters iterations. */
int orc_sinkhorn_log_points_damped(const double* x, const double* y, int64_t n, int d, double eps,
                                   const double* a, const double* b, double* f, double* g,
                                   int max_iters, double eta, int geometric) {
  double* t1 = (double*)malloc(sizeof(double) * (size_t)n);
  if (!t1) return -1;
  for (int t = 0; t < max_iters; ++t) {
    for (int side = 0; side < 2; ++side) {
      double* pot = side == 0 ? f : g;
      if (side == 0) orc_log_update_points(x, a, y, g, n, d, eps, NULL, n, t1);
      else orc_log_update_points(y, b, x, f, n, d, eps, NULL, n, t1);
      for (int64_t i = 0; i < n; ++i) {
        if (geometric) {
          pot[i] = (1.0 - eta) * pot[i] + eta * t1[i];
        } else {
          double M = pot[i] > t1[i] ? pot[i] : t1[i];
          pot[i] = M + eps * log((1.0 - eta) * exp((pot[i] - M) / eps) + eta * exp((t1[i] - M) / eps));
        }
      }
    }
  }
  free(t1);
  return 0;
}

/* Log-domain Sinkhorn on an explicit n x n cost matrix (small n; used to tie
 * the log form to the dense form on the same C). */
int orc_sinkhorn_log_cost(const double* C, int64_t n, double eps, const double* a, const double* b,
                          double* f, double* g, int iters) {
  double* z = (double*)malloc(sizeof(double) * (size_t)n);
  for (int t = 0; t < iters; ++t) {
    for (int64_t i = 0; i < n; ++i) {
      for (int64_t j = 0; j < n; ++j) z[j] = (g[j] - C[i * n + j]) / eps;
      f[i] = eps * log(a[i]) - eps * orc_lse(z, n);
    }
    for (int64_t j = 0; j < n; ++j) {
      for (int64_t i = 0; i < n; ++i) z[i] = (f[i] - C[i * n + j]) / eps;
      g[j] = eps * log(b[j]) - eps * orc_lse(z, n);
    }
  }
  free(z);
  return 0;
}
