/*
 * CPU oracle for the GaLore optimizer step (arXiv 2403.03507).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the step computes.  It is called by the tests, by the smoke check and
 * by the benchmark's cpu_baseline leg, never by the product path, and it
 * shares no code with the HIP library.
 *
 * Every routine is the textbook definition written as loops:
 *   - projection  R = P^T G  (m <= n)  or  R = G Q  (m > n)      [Algorithm 2, projection line; Sec. 4.2 one-sided rule]
 *   - Adam on R with bias correction and N = Mhat / (sqrt(Vhat) + eps)   [Algorithm 2, update block; Eq. for N_t in Sec. 4.2]
 *   - projection back and weight update  W <- W - lr*alpha*P N            [Algorithm 2, last three lines]
 *   - top-r singular vectors of G by one-sided Jacobi (no LAPACK)         [Sec. 3.3, SVD equation for P_t, Q_t; Algorithm 2, refresh branch]
 *   - the two-sided form of Definition 3.6,  G~ = P rho(P^T G Q) Q^T  with rho = Adam,
 *     P = [u_1..u_r], Q = [v_1..v_r]                                      [Sec. 3.3, Definition 3.6 and the SVD equation]
 *   - Adafactor with first-order statistics as the entry-wise optimizer rho on R                [Sec. 4.3 and Sec. 5 name it; PARITY UNPINNED by the paper,
 *     which prints no equations for it: the routine states the published Adafactor update, see oracle_adafactor]
 *
 * Matrices are dense row-major double arrays.  OpenMP is used on outermost
 * loops only; there is no blocking, no intrinsics and no library call.
 *
 * Parity pins (tests/test_oracle_*.py): hand-computed Adam steps, closed forms,
 * the r = m, P = I reduction to plain Adam, brute-force SVDs built from known
 * factors, Eckart-Young residuals, and comparison of the Jacobi SVD against a
 * LAPACK SVD.  Decoupled weight decay is not defined by the paper: its only
 * pin is a hand calculation ("parity unpinned" beyond weight_decay = 0).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Threads the parallel loops below use from now on (timing on one core vs. all cores; no effect on results). */
void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* ---------- storage rounding (round-to-nearest-even from fp64) ------------ */

/* Round x to a binary format with `p` significand bits (hidden bit included)
 * and minimum normal exponent 2^-126 (true for both fp32, p = 24, and bf16,
 * p = 8).  Ties go to even.  Values past the largest finite number become
 * infinity.  Relies on the default rounding mode of nearbyint (to nearest
 * even). */
static double round_to_format(double x, int p) {
  if (x == 0.0 || isnan(x) || isinf(x)) return x;
  int e;
  double f = frexp(x, &e); /* x = f * 2^e, 0.5 <= |f| < 1 */
  int bits = p;
  if (e < -125) bits = p - (-125 - e); /* subnormal range: fewer bits */
  double scaled = ldexp(f, bits);
  double rounded = nearbyint(scaled);
  double y = ldexp(rounded, e - bits);
  /* largest finite: (2 - 2^(1-p)) * 2^127 */
  double maxv = ldexp(2.0 - ldexp(1.0, 1 - p), 127);
  if (fabs(y) > maxv) y = (y > 0) ? INFINITY : -INFINITY;
  return y;
}

void oracle_round_bf16(double* x, int64_t count) {
  for (int64_t i = 0; i < count; ++i) x[i] = round_to_format(x[i], 8);
}

void oracle_round_f32(double* x, int64_t count) {
  for (int64_t i = 0; i < count; ++i) x[i] = round_to_format(x[i], 24);
}

/* ---------- projection ----------------------------------------------------- */

/* R (r x n) = P^T G, with P (m x r) and G (m x n).  Algorithm 2: R_t = P_t^T G_t. */
void oracle_project_left(const double* P, const double* G, double* R,
                         int64_t m, int64_t n, int64_t r) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < r; ++i) {
    double* Ri = R + i * n;
    for (int64_t j = 0; j < n; ++j) Ri[j] = 0.0;
    for (int64_t k = 0; k < m; ++k) {
      const double pki = P[k * r + i];
      const double* Gk = G + k * n;
      for (int64_t j = 0; j < n; ++j) Ri[j] += pki * Gk[j];
    }
  }
}

/* R (m x r) = G Q, with G (m x n) and Q (n x r).  Sec. 4.2: project to G Q when m > n. */
void oracle_project_right(const double* G, const double* Q, double* R,
                          int64_t m, int64_t n, int64_t r) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < m; ++i) {
    double* Ri = R + i * r;
    for (int64_t j = 0; j < r; ++j) Ri[j] = 0.0;
    for (int64_t k = 0; k < n; ++k) {
      const double gik = G[i * n + k];
      const double* Qk = Q + k * r;
      for (int64_t j = 0; j < r; ++j) Ri[j] += gik * Qk[j];
    }
  }
}

/* ---------- Adam on the projected gradient --------------------------------- */

/* One Adam update on `count` entries (Algorithm 2, update block), k = 1-based
 * step number used by the bias correction:
 *   M <- b1 M + (1-b1) R ;  V <- b2 V + (1-b2) R^2
 *   Mhat = M / (1 - b1^k) ; Vhat = V / (1 - b2^k)     (temporaries; M, V stay uncorrected)
 *   N = Mhat / (sqrt(Vhat) + eps)
 */
void oracle_adam(const double* R, double* M, double* V, double* N, int64_t count,
                 double beta1, double beta2, double eps, int64_t k) {
  const double c1 = 1.0 - pow(beta1, (double)k);
  const double c2 = 1.0 - pow(beta2, (double)k);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    const double g = R[i];
    const double mi = beta1 * M[i] + (1.0 - beta1) * g;
    const double vi = beta2 * V[i] + (1.0 - beta2) * g * g;
    M[i] = mi;
    V[i] = vi;
    const double mhat = mi / c1;
    const double vhat = vi / c2;
    N[i] = mhat / (sqrt(vhat) + eps);
  }
}

/* ---------- Adafactor on the projected gradient ---------------------------- */

/* The paper applies GaLore to Adafactor with first-order statistics (Sec. 4.3, Sec. 5) and prints no
 * equations for it: PARITY UNPINNED by the paper.  What is stated here is the published Adafactor update
 * for a matrix (Shazeer and Stern 2018: factored second moment, update clipping, decay rate
 * 1 - k^decay_pow, optional momentum) on the rows x cols projected gradient R, with the learning rate
 * left to the caller as in Algorithm 2 (no relative step size, no parameter scaling), k the 1-based step:
 *   b2    = 1 - k^decay_pow                                    (decay_pow = -0.8 in the publication)
 *   rowv_i <- b2 rowv_i + (1 - b2) sum_j (R_ij^2 + eps1)       (rows entries)
 *   colv_j <- b2 colv_j + (1 - b2) sum_i (R_ij^2 + eps1)       (cols entries)
 *   Vhat_ij = rowv_i colv_j / sum_i rowv_i
 *   U = R / sqrt(Vhat) ;  Uhat = U / max(1, RMS(U) / clip_d)   (RMS over all rows x cols entries)
 *   M <- b1 M + (1 - b1) Uhat ;  N = M                         (first-order statistics; b1 = 0: N = Uhat)
 * State: M (rows x cols), rowv, colv.  Pins: tests/test_oracle_adafactor.py (torch.optim.Adafactor for
 * b1 = 0, closed forms at rank-one |R|, scale invariance, the constant-gradient momentum sum, a hand-worked
 * 2 x 2 step). */
void oracle_adafactor(const double* R, double* M, double* rowv, double* colv, double* N,
                      int64_t rows, int64_t cols, double beta1, double decay_pow, double eps1,
                      double clip_d, int64_t k) {
  const double b2 = 1.0 - pow((double)k, decay_pow);
  for (int64_t i = 0; i < rows; ++i) {
    double s = 0.0;
    for (int64_t j = 0; j < cols; ++j) s += R[i * cols + j] * R[i * cols + j] + eps1;
    rowv[i] = b2 * rowv[i] + (1.0 - b2) * s;
  }
  for (int64_t j = 0; j < cols; ++j) {
    double s = 0.0;
    for (int64_t i = 0; i < rows; ++i) s += R[i * cols + j] * R[i * cols + j] + eps1;
    colv[j] = b2 * colv[j] + (1.0 - b2) * s;
  }
  double total = 0.0;
  for (int64_t i = 0; i < rows; ++i) total += rowv[i];
  double sumsq = 0.0;
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t j = 0; j < cols; ++j) {
      const double u = R[i * cols + j] / sqrt(rowv[i] * colv[j] / total);
      N[i * cols + j] = u;     /* U for now */
      sumsq += u * u;
    }
  const double rms = sqrt(sumsq / ((double)rows * (double)cols));
  const double denom = rms / clip_d > 1.0 ? rms / clip_d : 1.0;
  for (int64_t e = 0; e < rows * cols; ++e) {
    const double uhat = N[e] / denom;
    M[e] = beta1 * M[e] + (1.0 - beta1) * uhat;
    N[e] = M[e];
  }
}

/* ---------- projection back + weight update -------------------------------- */

/* W (m x n) <- (1 - lr*wd) W - lr*alpha * P N, P (m x r), N (r x n).
 * Algorithm 2: G~ = alpha P N, W <- W + eta G~ with G = -grad; here the caller
 * passes the positive gradient so the update is subtracted.  The weight-decay
 * term is the decoupled (AdamW) form applied to the pre-update weight; the
 * paper prints no formula for it. */
void oracle_apply_left(double* W, const double* P, const double* N,
                       int64_t m, int64_t n, int64_t r,
                       double lr, double alpha, double weight_decay) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < m; ++i) {
    double* upd = (double*)malloc((size_t)n * sizeof(double));
    for (int64_t j = 0; j < n; ++j) upd[j] = 0.0;
    for (int64_t k = 0; k < r; ++k) {
      const double pik = P[i * r + k];
      const double* Nk = N + k * n;
      for (int64_t j = 0; j < n; ++j) upd[j] += pik * Nk[j];
    }
    double* Wi = W + i * n;
    for (int64_t j = 0; j < n; ++j)
      Wi[j] = Wi[j] - lr * weight_decay * Wi[j] - lr * alpha * upd[j];
    free(upd);
  }
}

/* W (m x n) <- (1 - lr*wd) W - lr*alpha * N Q^T, N (m x r), Q (n x r). */
void oracle_apply_right(double* W, const double* N, const double* Q,
                        int64_t m, int64_t n, int64_t r,
                        double lr, double alpha, double weight_decay) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < m; ++i) {
    double* Wi = W + i * n;
    const double* Ni = N + i * r;
    for (int64_t j = 0; j < n; ++j) {
      const double* Qj = Q + j * r;
      double s = 0.0;
      for (int64_t k = 0; k < r; ++k) s += Ni[k] * Qj[k];
      Wi[j] = Wi[j] - lr * weight_decay * Wi[j] - lr * alpha * s;
    }
  }
}

/* ---------- singular vectors by one-sided Jacobi --------------------------- */

/* Leading r left singular vectors of A (p x q, any p, q) and all p singular
 * values (the last p - min(p,q) are zero up to rounding).
 *
 * Hestenes' one-sided Jacobi on the rows of A: plane rotations of row pairs
 * are applied until all rows are mutually orthogonal, B = J^T A.  Then
 * A = J diag(|b_i|) [b_i/|b_i|]^T is a singular value decomposition with
 * U = J, so u_i is the i-th row of the accumulated J^T.  Rows are then ordered
 * by decreasing norm ("largest" singular vectors come first), and each column
 * of the result is given a canonical sign: its entry of largest magnitude
 * (lowest index on ties) is positive.
 *
 * Pairs are visited in round-robin tournament order so the disjoint pairs of
 * one round can be rotated in parallel; a sweep is p-1 (or p) rounds covering
 * every pair once.  Iteration stops after a sweep in which every pair already
 * satisfied |b_i.b_j| <= tol |b_i| |b_j|.  A row whose norm has fallen to
 * rounding level of the whole matrix (<= eps max(p,q) |A|_F) belongs to a zero
 * singular value: its direction is rounding noise that every rotation with a
 * large row renews, so the relative test can never settle for it and it is
 * left alone, as an exactly zero row is.  Its singular vector is arbitrary
 * within the null space; the accumulated J stays orthogonal either way.
 *
 * U_r: p x r row-major.  sigma: p values, descending.  Returns the number of
 * sweeps used, or -1 if max_sweeps was reached without convergence. */
int oracle_top_left_singular_vectors(const double* A, int64_t p, int64_t q, int64_t r,
                                     double* U_r, double* sigma,
                                     double tol, int max_sweeps) {
  double* B = (double*)malloc((size_t)p * q * sizeof(double));
  double* T = (double*)calloc((size_t)p * p, sizeof(double)); /* J^T */
  memcpy(B, A, (size_t)p * q * sizeof(double));
  for (int64_t i = 0; i < p; ++i) T[i * p + i] = 1.0;

  double fro2 = 0.0;
  for (int64_t i = 0; i < p * q; ++i) fro2 += A[i] * A[i];
  const double zero_norm = DBL_EPSILON * (double)(p > q ? p : q) * sqrt(fro2);
  const double zero2 = zero_norm * zero_norm; /* squared norm at or below which a row counts as zero */

  const int64_t np = (p % 2 == 0) ? p : p + 1; /* players; index p is a bye when p is odd */
  int64_t* seat = (int64_t*)malloc((size_t)np * sizeof(int64_t));
  int sweeps = 0, converged = 0;
  while (sweeps < max_sweeps && !converged) {
    ++sweeps;
    int64_t rotations = 0;
    for (int64_t i = 0; i < np; ++i) seat[i] = i;
    for (int64_t round = 0; round < np - 1; ++round) {
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : rotations)
      for (int64_t s = 0; s < np / 2; ++s) {
        int64_t i = seat[s], j = seat[np - 1 - s];
        if (i >= p || j >= p) continue;
        if (i > j) { int64_t t = i; i = j; j = t; }
        double* bi = B + i * q;
        double* bj = B + j * q;
        double a = 0.0, b = 0.0, c = 0.0;
        for (int64_t k = 0; k < q; ++k) { a += bi[k] * bi[k]; b += bj[k] * bj[k]; c += bi[k] * bj[k]; }
        if (a <= zero2 || b <= zero2) continue;
        if (fabs(c) <= tol * sqrt(a) * sqrt(b)) continue;
        ++rotations;
        const double zeta = (b - a) / (2.0 * c);
        const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        const double cs = 1.0 / sqrt(1.0 + t * t);
        const double sn = cs * t;
        for (int64_t k = 0; k < q; ++k) {
          const double x = bi[k], y = bj[k];
          bi[k] = cs * x - sn * y;
          bj[k] = sn * x + cs * y;
        }
        double* ti = T + i * p;
        double* tj = T + j * p;
        for (int64_t k = 0; k < p; ++k) {
          const double x = ti[k], y = tj[k];
          ti[k] = cs * x - sn * y;
          tj[k] = sn * x + cs * y;
        }
      }
      /* rotate seats 1..np-1, seat 0 fixed */
      int64_t last = seat[np - 1];
      for (int64_t i = np - 1; i > 1; --i) seat[i] = seat[i - 1];
      seat[1] = last;
    }
    if (rotations == 0) converged = 1;
  }

  /* singular values = row norms; order descending (stable on ties) */
  double* nrm = (double*)malloc((size_t)p * sizeof(double));
  int64_t* idx = (int64_t*)malloc((size_t)p * sizeof(int64_t));
  for (int64_t i = 0; i < p; ++i) {
    double a = 0.0;
    for (int64_t k = 0; k < q; ++k) a += B[i * q + k] * B[i * q + k];
    nrm[i] = sqrt(a);
    idx[i] = i;
  }
  for (int64_t i = 1; i < p; ++i) { /* insertion sort, descending, stable */
    int64_t key = idx[i];
    int64_t j = i - 1;
    while (j >= 0 && nrm[idx[j]] < nrm[key]) { idx[j + 1] = idx[j]; --j; }
    idx[j + 1] = key;
  }
  for (int64_t i = 0; i < p; ++i) sigma[i] = nrm[idx[i]];
  for (int64_t c = 0; c < r; ++c) {
    const double* u = T + idx[c] * p; /* row of J^T = column of J */
    int64_t arg = 0;
    double best = 0.0;
    for (int64_t k = 0; k < p; ++k)
      if (fabs(u[k]) > best) { best = fabs(u[k]); arg = k; }
    const double sgn = (u[arg] < 0.0) ? -1.0 : 1.0;
    for (int64_t k = 0; k < p; ++k) U_r[k * r + c] = sgn * u[k];
  }
  free(B); free(T); free(seat); free(nrm); free(idx);
  return converged ? sweeps : -1;
}

/* Projector for a gradient G (m x n):  P = U[:, :r] (m x r) when m <= n, else
 * Q = V[:, :r] (n x r), the leading right singular vectors, obtained as the
 * leading left singular vectors of G^T.  `proj` is (min(m,n)) x r; sigma has
 * min(m,n) entries.  Returns sweeps used or -1. */
int oracle_projector(const double* G, int64_t m, int64_t n, int64_t r,
                     double* proj, double* sigma, double tol, int max_sweeps) {
  if (m <= n) return oracle_top_left_singular_vectors(G, m, n, r, proj, sigma, tol, max_sweeps);
  double* Gt = (double*)malloc((size_t)m * n * sizeof(double));
  for (int64_t i = 0; i < m; ++i)
    for (int64_t j = 0; j < n; ++j) Gt[j * m + i] = G[i * n + j];
  int rc = oracle_top_left_singular_vectors(Gt, n, m, r, proj, sigma, tol, max_sweeps);
  free(Gt);
  return rc;
}

/* ---------- two-sided projection (Definition 3.6) --------------------------- */

/* R (r x r) = P^T G Q, with P (m x r), G (m x n), Q (n x r): the projected gradient R_t of
 * Definition 3.6 / Theorem 3.8.  Written as the two plain products above, (P^T G) Q. */
void oracle_project_two_sided(const double* P, const double* G, const double* Q, double* R,
                              int64_t m, int64_t n, int64_t r) {
  double* T = (double*)malloc((size_t)r * n * sizeof(double));
  oracle_project_left(P, G, T, m, n, r);       /* T = P^T G   (r x n) */
  oracle_project_right(T, Q, R, r, n, r);      /* R = T Q     (r x r) */
  free(T);
}

/* W (m x n) <- (1 - lr*wd) W - lr*alpha * P N Q^T, with N (r x r): G~_t = P_t rho_t(R_t) Q_t^T of
 * Definition 3.6, scaled by alpha and subtracted as in Algorithm 2 (positive-gradient convention). */
void oracle_apply_two_sided(double* W, const double* P, const double* N, const double* Q,
                            int64_t m, int64_t n, int64_t r,
                            double lr, double alpha, double weight_decay) {
  double* S = (double*)malloc((size_t)r * n * sizeof(double));   /* S = N Q^T (r x n) */
  for (int64_t i = 0; i < r; ++i)
    for (int64_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (int64_t k = 0; k < r; ++k) acc += N[i * r + k] * Q[j * r + k];
      S[i * n + j] = acc;
    }
  oracle_apply_left(W, P, S, m, n, r, lr, alpha, weight_decay);
  free(S);
}

/* Both projectors of the SVD equation of Sec. 3.3: P = [u_1..u_r] (m x r), Q = [v_1..v_r] (n x r)
 * of G = U S V^T.  The vectors of the SHORT side come from the Jacobi routine above with their
 * canonical signs (they are the one-sided projector of Algorithm 2); each vector of the long side
 * is the one the decomposition pairs with it, v_i = G^T u_i / s_i (or u_i = G v_i / s_i), so that
 * sum_i s_i u_i v_i^T is the leading part of G.  Needs s_r > 0, i.e. above the rounding level
 * eps max(m,n) |G|_F that the Jacobi routine treats as zero (returns -2 otherwise: the partner
 * vector is then not determined by G).  sigma: min(m, n) values.  Returns the sweeps used or -1. */
int oracle_projector_pair(const double* G, int64_t m, int64_t n, int64_t r,
                          double* P, double* Q, double* sigma, double tol, int max_sweeps) {
  const int left = m <= n;
  double* S = left ? P : Q;                       /* short side: k x r */
  double* L = left ? Q : P;                       /* long side:  l x r */
  const int64_t l = left ? n : m;
  const int rc = oracle_projector(G, m, n, r, S, sigma, tol, max_sweeps);
  if (rc < 0) return rc;
  double fro2 = 0.0;
  for (int64_t i = 0; i < m * n; ++i) fro2 += G[i] * G[i];
  const double zero_norm = DBL_EPSILON * (double)(m > n ? m : n) * sqrt(fro2);
  for (int64_t c = 0; c < r; ++c) {
    double nrm2 = 0.0;
    for (int64_t j = 0; j < l; ++j) {
      double acc = 0.0;
      if (left) { for (int64_t i = 0; i < m; ++i) acc += G[i * n + j] * P[i * r + c]; }   /* (G^T u_c)[j] */
      else      { for (int64_t i = 0; i < n; ++i) acc += G[j * n + i] * Q[i * r + c]; }   /* (G v_c)[j]   */
      L[j * r + c] = acc;
      nrm2 += acc * acc;
    }
    const double nrm = sqrt(nrm2);   /* = s_c */
    if (!(nrm > zero_norm)) return -2;
    for (int64_t j = 0; j < l; ++j) L[j * r + c] /= nrm;
  }
  return rc;
}
