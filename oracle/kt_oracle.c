/*
 * kt_oracle.c -- plain fp64 CPU oracle for the KurTail rotation-learning step.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call into this
 * file; it exists so that the HIP kernels can be checked against an obviously
 * correct, slow implementation that shares no code with them.
 *
 * Every function writes out a definition from the paper (arXiv 2503.01483)
 * with plain loops, in double precision, two-pass where a mean is involved,
 * with no blocking, fusion or raw-moment shortcuts:
 *
 *   kto_rotate          Y = X R            ("Learning the Rotations": the
 *                                           linear layer of the small network)
 *   kto_row_moments     mu, m2, m3, m4, kappa of one row
 *                                          (Background, "Kurtosis", Eq. 3:
 *                                           population moments about the mean,
 *                                           not excess)
 *   kto_loss_grad       loss = mean_i f(kappa_i), dL/dR = X^T (dL/dY)
 *                                          (kurtosis loss of Sec. 2 in its
 *                                           per-token-row reading; gradient by
 *                                           the chain rule through Eq. 3)
 *   kto_pooled_loss_grad  the loss as the paper writes it: kurtosis of the
 *                                          concatenation of all tokens' activations
 *                                          after the linear layer and an RMSNorm,
 *                                          |kappa - kappa_u| (loss equation of the
 *                                          "Kurtosis" paragraph; "Learning the
 *                                          Rotations": linear layer + RMSNorm)
 *   kto_cayley_step     R+ = (I + lr/2 A)^-1 (I - lr/2 A) R,  A = G R^T - R G^T
 *                                          ("Optimization in the Orthogonal
 *                                           Space": Cayley SGD on the Stiefel
 *                                           manifold; exact solve by LU with
 *                                           partial pivoting)
 *   kto_cayley_step_right  the same retraction written on the right of R
 *   kto_cayley_adam_step  one step of the Cayley Adam optimiser that the paper
 *                                          names ("Learning the Rotations", Setup)
 *                                          and defers to the cited work on Stiefel
 *                                          optimisation for; the paper prints no
 *                                          formula, so this follows that published
 *                                          algorithm as this build reads it, with
 *                                          the Cayley transform solved exactly
 *   kto_fakequant_int4  per-token symmetric 4-bit fake quantisation of X R
 *                                          (Background, "Uniform Quantization
 *                                           for k-bit Precision": b = 0,
 *                                           s = max|x| / (2^(k-1) - 1); MSE of
 *                                           Eq. 1; Setup: one scale per row)
 *
 *   kto_quant_metrics   per-token quantisation-quality figures of Y = X R: largest
 *                                          magnitude before / after the rotation (the
 *                                          "success rate" of "Evaluation of ... on Channel
 *                                          Outliers"), symmetric int4 error with the scale
 *                                          clipped at a quantile of |y| (Setup: quantile
 *                                          0.98), asymmetric int4 error (Background:
 *                                          b = min, s = (max - min)/(2^k - 1); Setup: KV)
 *
 *   kto_quant_sensitivity  optimal step of a symmetric k-bit uniform quantiser over a whole tensor and
 *                                          the quantisation sensitivity Gamma of the Definition in the
 *                                          Background ("Quantization Sensitivity"): the rise of the MSE
 *                                          (Eq. 1) when the step moves off the optimum by a fraction of it
 *   kto_hadamard_rows   the online rotations R3-R5 ("Placement of the Rotations": random
 *                                          Hadamard matrices): y = (x * signs) H_d / sqrt(d), H_d the
 *                                          Sylvester matrix for powers of two, else a Paley matrix
 *                                          of small order (x) a Sylvester matrix
 *   kto_fuse_rotation   merging a fusible rotation into a weight matrix ("Placement of
 *                                          the Rotations"): W R or R^T W
 *
 * Degenerate rows (no spread: m2 <= 1e-30 * mean(y^2), or an all-zero row):
 * kappa := 0, gradient row := 0, the row still counts in the 1/n.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * closed forms, brute force and library routines it does not itself use.
 * kto_cayley_adam_step: the arithmetic of the step is pinned that way too; that its
 * constants (start value of v, form of the bias correction, q) are those of the cited
 * algorithm cannot be checked here (the paper prints none of them): parity unpinned
 * in that respect.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int kto_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Y[n][d] = X[n][d] * R[d][d], all row-major doubles. */
void kto_rotate(const double *X, const double *R, int64_t n, int64_t d, double *Y) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    double *y = Y + i * d;
    for (int64_t j = 0; j < d; ++j) y[j] = 0.0;
    for (int64_t k = 0; k < d; ++k) {
      const double x = X[i * d + k];
      const double *r = R + k * d;
      for (int64_t j = 0; j < d; ++j) y[j] += x * r[j];
    }
  }
}

/* Moments of one row about its mean (Eq. 3).  out = {mu, m2, m3, m4, kappa}.
 * Returns 1 if the row is degenerate (kappa set to 0). */
int kto_row_moments(const double *y, int64_t d, double out[5]) {
  double s = 0.0, raw2 = 0.0;
  for (int64_t j = 0; j < d; ++j) { s += y[j]; raw2 += y[j] * y[j]; }
  const double mu = s / (double)d;
  double m2 = 0.0, m3 = 0.0, m4 = 0.0;
  for (int64_t j = 0; j < d; ++j) {
    const double c = y[j] - mu;
    const double c2 = c * c;
    m2 += c2; m3 += c2 * c; m4 += c2 * c2;
  }
  m2 /= (double)d; m3 /= (double)d; m4 /= (double)d; raw2 /= (double)d;
  out[0] = mu; out[1] = m2; out[2] = m3; out[3] = m4;
  if (!(m2 > 1e-30 * raw2)) { out[4] = 0.0; return 1; }
  out[4] = m4 / (m2 * m2);
  return 0;
}

static double sgn(double v) { return (v > 0.0) - (v < 0.0); }

/*
 * loss = (1/n) sum_i f(kappa_i), f(k) = k if kappa_target == 0 else |k - kappa_target|.
 * dL/dy_ij = s_i * 4/(n d m2_i^2) * [c_ij^3 - m3_i - kappa_i m2_i c_ij],
 *   s_i = 1 (or sign(kappa_i - kappa_target)); dR = X^T (dL/dY).
 * row_kurt (n), G (n*d) and dR (d*d) may each be NULL.
 */
void kto_loss_grad(const double *X, const double *R, int64_t n, int64_t d,
                   double kappa_target, double *loss, double *row_kurt,
                   double *G, double *dR) {
  double *Y = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
  double *Gl = G;
  if (dR && !Gl) Gl = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
  double *kap = (double *)malloc(sizeof(double) * (size_t)n);
  kto_rotate(X, R, n, d, Y);

#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    double mo[5];
    const double *y = Y + i * d;
    const int degenerate = kto_row_moments(y, d, mo);
    kap[i] = mo[4];
    if (Gl) {
      double *g = Gl + i * d;
      if (degenerate) {
        for (int64_t j = 0; j < d; ++j) g[j] = 0.0;
      } else {
        const double mu = mo[0], m2 = mo[1], m3 = mo[2], kappa = mo[4];
        const double si = (kappa_target == 0.0) ? 1.0 : sgn(kappa - kappa_target);
        const double a = si * 4.0 / ((double)n * (double)d * m2 * m2);
        for (int64_t j = 0; j < d; ++j) {
          const double c = y[j] - mu;
          g[j] = a * (c * c * c - m3 - kappa * m2 * c);
        }
      }
    }
  }

  double acc = 0.0;
  for (int64_t i = 0; i < n; ++i)
    acc += (kappa_target == 0.0) ? kap[i] : fabs(kap[i] - kappa_target);
  if (loss) *loss = acc / (double)n;
  if (row_kurt) memcpy(row_kurt, kap, sizeof(double) * (size_t)n);

  if (dR) {
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < d; ++k) {
      double *o = dR + k * d;
      for (int64_t j = 0; j < d; ++j) o[j] = 0.0;
      for (int64_t i = 0; i < n; ++i) {
        const double x = X[i * d + k];
        const double *g = Gl + i * d;
        for (int64_t j = 0; j < d; ++j) o[j] += x * g[j];
      }
    }
  }
  free(Y);
  free(kap);
  if (Gl && Gl != G) free(Gl);
}

/* C[d][d] = A[d][d] * B[d][d]^T */
/*
 * Pooled (paper-literal) kurtosis loss of one problem.
 *   Y = X R;  rho_i = sqrt(mean_j y_ij^2 + rms_eps);  Z = Y / rho   (RMSNorm, no gain)
 *   kappa = kurtosis of all n*d entries of Z taken as ONE sample (Eq. 3)
 *   loss  = |kappa - kappa_target|   (kappa_target == 0: loss = kappa)
 * Gradient by the chain rule: dL/dz = s 4/(N m2^2) [c^3 - m3 - kappa m2 c], c = z - mu, N = n d;
 * through the RMSNorm  dL/dy_i = (dL/dz_i)/rho_i - y_i (y_i . dL/dz_i) / (d rho_i^3);  dR = X^T dL/dY.
 * A row of zeros with rms_eps == 0 is taken as z = 0 with no gradient.
 * kappa_out, G (n*d, = dL/dY) and dR may each be NULL.
 */
void kto_pooled_loss_grad(const double *X, const double *R, int64_t n, int64_t d,
                          double kappa_target, double rms_eps, double *loss,
                          double *kappa_out, double *G, double *dR) {
  const size_t nd = (size_t)n * (size_t)d;
  double *Y = (double *)malloc(sizeof(double) * nd);
  double *Z = (double *)malloc(sizeof(double) * nd);
  double *rho = (double *)malloc(sizeof(double) * (size_t)n);
  double *Gl = G;
  if (dR && !Gl) Gl = (double *)malloc(sizeof(double) * nd);
  kto_rotate(X, R, n, d, Y);
  for (int64_t i = 0; i < n; ++i) {
    double s2 = 0.0;
    for (int64_t j = 0; j < d; ++j) s2 += Y[i * d + j] * Y[i * d + j];
    rho[i] = sqrt(s2 / (double)d + rms_eps);
    for (int64_t j = 0; j < d; ++j) Z[i * d + j] = rho[i] > 0.0 ? Y[i * d + j] / rho[i] : 0.0;
  }
  const double N = (double)n * (double)d;
  double mu = 0.0;
  for (size_t t = 0; t < nd; ++t) mu += Z[t];
  mu /= N;
  double m2 = 0.0, m3 = 0.0, m4 = 0.0;
  for (size_t t = 0; t < nd; ++t) {
    const double c = Z[t] - mu, c2 = c * c;
    m2 += c2; m3 += c2 * c; m4 += c2 * c2;
  }
  m2 /= N; m3 /= N; m4 /= N;
  const int degenerate = !(m2 > 0.0);
  const double kappa = degenerate ? 0.0 : m4 / (m2 * m2);
  if (kappa_out) *kappa_out = kappa;
  if (loss) *loss = (kappa_target == 0.0) ? kappa : fabs(kappa - kappa_target);
  if (Gl) {
    const double si = (kappa_target == 0.0) ? 1.0 : sgn(kappa - kappa_target);
    const double a = degenerate ? 0.0 : si * 4.0 / (N * m2 * m2);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
      double *g = Gl + i * d;
      const double *y = Y + i * d, *z = Z + i * d;
      if (!(rho[i] > 0.0) || a == 0.0) {
        for (int64_t j = 0; j < d; ++j) g[j] = 0.0;
        continue;
      }
      double dot = 0.0; /* y_i . dL/dz_i */
      for (int64_t j = 0; j < d; ++j) {
        const double c = z[j] - mu;
        g[j] = a * (c * c * c - m3 - kappa * m2 * c); /* dL/dz */
        dot += y[j] * g[j];
      }
      const double r3 = rho[i] * rho[i] * rho[i];
      for (int64_t j = 0; j < d; ++j) g[j] = g[j] / rho[i] - y[j] * dot / ((double)d * r3);
    }
  }
  if (dR) {
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < d; ++k) {
      double *o = dR + k * d;
      for (int64_t j = 0; j < d; ++j) o[j] = 0.0;
      for (int64_t i = 0; i < n; ++i) {
        const double x = X[i * d + k];
        const double *g = Gl + i * d;
        for (int64_t j = 0; j < d; ++j) o[j] += x * g[j];
      }
    }
  }
  free(Y); free(Z); free(rho);
  if (Gl && Gl != G) free(Gl);
}

static void mat_abt(const double *A, const double *B, int64_t d, double *C) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = 0; j < d; ++j) {
      double s = 0.0;
      for (int64_t k = 0; k < d; ++k) s += A[i * d + k] * B[j * d + k];
      C[i * d + j] = s;
    }
}

/* C[d][d] = A[d][d] * B[d][d] */
static void mat_ab(const double *A, const double *B, int64_t d, double *C) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < d; ++i) {
    double *c = C + i * d;
    for (int64_t j = 0; j < d; ++j) c[j] = 0.0;
    for (int64_t k = 0; k < d; ++k) {
      const double a = A[i * d + k];
      const double *b = B + k * d;
      for (int64_t j = 0; j < d; ++j) c[j] += a * b[j];
    }
  }
}

/* C[d][d] = A[d][d]^T * B[d][d] */
static void mat_atb(const double *A, const double *B, int64_t d, double *C) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < d; ++i) {
    double *c = C + i * d;
    for (int64_t j = 0; j < d; ++j) c[j] = 0.0;
    for (int64_t k = 0; k < d; ++k) {
      const double a = A[k * d + i];
      const double *b = B + k * d;
      for (int64_t j = 0; j < d; ++j) c[j] += a * b[j];
    }
  }
}

/*
 * Solve M Z = B in place (Z overwrites B) by Gaussian elimination with partial
 * pivoting.  M (d x d) is destroyed.  B has nrhs columns, row-major.
 * Returns 0, or -1 if a pivot is exactly zero.
 */
static int lu_solve(double *M, double *B, int64_t d, int64_t nrhs) {
  for (int64_t c = 0; c < d; ++c) {
    int64_t p = c;
    double best = fabs(M[c * d + c]);
    for (int64_t r = c + 1; r < d; ++r) {
      const double v = fabs(M[r * d + c]);
      if (v > best) { best = v; p = r; }
    }
    if (best == 0.0) return -1;
    if (p != c) {
      for (int64_t j = 0; j < d; ++j) { double t = M[c * d + j]; M[c * d + j] = M[p * d + j]; M[p * d + j] = t; }
      for (int64_t j = 0; j < nrhs; ++j) { double t = B[c * nrhs + j]; B[c * nrhs + j] = B[p * nrhs + j]; B[p * nrhs + j] = t; }
    }
    const double piv = M[c * d + c];
#pragma omp parallel for schedule(static)
    for (int64_t r = c + 1; r < d; ++r) {
      const double f = M[r * d + c] / piv;
      if (f != 0.0) {
        for (int64_t j = c + 1; j < d; ++j) M[r * d + j] -= f * M[c * d + j];
        for (int64_t j = 0; j < nrhs; ++j) B[r * nrhs + j] -= f * B[c * nrhs + j];
      }
      M[r * d + c] = 0.0;
    }
  }
  for (int64_t c = d - 1; c >= 0; --c) {
    const double piv = M[c * d + c];
    for (int64_t j = 0; j < nrhs; ++j) B[c * nrhs + j] /= piv;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < c; ++r) {
      const double f = M[r * d + c];
      if (f != 0.0)
        for (int64_t j = 0; j < nrhs; ++j) B[r * nrhs + j] -= f * B[c * nrhs + j];
    }
  }
  return 0;
}

/*
 * Cayley SGD step, left form:  A = G R^T - R G^T (skew),
 * (I + lr/2 A) R+ = (I - lr/2 A) R.   A_out (d*d) may be NULL.
 */
int kto_cayley_step(const double *R, const double *G, int64_t d, double lr,
                    double *Rout, double *A_out) {
  const size_t dd = (size_t)d * (size_t)d;
  double *GRt = (double *)malloc(sizeof(double) * dd);
  double *A = (double *)malloc(sizeof(double) * dd);
  double *M = (double *)malloc(sizeof(double) * dd);
  double *N = (double *)malloc(sizeof(double) * dd);
  mat_abt(G, R, d, GRt);
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = 0; j < d; ++j) A[i * d + j] = GRt[i * d + j] - GRt[j * d + i];
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = 0; j < d; ++j) {
      const double e = (i == j) ? 1.0 : 0.0;
      M[i * d + j] = e + 0.5 * lr * A[i * d + j];
      N[i * d + j] = e - 0.5 * lr * A[i * d + j];
    }
  mat_ab(N, R, d, Rout);
  const int rc = lu_solve(M, Rout, d, d);
  if (A_out) memcpy(A_out, A, sizeof(double) * dd);
  free(GRt); free(A); free(M); free(N);
  return rc;
}

/*
 * One step of Cayley Adam on the orthogonal group (square R), step counter k >= 1.
 *   M1   = beta1 M + (1 - beta1) G                       first moment
 *   v1   = beta2 v + (1 - beta2) ||G||_F^2               scalar second moment
 *   r    = (1 - beta1^k) sqrt(v1 / (1 - beta2^k) + eps)  both bias corrections in one factor
 *   What = M1 R^T - 1/2 R (R^T M1 R^T),  W = (What - What^T) / r     skew
 *   M+   = r W R                                         momentum moved into the tangent space at R
 *   a    = min(lr, 2 q / (||W||_F + eps))                keeps the fixed point of the transform contractive
 *   R+   = (I + a/2 W)^-1 (I - a/2 W) R                  Cayley transform, solved exactly here
 * Outputs: Rout, Mout (d*d), v_out, and scal_out[3] = {r, a, ||W||_F} (may be NULL).
 * Returns 0, or -1 if the solve hit a zero pivot.
 */
int kto_cayley_adam_step(const double *R, const double *G, const double *M, double v,
                         int64_t d, int64_t k, double lr, double beta1, double beta2,
                         double eps, double q, double *Rout, double *Mout, double *v_out,
                         double *scal_out) {
  const size_t dd = (size_t)d * (size_t)d;
  double *M1 = (double *)malloc(sizeof(double) * dd);
  double *T1 = (double *)malloc(sizeof(double) * dd);
  double *T2 = (double *)malloc(sizeof(double) * dd);
  double *T3 = (double *)malloc(sizeof(double) * dd);
  double *W = (double *)malloc(sizeof(double) * dd);
  double *P = (double *)malloc(sizeof(double) * dd);
  double *N = (double *)malloc(sizeof(double) * dd);
  double g2 = 0.0;
  for (size_t i = 0; i < dd; ++i) {
    M1[i] = beta1 * M[i] + (1.0 - beta1) * G[i];
    g2 += G[i] * G[i];
  }
  const double v1 = beta2 * v + (1.0 - beta2) * g2;
  const double r = (1.0 - pow(beta1, (double)k)) * sqrt(v1 / (1.0 - pow(beta2, (double)k)) + eps);
  mat_abt(M1, R, d, T1);  /* M1 R^T */
  mat_atb(R, T1, d, T2);  /* R^T M1 R^T */
  mat_ab(R, T2, d, T3);   /* R R^T M1 R^T */
  for (size_t i = 0; i < dd; ++i) T1[i] -= 0.5 * T3[i]; /* What */
  double w2 = 0.0;
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = 0; j < d; ++j) {
      const double w = (T1[i * d + j] - T1[j * d + i]) / r;
      W[i * d + j] = w;
      w2 += w * w;
    }
  const double wn = sqrt(w2);
  mat_ab(W, R, d, Mout);
  for (size_t i = 0; i < dd; ++i) Mout[i] *= r;
  const double a1 = 2.0 * q / (wn + eps);
  const double a = lr < a1 ? lr : a1;
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = 0; j < d; ++j) {
      const double e = (i == j) ? 1.0 : 0.0;
      P[i * d + j] = e + 0.5 * a * W[i * d + j];
      N[i * d + j] = e - 0.5 * a * W[i * d + j];
    }
  mat_ab(N, R, d, Rout);
  const int rc = lu_solve(P, Rout, d, d);
  *v_out = v1;
  if (scal_out) { scal_out[0] = r; scal_out[1] = a; scal_out[2] = wn; }
  free(M1); free(T1); free(T2); free(T3); free(W); free(P); free(N);
  return rc;
}

/*
 * The same retraction written on the right of R (equal to the left form when R
 * is orthogonal):  W = R^T G - G^T R,  R+ = R (I + lr/2 W)^-1 (I - lr/2 W).
 * Solved as (I + lr/2 W)^T Z^T = R^T after forming R (.) via Z = R (I + lr/2 W)^-1.
 */
int kto_cayley_step_right(const double *R, const double *G, int64_t d, double lr,
                          double *Rout) {
  const size_t dd = (size_t)d * (size_t)d;
  double *RtG = (double *)malloc(sizeof(double) * dd);
  double *Mt = (double *)malloc(sizeof(double) * dd);
  double *N = (double *)malloc(sizeof(double) * dd);
  double *Zt = (double *)malloc(sizeof(double) * dd);
  double *Z = (double *)malloc(sizeof(double) * dd);
  mat_atb(R, G, d, RtG);
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = 0; j < d; ++j) {
      const double w = RtG[i * d + j] - RtG[j * d + i];
      const double e = (i == j) ? 1.0 : 0.0;
      Mt[j * d + i] = e + 0.5 * lr * w; /* transposed */
      N[i * d + j] = e - 0.5 * lr * w;
      Zt[j * d + i] = R[i * d + j];     /* R^T */
    }
  /* Z M = R  <=>  M^T Z^T = R^T */
  const int rc = lu_solve(Mt, Zt, d, d);
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = 0; j < d; ++j) Z[i * d + j] = Zt[j * d + i];
  mat_ab(Z, N, d, Rout);
  free(RtG); free(Mt); free(N); free(Zt); free(Z);
  return rc;
}

/*
 * Per-token symmetric int4 fake quantisation of Y = X R.
 * The rotation is fp64; the rounding-critical part is carried out in IEEE
 * single precision, one operation at a time:
 *   yf = (float)y;  amax = max_j |yf|;  s = (clip * amax) / 7.0f   (or scales_in)
 *   r = 1.0f / s;   q = clamp(rint(yf * r), -7, 7)   (round half to even)
 *   yhat = q * s;   err = { sum_j (y - yhat)^2, sum_j y^2 }  in fp64 on y.
 * A row with s == 0 gets codes 0 and yhat 0.
 * scales_in, scales_out, codes, err may each be NULL.
 */
void kto_fakequant_int4(const double *X, const double *R, int64_t n, int64_t d,
                        float clip, const float *scales_in, float *scales_out,
                        int8_t *codes, double *err) {
  double *Y = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
  kto_rotate(X, R, n, d, Y);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const double *y = Y + i * d;
    float s;
    if (scales_in) {
      s = scales_in[i];
    } else {
      float amax = 0.0f;
      for (int64_t j = 0; j < d; ++j) {
        const float a = fabsf((float)y[j]);
        if (a > amax) amax = a;
      }
      volatile float num = clip * amax;
      s = num / 7.0f;
    }
    if (scales_out) scales_out[i] = s;
    double e2 = 0.0, y2 = 0.0;
    if (s > 0.0f) {
      volatile float r = 1.0f / s;
      for (int64_t j = 0; j < d; ++j) {
        const float yf = (float)y[j];
        volatile float t = yf * r;
        float q = rintf(t);
        if (q > 7.0f) q = 7.0f;
        if (q < -7.0f) q = -7.0f;
        if (codes) codes[i * d + j] = (int8_t)q;
        const double yhat = (double)q * (double)s;
        const double diff = y[j] - yhat;
        e2 += diff * diff;
        y2 += y[j] * y[j];
      }
    } else {
      for (int64_t j = 0; j < d; ++j) {
        if (codes) codes[i * d + j] = 0;
        e2 += y[j] * y[j];
        y2 += y[j] * y[j];
      }
    }
    if (err) { err[2 * i] = e2; err[2 * i + 1] = y2; }
  }
  free(Y);
}

static int cmp_float(const void *a, const void *b) {
  const float x = *(const float *)a, y = *(const float *)b;
  return (x > y) - (x < y);
}

/*
 * Per token row of Y = X R, with yf = (float)y and every rounding-critical step in IEEE single:
 *   amax[i]   = { max_j |x_ij| as float, max_j |yf_ij| };   success = amax_rot < amax_base
 *   symmetric int4, scale clipped at the quantile `quant` of |yf| over the row (linear
 *   interpolation between order statistics: pos = quant (d-1), k = floor(pos),
 *   t = a_k + (float)(pos - k) (a_{k+1} - a_k) on the ascending a; quant >= 1: t = amax):
 *     s = t / 7.0f, r = 1.0f / s, q = clamp(rint(yf r), -7, 7), yhat = q s
 *   asymmetric int4:  b = min_j yf, s = (max_j yf - b) / 15.0f, r = 1.0f / s,
 *     q = clamp(rint((yf - b) r), 0, 15), yhat = q s + b
 *   err_sym[i] = err_asym[i] = { sum_j (y - yhat)^2, sum_j y^2 } in fp64.
 * A row with s == 0 reproduces itself for asym (yhat = b) and gives yhat = 0 for sym.
 * Returns the number of successes.  Output pointers may be NULL.
 */
int64_t kto_quant_metrics(const double *X, const double *R, int64_t n, int64_t d,
                          double quant, float *amax, float *thr, double *err_sym, double *err_asym) {
  double *Y = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
  kto_rotate(X, R, n, d, Y);
  int64_t succ = 0;
#pragma omp parallel for schedule(static) reduction(+ : succ)
  for (int64_t i = 0; i < n; ++i) {
    float *a = (float *)malloc(sizeof(float) * (size_t)d);
    float ab = 0.0f, ar = 0.0f, mn = 0.0f, mx = 0.0f;
    double y2 = 0.0;
    for (int64_t j = 0; j < d; ++j) {
      const double yd = Y[i * d + j];
      const float yf = (float)yd;
      const float xa = fabsf((float)X[i * d + j]);
      if (xa > ab) ab = xa;
      a[j] = fabsf(yf);
      if (a[j] > ar) ar = a[j];
      if (j == 0 || yf < mn) mn = yf;
      if (j == 0 || yf > mx) mx = yf;
      y2 += yd * yd;
    }
    if (ar < ab) succ += 1;
    if (amax) { amax[2 * i] = ab; amax[2 * i + 1] = ar; }
    float t = ar;
    if (quant < 1.0) {
      qsort(a, (size_t)d, sizeof(float), cmp_float);
      const double pos = quant * (double)(d - 1);
      const int64_t k = (int64_t)floor(pos);
      const float frac = (float)(pos - (double)k);
      const float hi = a[k + 1 < d ? k + 1 : k];
      volatile float diff = hi - a[k];
      volatile float inc = frac * diff;
      t = a[k] + inc;
    }
    if (thr) thr[i] = t;
    const float ss = t / 7.0f;
    volatile float span = mx - mn;
    const float sa = span / 15.0f;
    double es = 0.0, ea = 0.0;
    for (int64_t j = 0; j < d; ++j) {
      const double yd = Y[i * d + j];
      const float yf = (float)yd;
      double yh = 0.0;
      if (ss > 0.0f) {
        volatile float r = 1.0f / ss;
        volatile float u = yf * r;
        float q = rintf(u);
        if (q > 7.0f) q = 7.0f;
        if (q < -7.0f) q = -7.0f;
        yh = (double)q * (double)ss;
      }
      es += (yd - yh) * (yd - yh);
      double ya = (double)mn;
      if (sa > 0.0f) {
        volatile float r = 1.0f / sa;
        volatile float c = yf - mn;
        volatile float u = c * r;
        float q = rintf(u);
        if (q > 15.0f) q = 15.0f;
        if (q < 0.0f) q = 0.0f;
        ya = (double)q * (double)sa + (double)mn;
      }
      ea += (yd - ya) * (yd - ya);
    }
    if (err_sym) { err_sym[2 * i] = es; err_sym[2 * i + 1] = y2; }
    if (err_asym) { err_asym[2 * i] = ea; err_asym[2 * i + 1] = y2; }
    free(a);
  }
  free(Y);
  return succ;
}

/*
 * Hadamard matrices for the online rotations ("Placement of the Rotations": random Hadamard
 * matrices; the hidden and FFN sizes of the models in the Setup are m 2^k with small m, not
 * always powers of two).  The paper does not say which Hadamard matrix of a given order is meant:
 * any one is an orthogonal rotation after scaling.  This library fixes
 *   H_d = H_m (x) S_{2^k}     (Kronecker product, index a 2^k + b, a < m, b < 2^k)
 * with S the Sylvester matrix and H_m, for d = r 2^t with r odd:
 *   r = 1:  m = 1 when t <= 12, else m = max(4, 2^(t-12)); H_m = S_m (so H_d = S_d always)
 *   r > 1:  m = r 2^j for the smallest j >= 2 (m <= 256) that admits
 *           Paley's first construction  (q = m - 1 prime; then q = 3 mod 4), else
 *           Paley's second construction (q = m/2 - 1 prime with q = 1 mod 4).
 * Paley I:  H = I + S,  S = [[0, 1^T], [-1, Q]],  Q[u][v] = chi(u - v) the quadratic character
 *           of Z_q (Q is skew for q = 3 mod 4).
 * Paley II: C = [[0, 1^T], [1, Q]] (symmetric for q = 1 mod 4),  H = [[C + I, C - I], [C - I, -C - I]].
 * Everything below is the definition written out: O(q) per character value, O(d^2) per row.
 */
static int kto_is_prime(int64_t q) {
  if (q < 2) return 0;
  for (int64_t t = 2; t * t <= q; ++t)
    if (q % t == 0) return 0;
  return 1;
}

/* quadratic character of x modulo the prime q: 0, +1 (a non-zero square) or -1 */
static int kto_chi(int64_t x, int64_t q) {
  x %= q;
  if (x < 0) x += q;
  if (x == 0) return 0;
  for (int64_t t = 1; t < q; ++t)
    if ((t * t) % q == x) return 1;
  return -1;
}

/* d = m * p2 as described above; kind 0 Sylvester, 1 Paley I, 2 Paley II.  Returns 0, or -1 when
 * no construction is found. */
int kto_hadamard_factor(int64_t d, int64_t *m_out, int64_t *p2_out, int *kind_out) {
  if (d < 1) return -1;
  int64_t r = d, t = 0;
  while ((r & 1) == 0) { r >>= 1; ++t; }
  if (r == 1) {
    int64_t m = 1;
    if (t > 12) { m = (int64_t)1 << (t - 12); if (m < 4) m = 4; }
    *m_out = m; *p2_out = d / m; *kind_out = 0;
    return 0;
  }
  for (int64_t j = 2; j <= t; ++j) {
    const int64_t m = r << j;
    if (m > 256) break;
    if (kto_is_prime(m - 1)) { *m_out = m; *p2_out = d / m; *kind_out = 1; return 0; }
    if (kto_is_prime(m / 2 - 1) && (m / 2 - 1) % 4 == 1) { *m_out = m; *p2_out = d / m; *kind_out = 2; return 0; }
  }
  return -1;
}

/* H [m][m] of the given kind (entries +-1) */
void kto_hadamard_matrix(int64_t m, int kind, int8_t *H) {
  if (kind == 0) {
    for (int64_t a = 0; a < m; ++a)
      for (int64_t b = 0; b < m; ++b) H[a * m + b] = (__builtin_popcountll((unsigned long long)(a & b)) & 1) ? -1 : 1;
  } else if (kind == 1) {
    const int64_t q = m - 1;
    for (int64_t i = 0; i < m; ++i)
      for (int64_t j = 0; j < m; ++j) {
        int s;                                   /* entry of S */
        if (i == 0) s = j == 0 ? 0 : 1;
        else if (j == 0) s = -1;
        else s = kto_chi(i - j, q);
        H[i * m + j] = (int8_t)(s + (i == j ? 1 : 0));
      }
  } else {
    const int64_t h = m / 2, q = h - 1;
    for (int64_t i = 0; i < m; ++i)
      for (int64_t j = 0; j < m; ++j) {
        const int64_t u = i % h, v = j % h;
        int c;                                   /* entry of C */
        if (u == v) c = 0;
        else if (u == 0 || v == 0) c = 1;
        else c = kto_chi(u - v, q);
        const int id = u == v ? 1 : 0;
        int e;
        if (i < h && j < h) e = c + id;
        else if (i >= h && j >= h) e = -c - id;
        else e = c - id;
        H[i * m + j] = (int8_t)e;
      }
  }
}

/*
 * Y[i][:] = (X[i][:] * signs) H_d / sqrt(d) with H_d as defined above.  The Sylvester factor is
 * written out entry by entry: S[a][b] = (-1)^popcount(a & b)  (the closed form of the recursion
 * S_1 = [1], S_2m = [[S_m, S_m], [S_m, -S_m]]).  signs (d values +-1) may be NULL.
 * Plain O(d^2) per row: this is the definition, not a fast transform.  Returns 0, or -1 when d
 * has no construction.
 */
int kto_hadamard_rows(const double *X, const double *signs, int64_t n, int64_t d, double *Y) {
  int64_t m, p2;
  int kind;
  if (kto_hadamard_factor(d, &m, &p2, &kind) != 0) return -1;
  int8_t *H = (int8_t *)malloc((size_t)(m * m));
  kto_hadamard_matrix(m, kind, H);
  const double sc = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    for (int64_t ao = 0; ao < m; ++ao)
      for (int64_t bo = 0; bo < p2; ++bo) {
        double acc = 0.0;
        for (int64_t ai = 0; ai < m; ++ai) {
          const double h = (double)H[ai * m + ao];
          for (int64_t bi = 0; bi < p2; ++bi) {
            const int64_t k = ai * p2 + bi;
            const double x = X[i * d + k] * (signs ? signs[k] : 1.0) * h;
            acc += (__builtin_popcountll((unsigned long long)(bi & bo)) & 1) ? -x : x;
          }
        }
        Y[i * d + ao * p2 + bo] = acc * sc;
      }
  }
  free(H);
  return 0;
}

/*
 * Fusing a rotation into a weight matrix: side = 0: Wout[k][d] = W[k][d] R[d][d]   (rotation on the
 * right of the weight);  side = 1: Wout[d][k] = R^T[d][d] W[d][k]   (inverse rotation on its left).
 */
void kto_fuse_rotation(const double *W, const double *R, int64_t k, int64_t d, int side, double *Wout) {
  if (side == 0) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < k; ++i)
      for (int64_t j = 0; j < d; ++j) {
        double acc = 0.0;
        for (int64_t m = 0; m < d; ++m) acc += W[i * d + m] * R[m * d + j];
        Wout[i * d + j] = acc;
      }
  } else {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < d; ++i)
      for (int64_t j = 0; j < k; ++j) {
        double acc = 0.0;
        for (int64_t m = 0; m < d; ++m) acc += R[m * d + i] * W[m * k + j];
        Wout[i * k + j] = acc;
      }
  }
}

/* MSE (Eq. 1) of the symmetric k-bit uniform quantiser with step s over y[0..count):
 * q = clamp(rint(y / s), -L, L), L = 2^(bits-1) - 1; the decision y * (1/s) is taken in fp32 like
 * every quantiser here, the error in fp64. */
static double mse_at_step(const float *y, int64_t count, float s, int L) {
  if (!(s > 0.0f)) {
    double a = 0.0;
    for (int64_t i = 0; i < count; ++i) a += (double)y[i] * (double)y[i];
    return a / (double)count;
  }
  volatile float r = 1.0f / s;
  double acc = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : acc)
  for (int64_t i = 0; i < count; ++i) {
    volatile float u = y[i] * r;
    float q = rintf(u);
    if (q > (float)L) q = (float)L;
    if (q < -(float)L) q = -(float)L;
    const double dd = (double)y[i] - (double)q * (double)s;
    acc += dd * dd;
  }
  return acc / (double)count;
}

/* Eq. 1 at one step, exported for the pins. */
double kto_quant_mse(const float *y, int64_t count, int bits, float s) {
  return mse_at_step(y, count, s, (1 << (bits - 1)) - 1);
}

/*
 * Quantisation sensitivity (Background: Definition "Quantization Sensitivity", Eq. 1), as the
 * definition reads: s_opt = argmin_s MSE(s), Gamma(alpha) = | MSE(s_opt (1 + alpha)) - MSE(s_opt) |.
 * The argmin is taken by a dense scan: KTO_SENS_GRID steps spaced evenly in log s from
 * smax = max|y| / L (the largest step that still uses the outermost level; beyond it nothing is
 * clipped and the error only grows) down to smax / 1024, then a golden-section search between the
 * two grid neighbours of the best grid point; s_opt is the best step evaluated anywhere.
 *   out[0] = s_opt, out[1] = MSE(s_opt),
 *   out[2], out[3] = the smallest and the largest grid step whose MSE is within (1 + flat_tol) of
 *                    MSE(s_opt): how far apart steps that are as good as the optimum lie (for a
 *                    small sample MSE(s) is jagged and such steps need not be neighbours).
 *   gamma[i] = | MSE(s_opt (1 + alphas[i])) - MSE(s_opt) |   (step formed in fp32).
 */
#define KTO_SENS_GRID 4096
void kto_quant_sensitivity(const float *y, int64_t count, int bits, const float *alphas, int n_alpha,
                           double flat_tol, double *out, double *gamma) {
  const int L = (1 << (bits - 1)) - 1;
  float amax = 0.0f;
  for (int64_t i = 0; i < count; ++i) { const float a = fabsf(y[i]); if (a > amax) amax = a; }
  const double smax = (double)amax / (double)L;
  double *mse = (double *)malloc(sizeof(double) * KTO_SENS_GRID);
  float *grid = (float *)malloc(sizeof(float) * KTO_SENS_GRID);
  int arg = 0;
  for (int k = 0; k < KTO_SENS_GRID; ++k) {       /* descending: grid[0] = smax */
    grid[k] = (float)(smax * exp(-log(1024.0) * (double)k / (double)(KTO_SENS_GRID - 1)));
    mse[k] = mse_at_step(y, count, grid[k], L);
    if (mse[k] < mse[arg]) arg = k;
  }
  double best = mse[arg];
  float best_s = grid[arg];
  /* golden-section search on [a, b] = the two neighbours of the best grid point */
  double a = (double)grid[arg + 1 < KTO_SENS_GRID ? arg + 1 : arg], b = (double)grid[arg > 0 ? arg - 1 : arg];
  const double phi = 0.5 * (sqrt(5.0) - 1.0);
  double x1 = b - phi * (b - a), x2 = a + phi * (b - a);
  double f1 = mse_at_step(y, count, (float)x1, L), f2 = mse_at_step(y, count, (float)x2, L);
  for (int it = 0; it < 48 && b > a; ++it) {
    if (f1 < best) { best = f1; best_s = (float)x1; }
    if (f2 < best) { best = f2; best_s = (float)x2; }
    if (f1 <= f2) { b = x2; x2 = x1; f2 = f1; x1 = b - phi * (b - a); f1 = mse_at_step(y, count, (float)x1, L); }
    else          { a = x1; x1 = x2; f1 = f2; x2 = a + phi * (b - a); f2 = mse_at_step(y, count, (float)x2, L); }
  }
  if (f1 < best) { best = f1; best_s = (float)x1; }
  if (f2 < best) { best = f2; best_s = (float)x2; }
  int lo = arg, hi = arg;                         /* grid descends: lo is the smallest such step */
  for (int k = 0; k < KTO_SENS_GRID; ++k)
    if (mse[k] <= (1.0 + flat_tol) * best) { if (k > lo) lo = k; if (k < hi) hi = k; }
  out[0] = (double)best_s;
  out[1] = best;
  out[2] = (double)grid[lo];
  out[3] = (double)grid[hi];
  for (int i = 0; i < n_alpha; ++i) {
    volatile float f = 1.0f + alphas[i];
    const float s = best_s * f;
    gamma[i] = fabs(mse_at_step(y, count, s, L) - best);
  }
  free(mse);
  free(grid);
}
