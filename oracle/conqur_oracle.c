/*
 * CPU oracle for ConQuR's online rotation calibration -- TEST INFRASTRUCTURE.
 *
 * A plain, slow, fp64 restatement of what the calibration hot path computes,
 * written from the paper.  It shares no code with the HIP library and is used
 * only by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg; the product never calls it.
 *
 * Conventions.  Activations are rows (App. A, "X_hat = X R"), so the rotation
 * here is the transpose of the one in Sec. 3 (which writes R x), and the
 * cross-covariance kept here, M = Xn^T C, is the transpose of Sec. 3.3's
 * Z^T Xn; polar(M) is then the same rotation in the row convention.
 *
 *   rotate        y_i   = x_i R_op                          Eq. 1-2 (R x~)
 *   normalise     n_i   = ||x_i||_2 , xn_i = x_i / n_i       Sec. 3.3 (x~)
 *   corner        c_ij  = sgn(y_ij) / sqrt(d), sgn(0) = +1   Eq. 2
 *   accumulate    M    += xn_i^T c_i                         Sec. 3.3 (Z^T X~)
 *   l1 term       L    += ||y_i||_1 / n_i                    Sec. 3.2 identity
 *   Procrustes    M = U S V^T  ->  R = U V^T                 Sec. 3.3
 *   quantiser     q = D * round(y / D), D = max|y| / (2^(b-1) - 1)   App. B
 *
 * All arithmetic is fp64 with naive loops in a fixed summation order; the
 * OpenMP pragmas split only over independent output rows / disjoint column
 * pairs, so results do not depend on the thread count.  The SVD is a one-sided
 * (Hestenes) Jacobi iteration with a round-robin pair ordering.
 *
 * Parity pins: every exported function is pinned by tests/test_oracle_*.py
 * (closed forms, invariants, brute force, planted solutions, library cross
 * checks).  The only unpinned part is the choice of orthogonal completion on
 * the null space of a rank-deficient M with prox_lambda = 0, where every
 * completion is an equally optimal Procrustes solution: "parity unpinned"
 * for the entries of R on that block (the objective value and orthogonality
 * remain pinned).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oq_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Nearest bf16 (8 significant bits, ties to even) of a finite double in the
 * normal range; zero stays zero.  The result is exactly representable. */
double oq_round_bf16_f64(double y) {
  if (y == 0.0 || !isfinite(y)) return y;
  int e = ilogb(y);
  if (e < -126) e = -126; /* bf16 subnormals share the smallest exponent */
  double scaled = ldexp(y, 7 - e);
  return ldexp(nearbyint(scaled), e - 7); /* default rounding mode: ties to even */
}

/* The rotate operand (reading: the operand is the master rotation rounded to
 * the activation dtype).  dtype 0 = f32 (identity), 1 = bf16. */
void oq_round_operand(const float* R, float* R_op, uint64_t n, int dtype) {
  for (uint64_t i = 0; i < n; ++i)
    R_op[i] = dtype == 1 ? (float)oq_round_bf16_f64((double)R[i]) : R[i];
}

/*
 * One batch of the statistics loop (Alg. 1 inner loop; Sec. 3.4).
 *   X      [T][row_stride] floats, the first d entries of each row are used;
 *          head h owns columns [h*dh, (h+1)*dh), dh = d / heads
 *   R_op   [heads][dh][dh]   rotate operand (row convention: y = x R_op)
 *   M      [heads][dh][dh]   fp64 accumulators, updated in place
 *   L, n, skipped [heads]    l1 accumulator, rows used, rows skipped (in place)
 *   Y_out  [T][d] or NULL    rotated rows y (fp64), all rows, skipped ones too
 *   S_out  [T][d] or NULL    corner signs +1 / -1 (0 for skipped rows)
 * A row whose head slice is all zero or holds a non-finite value has no unit
 * vector; it is skipped and counted (reading; the paper leaves it undefined).
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int oq_step_batch(const float* X, uint64_t T, uint64_t d, uint64_t heads, uint64_t row_stride,
                  const float* R_op, double* M, double* L, uint64_t* n, uint64_t* skipped,
                  double* Y_out, int8_t* S_out) {
  if (!X || !R_op || !M || !L || !n || !skipped || heads == 0 || d % heads || row_stride < d) return -1;
  const uint64_t dh = d / heads;
  const double inv_sqrt_d = 1.0 / sqrt((double)dh);
  double* Y = (double*)malloc(sizeof(double) * T * dh);
  double* C = (double*)malloc(sizeof(double) * T * dh);
  double* nrm = (double*)malloc(sizeof(double) * T);
  if (!Y || !C || !nrm) { free(Y); free(C); free(nrm); return -1; }

  for (uint64_t h = 0; h < heads; ++h) {
    const float* Rh = R_op + h * dh * dh;
    double* Mh = M + h * dh * dh;
    /* rotate: y_ij = sum_k x_ik R_op[k][j], k ascending */
#pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < T; ++i) {
      const float* x = X + i * row_stride + h * dh;
      double* y = Y + i * dh;
      for (uint64_t j = 0; j < dh; ++j) y[j] = 0.0;
      for (uint64_t k = 0; k < dh; ++k) {
        const double xik = (double)x[k];
        const float* r = Rh + k * dh;
        for (uint64_t j = 0; j < dh; ++j) y[j] += xik * (double)r[j];
      }
      /* norm of the un-rotated row */
      double ss = 0.0;
      int finite = 1;
      for (uint64_t k = 0; k < dh; ++k) {
        double v = (double)x[k];
        if (!isfinite(v)) finite = 0;
        ss += v * v;
      }
      nrm[i] = (finite && ss > 0.0) ? sqrt(ss) : 0.0; /* 0 marks "skip" */
      /* corner target */
      for (uint64_t j = 0; j < dh; ++j) {
        double s = (y[j] >= 0.0) ? 1.0 : -1.0; /* sgn(0) = sgn(-0) = +1 */
        C[i * dh + j] = nrm[i] > 0.0 ? s * inv_sqrt_d : 0.0;
        if (S_out) S_out[i * d + h * dh + j] = nrm[i] > 0.0 ? (int8_t)s : 0;
        if (Y_out) Y_out[i * d + h * dh + j] = y[j];
      }
    }
    /* l1 term and counts, token order */
    for (uint64_t i = 0; i < T; ++i) {
      if (nrm[i] > 0.0) {
        double l1 = 0.0;
        for (uint64_t j = 0; j < dh; ++j) l1 += fabs(Y[i * dh + j]);
        L[h] += l1 / nrm[i];
        n[h] += 1;
      } else {
        skipped[h] += 1;
      }
    }
    /* accumulate: M[k][j] += (x_ik / n_i) * c_ij, tokens ascending */
#pragma omp parallel for schedule(static)
    for (uint64_t k = 0; k < dh; ++k) {
      double* m = Mh + k * dh;
      for (uint64_t i = 0; i < T; ++i) {
        if (!(nrm[i] > 0.0)) continue;
        const double xn = (double)X[i * row_stride + h * dh + k] / nrm[i];
        const double* c = C + i * dh;
        for (uint64_t j = 0; j < dh; ++j) m[j] += xn * c[j];
      }
    }
  }
  free(Y); free(C); free(nrm);
  return 0;
}

/* ---- one-sided Jacobi SVD ------------------------------------------------ */

/*
 * A [d][d] row-major (fp64).  On return U, V are [d][d] row-major with
 * orthonormal columns and sigma[j] >= 0 (not sorted) such that
 * A = U diag(sigma) V^T.  Columns of U that belong to numerically zero
 * singular values (sigma_j <= d * eps * sigma_max) are an orthonormal
 * completion built by Gram-Schmidt from the standard basis.
 * Returns the number of sweeps used, or -1 on failure.
 */
int oq_jacobi_svd(const double* A, uint64_t d, double* U, double* sigma, double* V) {
  const uint64_t np_ = d + (d & 1); /* players in the round-robin schedule */
  double* Bt = (double*)malloc(sizeof(double) * d * d); /* row p = column p of A V */
  double* Vt = (double*)malloc(sizeof(double) * d * d); /* row p = column p of V   */
  uint64_t* perm = (uint64_t*)malloc(sizeof(uint64_t) * np_);
  if (!Bt || !Vt || !perm) { free(Bt); free(Vt); free(perm); return -1; }
  for (uint64_t i = 0; i < d; ++i)
    for (uint64_t j = 0; j < d; ++j) {
      Bt[j * d + i] = A[i * d + j];
      Vt[j * d + i] = (i == j) ? 1.0 : 0.0;
    }
  const double tol = 1e-15;
  int sweeps = 0;
  for (; sweeps < 80; ++sweeps) {
    uint64_t rotations = 0;
    for (uint64_t i = 0; i < np_; ++i) perm[i] = i;
    for (uint64_t round = 0; round + 1 < np_; ++round) {
#pragma omp parallel for schedule(static) reduction(+ : rotations)
      for (uint64_t t = 0; t < np_ / 2; ++t) {
        uint64_t p = perm[t], q = perm[np_ - 1 - t];
        if (p >= d || q >= d) continue; /* the bye of an odd-sized schedule */
        if (p > q) { uint64_t s_ = p; p = q; q = s_; }
        double* bp = Bt + p * d; double* bq = Bt + q * d;
        double alpha = 0.0, beta = 0.0, gamma = 0.0;
        for (uint64_t r = 0; r < d; ++r) {
          alpha += bp[r] * bp[r]; beta += bq[r] * bq[r]; gamma += bp[r] * bq[r];
        }
        if (fabs(gamma) <= tol * sqrt(alpha * beta) || gamma == 0.0) continue;
        rotations += 1;
        const double zeta = (beta - alpha) / (2.0 * gamma);
        const double tt = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
        const double c = 1.0 / sqrt(1.0 + tt * tt), s = c * tt;
        double* vp = Vt + p * d; double* vq = Vt + q * d;
        for (uint64_t r = 0; r < d; ++r) {
          const double x = bp[r], y = bq[r];
          bp[r] = c * x - s * y; bq[r] = s * x + c * y;
          const double vx = vp[r], vy = vq[r];
          vp[r] = c * vx - s * vy; vq[r] = s * vx + c * vy;
        }
      }
      /* rotate the schedule: player 0 stays, the others shift by one */
      uint64_t last = perm[np_ - 1];
      for (uint64_t i = np_ - 1; i > 1; --i) perm[i] = perm[i - 1];
      perm[1] = last;
    }
    if (rotations == 0) break;
  }
  double smax = 0.0;
  for (uint64_t j = 0; j < d; ++j) {
    double ss = 0.0;
    for (uint64_t r = 0; r < d; ++r) ss += Bt[j * d + r] * Bt[j * d + r];
    sigma[j] = sqrt(ss);
    if (sigma[j] > smax) smax = sigma[j];
  }
  const double cut = (double)d * 2.220446049250313e-16 * smax;
  /* U columns of the non-null part */
  for (uint64_t j = 0; j < d; ++j) {
    if (sigma[j] > cut) {
      for (uint64_t r = 0; r < d; ++r) Bt[j * d + r] /= sigma[j];
    } else {
      sigma[j] = 0.0;
    }
  }
  /* orthonormal completion of the null columns (any completion is optimal) */
  uint64_t remaining = 0;
  for (uint64_t j = 0; j < d; ++j) remaining += (sigma[j] == 0.0);
  if (smax == 0.0) remaining = d;
  uint64_t cand = 0;
  double* w = (double*)malloc(sizeof(double) * d);
  if (!w) { free(Bt); free(Vt); free(perm); return -1; }
  uint8_t* have = (uint8_t*)calloc(d, 1);
  for (uint64_t j = 0; j < d; ++j) have[j] = sigma[j] > 0.0;
  for (uint64_t j = 0; j < d && remaining > 0; ++j) {
    if (have[j]) continue;
    for (;; ++cand) {
      if (cand >= d) { free(w); free(have); free(Bt); free(Vt); free(perm); return -1; }
      for (uint64_t r = 0; r < d; ++r) w[r] = (r == cand) ? 1.0 : 0.0;
      for (int pass = 0; pass < 2; ++pass)
        for (uint64_t c2 = 0; c2 < d; ++c2) {
          if (!have[c2]) continue;
          double dot = 0.0;
          for (uint64_t r = 0; r < d; ++r) dot += w[r] * Bt[c2 * d + r];
          for (uint64_t r = 0; r < d; ++r) w[r] -= dot * Bt[c2 * d + r];
        }
      double ss = 0.0;
      for (uint64_t r = 0; r < d; ++r) ss += w[r] * w[r];
      if (ss >= 0.5 * (double)remaining / (double)d) {
        const double inv = 1.0 / sqrt(ss);
        for (uint64_t r = 0; r < d; ++r) Bt[j * d + r] = w[r] * inv;
        have[j] = 1; remaining -= 1; ++cand;
        break;
      }
    }
  }
  free(w); free(have);
  for (uint64_t i = 0; i < d; ++i)
    for (uint64_t j = 0; j < d; ++j) {
      U[i * d + j] = Bt[j * d + i];
      V[i * d + j] = Vt[j * d + i];
    }
  free(Bt); free(Vt); free(perm);
  return sweeps;
}

/*
 * Orthogonal Procrustes update (Sec. 3.3) for one d x d block.
 *   A = M + lambda * tau * R_prev,  tau = ||M||_F / sqrt(d)
 *   A = U S V^T  ->  R = U V^T
 * lambda = 0 is the paper's update.  lambda > 0 is the proximal reading used
 * when M is rank deficient (fewer tokens than d since the last update): it
 * picks, among the maximisers of <R, M>, the one nearest the previous R.
 *   out: R_new [d][d] fp64; stats[0] = <R_new, M>, stats[1] = sum sigma(A),
 *        stats[2] = ||R_new^T R_new - I||_F, stats[3] = tau, stats[4] = sweeps
 */
int oq_procrustes(const double* M, const double* R_prev, uint64_t d, double lambda,
                  double* R_new, double* stats) {
  double* A = (double*)malloc(sizeof(double) * d * d);
  double* U = (double*)malloc(sizeof(double) * d * d);
  double* V = (double*)malloc(sizeof(double) * d * d);
  double* sg = (double*)malloc(sizeof(double) * d);
  if (!A || !U || !V || !sg) { free(A); free(U); free(V); free(sg); return -1; }
  double fro2 = 0.0;
  for (uint64_t i = 0; i < d * d; ++i) fro2 += M[i] * M[i];
  const double tau = sqrt(fro2) / sqrt((double)d);
  for (uint64_t i = 0; i < d * d; ++i)
    A[i] = M[i] + ((lambda != 0.0 && R_prev) ? lambda * tau * R_prev[i] : 0.0);
  int sweeps = oq_jacobi_svd(A, d, U, sg, V);
  if (sweeps < 0) { free(A); free(U); free(V); free(sg); return -1; }
#pragma omp parallel for schedule(static)
  for (uint64_t i = 0; i < d; ++i)
    for (uint64_t j = 0; j < d; ++j) {
      double acc = 0.0;
      for (uint64_t k = 0; k < d; ++k) acc += U[i * d + k] * V[j * d + k];
      R_new[i * d + j] = acc;
    }
  if (stats) {
    double ip = 0.0, nuc = 0.0;
    for (uint64_t i = 0; i < d * d; ++i) ip += R_new[i] * M[i];
    for (uint64_t j = 0; j < d; ++j) nuc += sg[j];
    double orth2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : orth2)
    for (uint64_t a = 0; a < d; ++a)
      for (uint64_t b = 0; b < d; ++b) {
        double g = 0.0;
        for (uint64_t r = 0; r < d; ++r) g += R_new[r * d + a] * R_new[r * d + b];
        g -= (a == b) ? 1.0 : 0.0;
        orth2 += g * g;
      }
    stats[0] = ip; stats[1] = nuc; stats[2] = sqrt(orth2); stats[3] = tau; stats[4] = (double)sweeps;
  }
  free(A); free(U); free(V); free(sg);
  return 0;
}

/*
 * Per-token symmetric b-bit fake-quantisation error of the rotated rows
 * (App. B, symmetric quantiser; Sec. 4.3 error metric).
 *   y = x R_op per head (fp64), stored in the activation dtype (dtype 1:
 *   rounded to bf16; dtype 0: rounded to fp32) -- the tensor a quantised
 *   linear layer would receive.  One scale per token over the whole row of
 *   width d:  D = max_j |y_j| / (2^(b-1) - 1),  q_j = D * rint(y_j / D)
 *   clamped to the level range; a zero row has zero error.
 * The integer code is decided in fp32 (the kernel's precision): D and y / D
 * are single-precision operations; the squared error is summed in fp64.
 *   out: *sse = sum (y - q)^2, *energy = sum y^2, row_sse[T] optional,
 *        codes[T][d] optional (int8).
 */
int oq_quant_error(const float* X, uint64_t T, uint64_t d, uint64_t heads, uint64_t row_stride,
                   const float* R_op, int dtype, int bits, double* sse, double* energy,
                   double* row_sse, int8_t* codes) {
  if (!X || !R_op || heads == 0 || d % heads || row_stride < d || bits < 2 || bits > 8) return -1;
  const uint64_t dh = d / heads;
  const float qmax = (float)((1 << (bits - 1)) - 1);
  double* rs = (double*)calloc(T, sizeof(double));
  double* re = (double*)calloc(T, sizeof(double));
  if (!rs || !re) { free(rs); free(re); return -1; }
#pragma omp parallel
  {
    double* y = (double*)malloc(sizeof(double) * d);
#pragma omp for schedule(static)
    for (uint64_t i = 0; i < T; ++i) {
      for (uint64_t h = 0; h < heads; ++h) {
        const float* x = X + i * row_stride + h * dh;
        const float* Rh = R_op + h * dh * dh;
        double* yh = y + h * dh;
        for (uint64_t j = 0; j < dh; ++j) yh[j] = 0.0;
        for (uint64_t k = 0; k < dh; ++k) {
          const double xik = (double)x[k];
          for (uint64_t j = 0; j < dh; ++j) yh[j] += xik * (double)Rh[k * dh + j];
        }
      }
      float amax = 0.0f;
      for (uint64_t j = 0; j < d; ++j) {
        y[j] = dtype == 1 ? oq_round_bf16_f64(y[j]) : (double)(float)y[j];
        float a = fabsf((float)y[j]);
        if (a > amax) amax = a;
      }
      double s = 0.0, e = 0.0;
      const float delta = amax / qmax;
      for (uint64_t j = 0; j < d; ++j) {
        float code = 0.0f;
        if (amax > 0.0f) {
          code = rintf((float)y[j] / delta);
          if (code > qmax) code = qmax;
          if (code < -qmax) code = -qmax;
        }
        const double q = (double)delta * (double)code;
        s += (y[j] - q) * (y[j] - q);
        e += y[j] * y[j];
        if (codes) codes[i * d + j] = (int8_t)code;
      }
      rs[i] = s; re[i] = e;
    }
    free(y);
  }
  double S = 0.0, E = 0.0;
  for (uint64_t i = 0; i < T; ++i) { S += rs[i]; E += re[i]; if (row_sse) row_sse[i] = rs[i]; }
  if (sse) *sse = S;
  if (energy) *energy = E;
  free(rs); free(re);
  return 0;
}

/*
 * Per-token asymmetric (zero-point) b-bit fake-quantisation error of the rotated rows
 * (App. B, "per-tensor asymmetric (zeropoint) quantizer": the affine range
 * [min_j y_j, max_j y_j] is mapped onto the unsigned grid {0, ..., 2^b - 1}; App. C
 * evaluates activations with a clipping ratio of 0.9).
 *   y as in oq_quant_error (x R_op per head, stored in the activation dtype).
 *   Per token, over the whole row of width d:
 *     lo = clip * min_j y_j,  hi = clip * max_j y_j        (clip in (0, 1]; 1 = the appendix's quantiser)
 *     D = (hi - lo) / (2^b - 1),  zeta = -rint(lo / D)     (integer zero point: lo lands on code 0)
 *     code_j = clamp(rint(y_j / D) + zeta, 0, 2^b - 1),  q_j = D * (code_j - zeta)
 *   A row with hi = lo (constant row) has the single level lo: q_j = lo.
 * As for the symmetric quantiser the integer code is decided in fp32 (lo, hi, D, y / D
 * are single-precision operations); the squared error is summed in fp64.
 *   out: *sse = sum (y - q)^2, *energy = sum y^2, row_sse[T] optional, codes[T][d] optional (uint8).
 */
int oq_quant_error_zp(const float* X, uint64_t T, uint64_t d, uint64_t heads, uint64_t row_stride,
                      const float* R_op, int dtype, int bits, float clip, double* sse, double* energy,
                      double* row_sse, uint8_t* codes) {
  if (!X || !R_op || heads == 0 || d % heads || row_stride < d || bits < 2 || bits > 8 || !(clip > 0.0f) || clip > 1.0f)
    return -1;
  const uint64_t dh = d / heads;
  const float qtop = (float)((1 << bits) - 1);
  double* rs = (double*)calloc(T, sizeof(double));
  double* re = (double*)calloc(T, sizeof(double));
  if (!rs || !re) { free(rs); free(re); return -1; }
#pragma omp parallel
  {
    double* y = (double*)malloc(sizeof(double) * d);
#pragma omp for schedule(static)
    for (uint64_t i = 0; i < T; ++i) {
      for (uint64_t h = 0; h < heads; ++h) {
        const float* x = X + i * row_stride + h * dh;
        const float* Rh = R_op + h * dh * dh;
        double* yh = y + h * dh;
        for (uint64_t j = 0; j < dh; ++j) yh[j] = 0.0;
        for (uint64_t k = 0; k < dh; ++k) {
          const double xik = (double)x[k];
          for (uint64_t j = 0; j < dh; ++j) yh[j] += xik * (double)Rh[k * dh + j];
        }
      }
      float mn = 0.0f, mx = 0.0f;
      for (uint64_t j = 0; j < d; ++j) {
        y[j] = dtype == 1 ? oq_round_bf16_f64(y[j]) : (double)(float)y[j];
        const float v = (float)y[j];
        if (j == 0 || v < mn) mn = v;
        if (j == 0 || v > mx) mx = v;
      }
      const float lo = clip * mn, hi = clip * mx;
      const float delta = (hi - lo) / qtop;
      const float zeta = delta > 0.0f ? -rintf(lo / delta) : 0.0f;
      double s = 0.0, e = 0.0;
      for (uint64_t j = 0; j < d; ++j) {
        double q;
        float code = 0.0f;
        if (delta > 0.0f) {
          code = rintf((float)y[j] / delta) + zeta;
          if (code > qtop) code = qtop;
          if (code < 0.0f) code = 0.0f;
          q = (double)delta * ((double)code - (double)zeta);
        } else {
          q = (double)lo;
        }
        s += (y[j] - q) * (y[j] - q);
        e += y[j] * y[j];
        if (codes) codes[i * d + j] = (uint8_t)code;
      }
      rs[i] = s; re[i] = e;
    }
    free(y);
  }
  double S = 0.0, E = 0.0;
  for (uint64_t i = 0; i < T; ++i) { S += rs[i]; E += re[i]; if (row_sse) row_sse[i] = rs[i]; }
  if (sse) *sse = S;
  if (energy) *energy = E;
  free(rs); free(re);
  return 0;
}

/*
 * Per-row diagnostics of the rotated activations (Sec. 4.2 and App. B):
 *   y as in oq_quant_error (x R_op per head, stored in the activation dtype), whole row of width d;
 *   pr[i]  = PR(y)/d = ||y||_2^4 / (d ||y||_4^4)          in [1/d, 1]   (normalised participation ratio)
 *   rho[i] = ||y||_inf^2 / ||y||_2^2                       in [1/d, 1]   (dynamic-range ratio of the SQNR bound)
 * A row with zero or non-finite energy gets pr = rho = 0.  All arithmetic in fp64.
 */
int oq_row_diagnostics(const float* X, uint64_t T, uint64_t d, uint64_t heads, uint64_t row_stride,
                       const float* R_op, int dtype, double* pr, double* rho) {
  if (!X || !R_op || heads == 0 || d % heads || row_stride < d) return -1;
  const uint64_t dh = d / heads;
#pragma omp parallel
  {
    double* y = (double*)malloc(sizeof(double) * d);
#pragma omp for schedule(static)
    for (uint64_t i = 0; i < T; ++i) {
      for (uint64_t h = 0; h < heads; ++h) {
        const float* x = X + i * row_stride + h * dh;
        const float* Rh = R_op + h * dh * dh;
        double* yh = y + h * dh;
        for (uint64_t j = 0; j < dh; ++j) yh[j] = 0.0;
        for (uint64_t k = 0; k < dh; ++k) {
          const double xik = (double)x[k];
          for (uint64_t j = 0; j < dh; ++j) yh[j] += xik * (double)Rh[k * dh + j];
        }
      }
      double s2 = 0.0, s4 = 0.0, mx = 0.0;
      for (uint64_t j = 0; j < d; ++j) {
        y[j] = dtype == 1 ? oq_round_bf16_f64(y[j]) : (double)(float)y[j];
        const double a = fabs(y[j]);
        if (a > mx) mx = a;
      }
      /* scaled by the row maximum so that fourth powers neither overflow nor vanish */
      for (uint64_t j = 0; j < d; ++j) {
        const double u = mx > 0.0 ? y[j] / mx : 0.0;
        s2 += u * u;
        s4 += u * u * u * u;
      }
      const int ok = mx > 0.0 && isfinite(mx) && isfinite(s2);
      if (pr) pr[i] = ok ? s2 * s2 / ((double)d * s4) : 0.0;
      if (rho) rho[i] = ok ? 1.0 / s2 : 0.0;
    }
    free(y);
  }
  return 0;
}

/*
 * The rotated rows themselves: Y = X R_op per head (fp64 accumulation), stored in the
 * activation dtype (dtype 1: rounded to bf16; dtype 0: rounded to fp32) -- Eq. 1's R x~ before
 * normalisation, and, with the rows of a weight matrix as X, the folding of the
 * learned rotation into that matrix (App. A).  Y: T rows of d floats.
 */
int oq_rotate(const float* X, uint64_t T, uint64_t d, uint64_t heads, uint64_t row_stride, const float* R_op, int dtype,
              float* Y) {
  if (!X || !R_op || !Y || heads == 0 || d % heads || row_stride < d) return -1;
  const uint64_t dh = d / heads;
#pragma omp parallel
  {
    double* y = (double*)malloc(sizeof(double) * dh);
#pragma omp for schedule(static)
    for (uint64_t i = 0; i < T; ++i)
      for (uint64_t h = 0; h < heads; ++h) {
        const float* x = X + i * row_stride + h * dh;
        const float* Rh = R_op + h * dh * dh;
        for (uint64_t j = 0; j < dh; ++j) y[j] = 0.0;
        for (uint64_t k = 0; k < dh; ++k) {
          const double xik = (double)x[k];
          for (uint64_t j = 0; j < dh; ++j) y[j] += xik * (double)Rh[k * dh + j];
        }
        for (uint64_t j = 0; j < dh; ++j)
          Y[i * d + h * dh + j] = dtype == 1 ? (float)oq_round_bf16_f64(y[j]) : (float)y[j];
      }
    free(y);
  }
  return 0;
}

/*
 * The fake-quantised rotated rows themselves: what a linear layer receives when its input is
 * quantised after the current rotation has been applied (Sec. 3.4, quantisation-aware calibration;
 * quantisers of App. B, clipping ratio of App. C).
 *   y = x R_op per head, stored in the activation dtype (as in oq_rotate);
 *   zero_point = 0: symmetric, D = max_j |y_j| / (2^(b-1) - 1), q_j = D clamp(rint(y_j / D), -qmax, qmax);
 *   zero_point = 1: range [clip min_j y_j, clip max_j y_j] on {0 .. 2^b - 1} with the integer zero point,
 *                   q_j = D (code_j - zeta), a constant row keeps its single level (see oq_quant_error_zp).
 *   The code is decided in fp32 as in the two error functions; q_j is the exact product D * (integer),
 *   rounded once into the activation dtype.  Yq: T rows of d floats.
 */
int oq_fake_quant(const float* X, uint64_t T, uint64_t d, uint64_t heads, uint64_t row_stride, const float* R_op, int dtype,
                  int bits, int zero_point, float clip, float* Yq) {
  if (!X || !R_op || !Yq || heads == 0 || d % heads || row_stride < d || bits < 2 || bits > 8) return -1;
  if (zero_point && (!(clip > 0.0f) || clip > 1.0f)) return -1;
  const uint64_t dh = d / heads;
  const float qsym = (float)((1 << (bits - 1)) - 1), qtop = (float)((1 << bits) - 1);
#pragma omp parallel
  {
    double* y = (double*)malloc(sizeof(double) * d);
#pragma omp for schedule(static)
    for (uint64_t i = 0; i < T; ++i) {
      for (uint64_t h = 0; h < heads; ++h) {
        const float* x = X + i * row_stride + h * dh;
        const float* Rh = R_op + h * dh * dh;
        double* yh = y + h * dh;
        for (uint64_t j = 0; j < dh; ++j) yh[j] = 0.0;
        for (uint64_t k = 0; k < dh; ++k) {
          const double xik = (double)x[k];
          for (uint64_t j = 0; j < dh; ++j) yh[j] += xik * (double)Rh[k * dh + j];
        }
      }
      float mn = 0.0f, mx = 0.0f, amax = 0.0f;
      for (uint64_t j = 0; j < d; ++j) {
        y[j] = dtype == 1 ? oq_round_bf16_f64(y[j]) : (double)(float)y[j];
        const float v = (float)y[j];
        if (j == 0 || v < mn) mn = v;
        if (j == 0 || v > mx) mx = v;
        if (fabsf(v) > amax) amax = fabsf(v);
      }
      for (uint64_t j = 0; j < d; ++j) {
        double q;
        if (zero_point) {
          const float lo = clip * mn, hi = clip * mx;
          const float delta = (hi - lo) / qtop;
          if (delta > 0.0f) {
            const float zeta = -rintf(lo / delta);
            float code = rintf((float)y[j] / delta) + zeta;
            if (code > qtop) code = qtop;
            if (code < 0.0f) code = 0.0f;
            q = (double)delta * ((double)code - (double)zeta);
          } else {
            q = (double)lo;
          }
        } else {
          const float delta = amax / qsym;
          float code = 0.0f;
          if (amax > 0.0f) {
            code = rintf((float)y[j] / delta);
            if (code > qsym) code = qsym;
            if (code < -qsym) code = -qsym;
          }
          q = (double)delta * (double)code;
        }
        Yq[i * d + j] = dtype == 1 ? (float)oq_round_bf16_f64(q) : (float)q;
      }
    }
    free(y);
  }
  return 0;
}
