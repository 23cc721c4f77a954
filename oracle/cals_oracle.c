/*
 * cals_oracle.c -- plain CPU reference ("oracle") for Concurrent ALS on a dense fp64 tensor of order 3
 * (the routines without a suffix) or of any order from 3 to ORACLE_MAX_MODES (the routines ending in _nd; Alg. 1
 * is stated for N modes).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, obviously-correct statement of what the GPU
 * path must compute.  Only the test-suite, the smoke check and the benchmark's CPU-baseline
 * leg may call it; the product library never does, and the two share no code.
 *
 * What is written out here, and from where in the paper:
 *   - MTTKRP by its element-wise definition (Alg. 1, the MTTKRP line; Sec. 3.1):
 *       M(n)[i_n, r] = sum over the other two indices of T[i1,i2,i3] * (Ua[ia,r] * Ub[ib,r]).
 *     The fused multi-model MTTKRP of Eq. (2) is this same definition applied to the
 *     concatenated factor matrices, so one routine serves both.  For N modes the product runs over
 *     the N-1 other factor matrices and the sum over the N-1 other indices (the _nd routines).
 *   - Hadamard product of Gramians, the normal-equation update, and the fast error formula
 *     (Alg. 1, remaining lines), per model (Alg. 2: "instances are treated separately").
 *   - Queue handling of Alg. 3: fill from the queue front until the next model does not fit,
 *     advance every active model one iteration, retire in slot order, keep survivors' order.
 *   - Line search (Sec. 5, "Line search") and non-negativity by an active-set method
 *     (Sec. 5, "Non-negativity constraints").
 *
 * Readings where the paper is silent or garbled (each is repeated in the design notes):
 *   - memory order: first index fastest, T[i1 + I1*(i2 + I2*i3)]; factor matrices column-major.
 *   - the printed error formula has the sign of its middle term wrong for a squared residual;
 *     used here: e = ||T||^2 + sum(H(N) * U(N)^T U(N)) - 2 sum(U(N) * M(N)).
 *   - fit F = 1 - sqrt(max(e,0)) / ||T||; a model stops when it >= 2 and |F - F_prev| < tol,
 *     or when it == max_iters.
 *   - the update is U(n) = M(n) H(n)^+ (Alg. 1, update line).  While H(n) is numerically positive definite --
 *     every Cholesky pivot above ORACLE_RANK_TOL times its diagonal entry -- the pseudo-inverse is the inverse and
 *     is applied through the Cholesky factor.  Otherwise H(n)^+ = V diag(1/l_i : l_i > ORACLE_RANK_TOL * l_max) V^T
 *     from the symmetric eigen-decomposition (cyclic Jacobi).  A non-finite H(n), or one without a positive
 *     eigenvalue, stops the model with status NUMERICAL, leaving the factors it had before the failing update.
 *   - every column of an updated factor is scaled to unit 2-norm, the norms kept in lambda.
 *   - non-negativity together with line search (the paper describes each alone): the extrapolated point is
 *     clipped at zero entry by entry before its error is evaluated, so every point a NONNEG model visits is feasible.
 *   - non-negativity: Lawson-Hanson active set on the normal equations per row; the passive set of the
 *     previous iteration is a warm start that is dropped when its sub-block of H is not positive definite.
 *   - order 3: sums over the two contracted indices are nested: the inner sum runs over the lower-
 *     numbered contracted mode into a fresh accumulator, the outer sum adds those up.  Higher orders:
 *     one running sum per output element over the contracted indices in memory order.
 *   - for N modes the error terms come from the update of mode N, and line search folds lambda into
 *     the factor of mode N (for N = 3 this is what the order-3 routines always did).
 *
 * Pins: every routine below is pinned in the CPU test-suite by something other than itself -- brute force on
 * tiny inputs, identities, closed forms, special cases that reduce to library routines (LAPACK Cholesky and
 * least squares, scipy's Lawson-Hanson), hand-computed queue schedules.  The paper prints no worked numeric
 * example (no factor, fit or error values), so none of the pins is a printed value.
 *
 * Build: gcc -O3 -fopenmp -fPIC -shared -o liboracle.so cals_oracle.c -lm
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_RUNNING 0
#define ORACLE_CONVERGED 1
#define ORACLE_MAX_ITERS 2
#define ORACLE_NUMERICAL 3

#define ORACLE_FLAG_NONNEG 1u
#define ORACLE_FLAG_LINESEARCH 2u

#define ORACLE_MAX_RANK 32
#define ORACLE_MAX_MODES 6
#define ORACLE_RANK_TOL 1e-12   /* relative size below which a pivot or an eigenvalue counts as zero */

/* ------------------------------------------------------------------------------------------ */
/* small dense helpers                                                                         */
/* ------------------------------------------------------------------------------------------ */

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ||T||^2, summed slab by slab (inner sums over a fibre, then a slab, then all slabs). */
double oracle_norm_sq(const double* T, const int64_t* dims) {
  const int64_t I1 = dims[0], I2 = dims[1], I3 = dims[2];
  double total = 0.0;
  for (int64_t i3 = 0; i3 < I3; ++i3) {
    double slab = 0.0;
    for (int64_t i2 = 0; i2 < I2; ++i2) {
      double fibre = 0.0;
      const double* t = T + I1 * (i2 + I2 * i3);
      for (int64_t i1 = 0; i1 < I1; ++i1) fibre += t[i1] * t[i1];
      slab += fibre;
    }
    total += slab;
  }
  return total;
}

/* ||T||^2 of an order-N tensor: fibres along the first index, summed per value of the last index, then added up
 * (for N = 3 the same order of additions as oracle_norm_sq). */
double oracle_norm_sq_nd(const double* T, int N, const int64_t* dims) {
  const int64_t I1 = dims[0], IN = dims[N - 1];
  int64_t fibres = 1;
  for (int n = 1; n < N - 1; ++n) fibres *= dims[n];
  double total = 0.0;
  for (int64_t s = 0; s < IN; ++s) {
    double slab = 0.0;
    for (int64_t f = 0; f < fibres; ++f) {
      double fibre = 0.0;
      const double* t = T + I1 * (f + fibres * s);
      for (int64_t i1 = 0; i1 < I1; ++i1) fibre += t[i1] * t[i1];
      slab += fibre;
    }
    total += slab;
  }
  return total;
}

/* G = U^T U for a column-major I x R matrix (Alg. 1, Gramians). */
void oracle_gram(const double* U, int64_t I, int R, double* G) {
  for (int r = 0; r < R; ++r)
    for (int s = 0; s < R; ++s) {
      double acc = 0.0;
      for (int64_t i = 0; i < I; ++i) acc += U[i + I * r] * U[i + I * s];
      G[r + R * s] = acc;
    }
}

/* H = Ga * Gb element-wise (Alg. 1, Hadamard product of Gramians). */
void oracle_hadamard(const double* Ga, const double* Gb, int R, double* H) {
  for (int e = 0; e < R * R; ++e) H[e] = Ga[e] * Gb[e];
}

/* Lower Cholesky factor of the symmetric R x R matrix H (column-major, lower part read).
 * Returns 0, or 1 when a pivot is not a positive finite number. */
int oracle_cholesky(const double* H, int R, double* L) {
  for (int e = 0; e < R * R; ++e) L[e] = 0.0;
  for (int j = 0; j < R; ++j) {
    double d = H[j + R * j];
    for (int k = 0; k < j; ++k) d -= L[j + R * k] * L[j + R * k];
    if (!(d > 0.0) || !isfinite(d)) return 1;
    d = sqrt(d);
    L[j + R * j] = d;
    for (int i = j + 1; i < R; ++i) {
      double v = H[i + R * j];
      for (int k = 0; k < j; ++k) v -= L[i + R * k] * L[j + R * k];
      L[i + R * j] = v / d;
    }
  }
  return 0;
}

/* The same factorisation for the plain update: H counts as (numerically) positive definite only if every pivot
 * exceeds ORACLE_RANK_TOL times the diagonal entry it started from.  Returns 0, or 1 when it does not. */
int oracle_cholesky_definite(const double* H, int R, double* L) {
  for (int e = 0; e < R * R; ++e) L[e] = 0.0;
  for (int j = 0; j < R; ++j) {
    double d = H[j + R * j];
    for (int k = 0; k < j; ++k) d -= L[j + R * k] * L[j + R * k];
    if (!(d > ORACLE_RANK_TOL * H[j + R * j]) || !isfinite(d)) return 1;
    d = sqrt(d);
    L[j + R * j] = d;
    for (int i = j + 1; i < R; ++i) {
      double v = H[i + R * j];
      for (int k = 0; k < j; ++k) v -= L[i + R * k] * L[j + R * k];
      L[i + R * j] = v / d;
    }
  }
  return 0;
}

/* Eigen-decomposition of the symmetric R x R matrix A by cyclic Jacobi rotations (rows p < q in order, sweep after
 * sweep until the off-diagonal part is negligible).  On exit the diagonal of A holds the eigenvalues and the
 * columns of V the eigenvectors (both column-major). */
static void jacobi_eigen(double* A, int R, double* V) {
  for (int e = 0; e < R * R; ++e) V[e] = 0.0;
  for (int i = 0; i < R; ++i) V[i + R * i] = 1.0;
  for (int sweep = 0; sweep < 100; ++sweep) {
    double off = 0.0, all = 0.0;
    for (int q = 0; q < R; ++q)
      for (int p = 0; p < R; ++p) {
        all += A[p + R * q] * A[p + R * q];
        if (p != q) off += A[p + R * q] * A[p + R * q];
      }
    if (!(off > 1e-34 * all)) break;
    for (int p = 0; p < R - 1; ++p)
      for (int q = p + 1; q < R; ++q) {
        const double apq = A[p + R * q];
        if (apq == 0.0) continue;
        /* rotation angle that annihilates A[p,q]: t = tan, the smaller root of t^2 + 2 tau t - 1 = 0 */
        const double tau = (A[q + R * q] - A[p + R * p]) / (2.0 * apq);
        const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
        const double c = 1.0 / sqrt(1.0 + t * t), sn = t * c;
        for (int k = 0; k < R; ++k) {          /* A <- A J (columns p, q) */
          const double akp = A[k + R * p], akq = A[k + R * q];
          A[k + R * p] = c * akp - sn * akq;
          A[k + R * q] = sn * akp + c * akq;
        }
        for (int k = 0; k < R; ++k) {          /* A <- J^T A (rows p, q) */
          const double apk = A[p + R * k], aqk = A[q + R * k];
          A[p + R * k] = c * apk - sn * aqk;
          A[q + R * k] = sn * apk + c * aqk;
        }
        for (int k = 0; k < R; ++k) {          /* V <- V J */
          const double vkp = V[k + R * p], vkq = V[k + R * q];
          V[k + R * p] = c * vkp - sn * vkq;
          V[k + R * q] = sn * vkp + c * vkq;
        }
      }
  }
}

/* Pseudo-inverse of the symmetric positive semi-definite R x R matrix H: P = sum over the eigenpairs with
 * l_i > ORACLE_RANK_TOL * l_max of v_i v_i^T / l_i.  *rank receives the number of eigenvalues kept.
 * Returns 0, or 1 when H has a non-finite entry or no positive eigenvalue. */
int oracle_pinv_sym(const double* H, int R, double* P, int* rank) {
  double A[ORACLE_MAX_RANK * ORACLE_MAX_RANK], V[ORACLE_MAX_RANK * ORACLE_MAX_RANK];
  if (rank) *rank = 0;
  for (int e = 0; e < R * R; ++e) {
    if (!isfinite(H[e])) return 1;
    A[e] = H[e];
  }
  jacobi_eigen(A, R, V);
  double lmax = 0.0;
  for (int i = 0; i < R; ++i) if (A[i + R * i] > lmax) lmax = A[i + R * i];
  if (!(lmax > 0.0)) return 1;
  for (int e = 0; e < R * R; ++e) P[e] = 0.0;
  int kept = 0;
  for (int i = 0; i < R; ++i) {
    const double l = A[i + R * i];
    if (!(l > ORACLE_RANK_TOL * lmax)) continue;
    kept += 1;
    for (int c = 0; c < R; ++c)
      for (int r = 0; r < R; ++r) P[r + R * c] += V[r + R * i] * V[c + R * i] / l;
  }
  if (rank) *rank = kept;
  return 0;
}

/* Solve (L L^T) x = b in place. */
void oracle_cholesky_solve(const double* L, int R, double* x) {
  for (int i = 0; i < R; ++i) {
    double v = x[i];
    for (int k = 0; k < i; ++k) v -= L[i + R * k] * x[k];
    x[i] = v / L[i + R * i];
  }
  for (int i = R - 1; i >= 0; --i) {
    double v = x[i];
    for (int k = i + 1; k < R; ++k) v -= L[k + R * i] * x[k];
    x[i] = v / L[i + R * i];
  }
}

/* ------------------------------------------------------------------------------------------ */
/* MTTKRP by definition                                                                        */
/* ------------------------------------------------------------------------------------------ */

/* Columns [c0, c0+nc) of the mode-`mode` MTTKRP (mode = 1, 2, 3).  U1,U2,U3 are column-major
 * with leading dimensions I1,I2,I3 and at least c0+nc columns; M is column-major, ld = I_mode.
 * `acc` is scratch of I_mode*nc doubles (modes 1,2) or nc doubles (mode 3). */
static void mttkrp_columns(const double* T, const int64_t* dims, int mode, const double* U1, const double* U2,
                           const double* U3, int64_t c0, int nc, double* M, double* acc) {
  const int64_t I1 = dims[0], I2 = dims[1], I3 = dims[2];
  double krp[ORACLE_MAX_RANK];
  if (mode == 1) {
    /* M1[i1,r] = sum_i3 ( sum_i2 T[i1,i2,i3] * (U2[i2,r] * U3[i3,r]) ) */
    for (int64_t e = 0; e < I1 * nc; ++e) M[e] = 0.0;
    for (int64_t i3 = 0; i3 < I3; ++i3) {
      for (int64_t e = 0; e < I1 * nc; ++e) acc[e] = 0.0;
      for (int64_t i2 = 0; i2 < I2; ++i2) {
        const double* t = T + I1 * (i2 + I2 * i3);
        for (int r = 0; r < nc; ++r) krp[r] = U2[i2 + I2 * (c0 + r)] * U3[i3 + I3 * (c0 + r)];
        for (int r = 0; r < nc; ++r) {
          double* a = acc + I1 * r;
          const double k = krp[r];
          for (int64_t i1 = 0; i1 < I1; ++i1) a[i1] += t[i1] * k;
        }
      }
      for (int64_t e = 0; e < I1 * nc; ++e) M[e] += acc[e];
    }
  } else if (mode == 2) {
    /* M2[i2,r] = sum_i3 ( sum_i1 T[i1,i2,i3] * (U1[i1,r] * U3[i3,r]) ) */
    for (int64_t e = 0; e < I2 * nc; ++e) M[e] = 0.0;
    for (int64_t i3 = 0; i3 < I3; ++i3) {
      for (int64_t i2 = 0; i2 < I2; ++i2) {
        const double* t = T + I1 * (i2 + I2 * i3);
        for (int r = 0; r < nc; ++r) acc[r] = 0.0;
        for (int64_t i1 = 0; i1 < I1; ++i1) {
          const double tv = t[i1];
          for (int r = 0; r < nc; ++r) acc[r] += tv * (U1[i1 + I1 * (c0 + r)] * U3[i3 + I3 * (c0 + r)]);
        }
        for (int r = 0; r < nc; ++r) M[i2 + I2 * r] += acc[r];
      }
    }
  } else {
    /* M3[i3,r] = sum_i2 ( sum_i1 T[i1,i2,i3] * (U1[i1,r] * U2[i2,r]) ) */
    for (int64_t i3 = 0; i3 < I3; ++i3) {
      double outer[ORACLE_MAX_RANK];
      for (int r = 0; r < nc; ++r) outer[r] = 0.0;
      for (int64_t i2 = 0; i2 < I2; ++i2) {
        const double* t = T + I1 * (i2 + I2 * i3);
        for (int r = 0; r < nc; ++r) acc[r] = 0.0;
        for (int64_t i1 = 0; i1 < I1; ++i1) {
          const double tv = t[i1];
          for (int r = 0; r < nc; ++r) acc[r] += tv * (U1[i1 + I1 * (c0 + r)] * U2[i2 + I2 * (c0 + r)]);
        }
        for (int r = 0; r < nc; ++r) outer[r] += acc[r];
      }
      for (int r = 0; r < nc; ++r) M[i3 + I3 * r] = outer[r];
    }
  }
}

/* MTTKRP for R columns (any R): M (I_mode x R, column-major) = T_(mode) (KRP of the other two).
 * With concatenated factor matrices this is the fused multi-model MTTKRP of Eq. (2).
 * Columns are independent, so they are handed out in blocks to threads; the value of every
 * output element does not depend on the number of threads. */
void oracle_mttkrp(const double* T, const int64_t* dims, int mode, int64_t R, const double* U1, const double* U2,
                   const double* U3, double* M) {
  const int64_t In = dims[mode - 1];
  const int blk = 8;
  const int64_t nblk = (R + blk - 1) / blk;
#pragma omp parallel
  {
    double* acc = (double*)malloc(sizeof(double) * (size_t)(In * blk + blk));
#pragma omp for schedule(dynamic, 1)
    for (int64_t b = 0; b < nblk; ++b) {
      const int64_t c0 = b * blk;
      const int nc = (int)((R - c0 < blk) ? (R - c0) : blk);
      mttkrp_columns(T, dims, mode, U1, U2, U3, c0, nc, M + In * c0, acc);
    }
    free(acc);
  }
}

/* One element of the MTTKRP in extended precision, and the sum of the absolute values of its
 * terms (the scale against which a rounding error of that element is judged). */
void oracle_mttkrp_element(const double* T, const int64_t* dims, int mode, const double* U1, const double* U2,
                           const double* U3, int64_t row, int64_t col, double* value, double* abs_sum) {
  const int64_t I1 = dims[0], I2 = dims[1], I3 = dims[2];
  long double s = 0.0L, sa = 0.0L;
  if (mode == 1) {
    for (int64_t i3 = 0; i3 < I3; ++i3)
      for (int64_t i2 = 0; i2 < I2; ++i2) {
        double k = U2[i2 + I2 * col] * U3[i3 + I3 * col];
        long double term = (long double)T[row + I1 * (i2 + I2 * i3)] * (long double)k;
        s += term; sa += fabsl(term);
      }
  } else if (mode == 2) {
    for (int64_t i3 = 0; i3 < I3; ++i3)
      for (int64_t i1 = 0; i1 < I1; ++i1) {
        double k = U1[i1 + I1 * col] * U3[i3 + I3 * col];
        long double term = (long double)T[i1 + I1 * (row + I2 * i3)] * (long double)k;
        s += term; sa += fabsl(term);
      }
  } else {
    for (int64_t i2 = 0; i2 < I2; ++i2)
      for (int64_t i1 = 0; i1 < I1; ++i1) {
        double k = U1[i1 + I1 * col] * U2[i2 + I2 * col];
        long double term = (long double)T[i1 + I1 * (i2 + I2 * row)] * (long double)k;
        s += term; sa += fabsl(term);
      }
  }
  *value = (double)s;
  *abs_sum = (double)sa;
}

/* Order-N MTTKRP by its definition (Alg. 1, the MTTKRP line, for N modes; mode = 1..N):
 *   M[i_mode, r] = sum over all other indices of T[i_1,...,i_N] * prod_{m != mode} U_m[i_m, r].
 * The tensor is walked once in memory order (first index fastest); every element adds its term straight into the
 * output element it belongs to, so each output element is one running sum over the contracted indices in memory
 * order.  The product of factor entries is taken in increasing mode order.  Columns [c0, c0+nc); M is column-major
 * with ld = I_mode and is written from its first column on. */
static void mttkrp_columns_nd(const double* T, int N, const int64_t* dims, int mode, const double* const* U,
                              int64_t c0, int nc, double* M) {
  const int n = mode - 1;
  const int64_t In = dims[n];
  int64_t idx[ORACLE_MAX_MODES];
  int64_t total = 1;
  for (int m = 0; m < N; ++m) { idx[m] = 0; total *= dims[m]; }
  for (int64_t e = 0; e < In * nc; ++e) M[e] = 0.0;
  for (int64_t e = 0; e < total; ++e) {
    const double tv = T[e];
    for (int r = 0; r < nc; ++r) {
      double k = 1.0;
      int first = 1;
      for (int m = 0; m < N; ++m) {
        if (m == n) continue;
        const double u = U[m][idx[m] + dims[m] * (c0 + r)];
        k = first ? u : k * u;
        first = 0;
      }
      M[idx[n] + In * r] += tv * k;
    }
    for (int m = 0; m < N; ++m) {             /* next index tuple, first index fastest */
      if (++idx[m] < dims[m]) break;
      idx[m] = 0;
    }
  }
}

/* Order-N MTTKRP for R columns (any R; fused or not), columns handed out to threads in blocks. */
void oracle_mttkrp_nd(const double* T, int N, const int64_t* dims, int mode, int64_t R, const double* const* U,
                      double* M) {
  const int64_t In = dims[mode - 1];
  const int blk = 8;
  const int64_t nblk = (R + blk - 1) / blk;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t b = 0; b < nblk; ++b) {
    const int64_t c0 = b * blk;
    const int nc = (int)((R - c0 < blk) ? (R - c0) : blk);
    mttkrp_columns_nd(T, N, dims, mode, U, c0, nc, M + In * c0);
  }
}

/* One element of the order-N MTTKRP in extended precision, and the sum of the absolute values of its terms. */
void oracle_mttkrp_element_nd(const double* T, int N, const int64_t* dims, int mode, const double* const* U,
                              int64_t row, int64_t col, double* value, double* abs_sum) {
  const int n = mode - 1;
  int64_t idx[ORACLE_MAX_MODES], stride[ORACLE_MAX_MODES];
  int64_t others = 1, s = 1;
  for (int m = 0; m < N; ++m) { idx[m] = 0; stride[m] = s; s *= dims[m]; if (m != n) others *= dims[m]; }
  idx[n] = row;
  long double acc = 0.0L, aabs = 0.0L;
  for (int64_t e = 0; e < others; ++e) {
    int64_t off = 0;
    double k = 1.0;
    int first = 1;
    for (int m = 0; m < N; ++m) {
      off += idx[m] * stride[m];
      if (m == n) continue;
      const double u = U[m][idx[m] + dims[m] * col];
      k = first ? u : k * u;
      first = 0;
    }
    const long double term = (long double)T[off] * (long double)k;
    acc += term; aabs += fabsl(term);
    for (int m = 0; m < N; ++m) {
      if (m == n) continue;
      if (++idx[m] < dims[m]) break;
      idx[m] = 0;
    }
  }
  *value = (double)acc;
  *abs_sum = (double)aabs;
}

/* ------------------------------------------------------------------------------------------ */
/* Non-negative least squares on the normal equations, one row (Sec. 5, active-set method)     */
/* ------------------------------------------------------------------------------------------ */

/* Minimise 1/2 x^T H x - m^T x subject to x >= 0.  `passive` is a bit mask of the variables
 * allowed to be non-zero: on entry the warm start (0 = none), on exit the final set.
 * A warm start is a hint: if its sub-block of H cannot be factorised (H may be only semi-definite, e.g. after a
 * component has died) it is dropped and the search restarts from the empty set.
 * Returns 0 on success, 1 if a sub-block reached by the search itself could not be factorised. */
int oracle_nnls_row(const double* H, const double* m, int R, double* x, uint32_t* passive) {
  uint32_t P = *passive & ((R >= 32) ? 0xffffffffu : ((1u << R) - 1u));
  double h1 = 0.0;
  for (int j = 0; j < R; ++j) {
    double cs = 0.0;
    for (int i = 0; i < R; ++i) cs += fabs(H[i + R * j]);
    if (cs > h1) h1 = cs;
  }
  const double tau = 10.0 * DBL_EPSILON * h1 * (double)R;
  const int cap = 30 * R;
  int steps = 0;
  int from_warm = (P != 0);   /* the passive set still derives from the warm start */
  double s[ORACLE_MAX_RANK], Hs[ORACLE_MAX_RANK * ORACLE_MAX_RANK], Ls[ORACLE_MAX_RANK * ORACLE_MAX_RANK];
  int idx[ORACLE_MAX_RANK];
  for (int j = 0; j < R; ++j) x[j] = 0.0;
  for (;;) {
    /* inner loop: make the least-squares solution on the passive set feasible */
    while (P) {
      int np = 0;
      for (int j = 0; j < R; ++j) if (P & (1u << j)) idx[np++] = j;
      for (int a = 0; a < np; ++a) {
        s[a] = m[idx[a]];
        for (int b = 0; b < np; ++b) Hs[a + np * b] = H[idx[a] + R * idx[b]];
      }
      if (oracle_cholesky(Hs, np, Ls)) {
        if (!from_warm) { *passive = P; return 1; }
        P = 0; from_warm = 0;
        for (int j = 0; j < R; ++j) x[j] = 0.0;
        break;
      }
      oracle_cholesky_solve(Ls, np, s);
      int feasible = 1;
      for (int a = 0; a < np; ++a) if (!(s[a] > 0.0)) feasible = 0;
      if (feasible) {
        for (int j = 0; j < R; ++j) x[j] = 0.0;
        for (int a = 0; a < np; ++a) x[idx[a]] = s[a];
        break;
      }
      double beta = 1.0;
      for (int a = 0; a < np; ++a)
        if (!(s[a] > 0.0)) {
          double xa = x[idx[a]];
          double q = xa / (xa - s[a]);
          if (q < beta) beta = q;
        }
      for (int a = 0; a < np; ++a) {
        int j = idx[a];
        /* a variable that bounds the step has reached zero and leaves the passive set, whatever rounding makes
         * of x + beta (s - x) for it (it can come out as a tiny positive number, and the search would stall) */
        const int bounding = !(s[a] > 0.0) && (x[j] / (x[j] - s[a]) == beta);
        x[j] = x[j] + beta * (s[a] - x[j]);
        if (bounding || !(x[j] > 0.0)) { x[j] = 0.0; P &= ~(1u << j); }
      }
      if (++steps > cap) break;
    }
    if (steps > cap) break;
    /* outer step: gradient test, move the most violating variable into the passive set */
    int best = -1;
    double wbest = tau;
    for (int j = 0; j < R; ++j) {
      if (P & (1u << j)) continue;
      double w = m[j];
      for (int k = 0; k < R; ++k) w -= H[j + R * k] * x[k];
      if (w > wbest) { wbest = w; best = j; }
    }
    if (best < 0) break;
    P |= (1u << best);
    from_warm = 0;
    if (++steps > cap) break;
  }
  *passive = P;
  return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* One CP-ALS instance (Alg. 1), advanced one iteration at a time                              */
/* ------------------------------------------------------------------------------------------ */

typedef struct oracle_model {
  int N;                /* number of modes (3 for the routines without the _nd suffix) */
  int64_t I[ORACLE_MAX_MODES];
  int R;
  double* U[ORACLE_MAX_MODES];   /* current factors, column-major I_n x R */
  double* M;                     /* MTTKRP result, max(I_n) x R */
  double* G[ORACLE_MAX_MODES];   /* Gramians of the current factors */
  double lambda[ORACLE_MAX_RANK];
  double fit, fit_prev, err;
  double tol, alpha;
  int max_iters, iters, status;
  uint32_t flags;
  uint32_t* passive[ORACLE_MAX_MODES]; /* NONNEG: per-row passive sets, kept between iterations */
  double* Aprev[ORACLE_MAX_MODES];     /* LINESEARCH: the point after the previous iteration */
  double* Anew[ORACLE_MAX_MODES];
  int ls_accepted;      /* number of accepted extrapolations */
  double ls_err_als, ls_err_new; /* the two errors the last line-search decision compared: after the iteration and
                                    at the extrapolated point (NaN before the first); kept for reporting only */
  double* scratch;
} oracle_model;

oracle_model* oracle_model_create_nd(int N, const int64_t* dims, int R, const double* const* init, double tol,
                                     int max_iters, uint32_t flags, double alpha) {
  if (R < 1 || R > ORACLE_MAX_RANK || N < 3 || N > ORACLE_MAX_MODES) return NULL;
  oracle_model* m = (oracle_model*)calloc(1, sizeof(oracle_model));
  int64_t imax = 0;
  m->N = N;
  m->R = R;
  for (int n = 0; n < N; ++n) {
    m->I[n] = dims[n];
    if (dims[n] > imax) imax = dims[n];
    m->U[n] = (double*)malloc(sizeof(double) * (size_t)(dims[n] * R));
    memcpy(m->U[n], init[n], sizeof(double) * (size_t)(dims[n] * R));
    m->G[n] = (double*)malloc(sizeof(double) * (size_t)(R * R));
    oracle_gram(m->U[n], dims[n], R, m->G[n]);
    if (flags & ORACLE_FLAG_NONNEG) m->passive[n] = (uint32_t*)calloc((size_t)dims[n], sizeof(uint32_t));
    if (flags & ORACLE_FLAG_LINESEARCH) {
      m->Aprev[n] = (double*)malloc(sizeof(double) * (size_t)(dims[n] * R));
      m->Anew[n] = (double*)malloc(sizeof(double) * (size_t)(dims[n] * R));
    }
  }
  m->M = (double*)malloc(sizeof(double) * (size_t)(imax * R));
  m->scratch = (double*)malloc(sizeof(double) * (size_t)(imax * R + R));
  for (int r = 0; r < R; ++r) m->lambda[r] = 1.0;
  m->tol = tol; m->alpha = alpha; m->max_iters = max_iters; m->flags = flags;
  m->fit = 0.0; m->fit_prev = 0.0; m->err = 0.0; m->iters = 0; m->status = ORACLE_RUNNING;
  m->ls_err_als = NAN; m->ls_err_new = NAN;
  return m;
}

oracle_model* oracle_model_create(const int64_t* dims, int R, const double* U1, const double* U2, const double* U3,
                                  double tol, int max_iters, uint32_t flags, double alpha) {
  const double* init[3] = {U1, U2, U3};
  return oracle_model_create_nd(3, dims, R, init, tol, max_iters, flags, alpha);
}

void oracle_model_destroy(oracle_model* m) {
  if (!m) return;
  for (int n = 0; n < m->N; ++n) { free(m->U[n]); free(m->G[n]); free(m->passive[n]); free(m->Aprev[n]); free(m->Anew[n]); }
  free(m->M); free(m->scratch); free(m);
}

/* MTTKRP of one model: order 3 by the nested sums of mttkrp_columns, higher orders by mttkrp_columns_nd. */
static void single_mttkrp(const double* T, const oracle_model* m, int mode, const double* const* U, double* M,
                          double* scratch) {
  if (m->N == 3) mttkrp_columns(T, m->I, mode, U[0], U[1], U[2], 0, m->R, M, scratch);
  else mttkrp_columns_nd(T, m->N, m->I, mode, U, 0, m->R, M);
}

/* H = Hadamard product of the Gramians of all modes but n, multiplied up in increasing mode order
 * (Alg. 1, Hadamard line). */
static void hadamard_of_others(double* const* G, int N, int n, int R, double* H) {
  int first = 1;
  for (int k = 0; k < N; ++k) {
    if (k == n) continue;
    if (first) memcpy(H, G[k], sizeof(double) * (size_t)(R * R));
    else oracle_hadamard(H, G[k], R, H);
    first = 0;
  }
}

/* e = ||T||^2 + normsq - 2 inner  ->  fit (Alg. 1, error line, with the corrected sign). */
static double fit_from_error(double err, double normT2) {
  return 1.0 - sqrt(err > 0.0 ? err : 0.0) / sqrt(normT2);
}

/* Advance one iteration (one update of every mode, then error, fit and the stop test).
 * Returns the status after the iteration (RUNNING means "not stopped"). */
int oracle_model_iterate(oracle_model* m, const double* T, double normT2) {
  if (m->status != ORACLE_RUNNING) return m->status;
  const int R = m->R, N = m->N, last = m->N - 1;
  double H[ORACLE_MAX_RANK * ORACLE_MAX_RANK], L[ORACLE_MAX_RANK * ORACLE_MAX_RANK];
  double Gt[ORACLE_MAX_RANK * ORACLE_MAX_RANK], row[ORACLE_MAX_RANK];
  double inner = 0.0, normsq = 0.0;
  m->iters += 1;
  for (int n = 0; n < N; ++n) {
    const int64_t In = m->I[n];
    single_mttkrp(T, m, n + 1, (const double* const*)m->U, m->M, m->scratch); /* MTTKRP           */
    hadamard_of_others(m->G, N, n, R, H);                                  /* H = * of Gramians */
    if (m->flags & ORACLE_FLAG_NONNEG) {                                   /* update, x >= 0    */
      double* Unew = m->scratch;
      int bad = 0;
      for (int64_t i = 0; i < In && !bad; ++i) {
        double x[ORACLE_MAX_RANK];
        uint32_t P = m->passive[n][i];
        for (int r = 0; r < R; ++r) row[r] = m->M[i + In * r];
        bad = oracle_nnls_row(H, row, R, x, &P);
        if (!bad) { m->passive[n][i] = P; for (int r = 0; r < R; ++r) Unew[i + In * r] = x[r]; }
      }
      if (bad) { m->status = ORACLE_NUMERICAL; m->iters -= 1; return m->status; }
      memcpy(m->U[n], Unew, sizeof(double) * (size_t)(In * R));
    } else if (!oracle_cholesky_definite(H, R, L)) {                       /* update, U = M H^-1 */
      for (int64_t i = 0; i < In; ++i) {
        for (int r = 0; r < R; ++r) row[r] = m->M[i + In * r];
        oracle_cholesky_solve(L, R, row);
        for (int r = 0; r < R; ++r) m->U[n][i + In * r] = row[r];
      }
    } else {                                                               /* rank-deficient: U = M H^+ */
      double* P = L;
      if (oracle_pinv_sym(H, R, P, NULL)) { m->status = ORACLE_NUMERICAL; m->iters -= 1; return m->status; }
      for (int64_t i = 0; i < In; ++i) {
        for (int r = 0; r < R; ++r) row[r] = m->M[i + In * r];
        for (int c = 0; c < R; ++c) {
          double v = 0.0;
          for (int k = 0; k < R; ++k) v += row[k] * P[k + R * c];
          m->U[n][i + In * c] = v;
        }
      }
    }
    if (n == last) {                                                       /* error terms        */
      for (int r = 0; r < R; ++r) {
        double col = 0.0;
        for (int64_t i = 0; i < In; ++i) col += m->U[last][i + In * r] * m->M[i + In * r];
        inner += col;
      }
      oracle_gram(m->U[last], In, R, Gt);
      for (int e = 0; e < R * R; ++e) normsq += H[e] * Gt[e];
    }
    for (int r = 0; r < R; ++r) {                                          /* unit columns       */
      double ss = 0.0;
      double* c = m->U[n] + In * r;
      for (int64_t i = 0; i < In; ++i) ss += c[i] * c[i];
      const double nrm = sqrt(ss);
      m->lambda[r] = nrm;
      if (nrm > 0.0) for (int64_t i = 0; i < In; ++i) c[i] = c[i] / nrm;
    }
    oracle_gram(m->U[n], In, R, m->G[n]);
  }
  m->err = normT2 + normsq - 2.0 * inner;
  m->fit = fit_from_error(m->err, normT2);

  if (m->flags & ORACLE_FLAG_LINESEARCH) {
    /* Sec. 5, line search: P_new = P_prev + alpha (P_cur - P_prev), kept only if its error is
     * lower.  A point is represented with lambda folded into the factor of the last mode. */
    const int64_t IN = m->I[last];
    if (m->iters >= 2) {
      for (int n = 0; n < N; ++n) {
        const int64_t In = m->I[n];
        for (int r = 0; r < R; ++r) {
          const double scale = (n == last) ? m->lambda[r] : 1.0;
          for (int64_t i = 0; i < In; ++i) {
            const double cur = m->U[n][i + In * r] * scale;
            const double prev = m->Aprev[n][i + In * r];
            double v = prev + m->alpha * (cur - prev);
            /* NONNEG models: the extrapolated point is projected back onto the feasible set */
            if ((m->flags & ORACLE_FLAG_NONNEG) && !(v > 0.0)) v = 0.0;
            m->Anew[n][i + In * r] = v;
          }
        }
      }
      single_mttkrp(T, m, N, (const double* const*)m->Anew, m->M, m->scratch);
      double inner2 = 0.0, normsq2 = 0.0;
      for (int r = 0; r < R; ++r) {
        double col = 0.0;
        for (int64_t i = 0; i < IN; ++i) col += m->Anew[last][i + IN * r] * m->M[i + IN * r];
        inner2 += col;
      }
      double Gn[ORACLE_MAX_MODES][ORACLE_MAX_RANK * ORACLE_MAX_RANK];
      for (int n = 0; n < N; ++n) oracle_gram(m->Anew[n], m->I[n], R, Gn[n]);
      for (int e = 0; e < R * R; ++e) {
        double h = Gn[0][e];
        for (int n = 1; n < N; ++n) h = h * Gn[n][e];
        normsq2 += h;
      }
      const double err2 = normT2 + normsq2 - 2.0 * inner2;
      m->ls_err_als = m->err; m->ls_err_new = err2;
      if (err2 < m->err) {
        for (int n = 0; n < N; ++n) {
          memcpy(m->U[n], m->Anew[n], sizeof(double) * (size_t)(m->I[n] * R));
          memcpy(m->G[n], Gn[n], sizeof(double) * (size_t)(R * R));
        }
        for (int r = 0; r < R; ++r) m->lambda[r] = 1.0;
        m->err = err2;
        m->fit = fit_from_error(err2, normT2);
        m->ls_accepted += 1;
      }
    }
    for (int n = 0; n < N; ++n) {
      const int64_t In = m->I[n];
      for (int r = 0; r < R; ++r) {
        const double scale = (n == last) ? m->lambda[r] : 1.0;
        for (int64_t i = 0; i < In; ++i) m->Aprev[n][i + In * r] = m->U[n][i + In * r] * scale;
      }
    }
  }

  if (m->iters >= 2 && fabs(m->fit - m->fit_prev) < m->tol) m->status = ORACLE_CONVERGED;
  else if (m->iters >= m->max_iters) m->status = ORACLE_MAX_ITERS;
  m->fit_prev = m->fit;
  return m->status;
}

/* out[n] (n < N; entries may be NULL) receive the factors. */
void oracle_model_get_nd(const oracle_model* m, double* const* out, double* lambda, double* fit, double* err,
                         int* iters, int* status, int* ls_accepted) {
  if (out)
    for (int n = 0; n < m->N; ++n)
      if (out[n]) memcpy(out[n], m->U[n], sizeof(double) * (size_t)(m->I[n] * m->R));
  if (lambda) memcpy(lambda, m->lambda, sizeof(double) * (size_t)m->R);
  if (fit) *fit = m->fit;
  if (err) *err = m->err;
  if (iters) *iters = m->iters;
  if (status) *status = m->status;
  if (ls_accepted) *ls_accepted = m->ls_accepted;
}

/* Reporting only: the two errors that the last line-search decision compared (NaN if there was none yet), so
 * that a caller can tell how close that decision was. */
void oracle_model_last_ls_errors(const oracle_model* m, double* err_als, double* err_new) {
  *err_als = m->ls_err_als;
  *err_new = m->ls_err_new;
}

void oracle_model_get(const oracle_model* m, double* U1, double* U2, double* U3, double* lambda, double* fit,
                      double* err, int* iters, int* status, int* ls_accepted) {
  double* out[3] = {U1, U2, U3};
  oracle_model_get_nd(m, out, lambda, fit, err, iters, status, ls_accepted);
}

/* Plain CP-ALS (Alg. 1) for one starting point: iterate until it stops.  fit_history, when
 * given, receives the fit after every iteration (max_iters entries). */
int oracle_cp_als(const double* T, const int64_t* dims, double normT2, int R, double* U1, double* U2, double* U3,
                  double* lambda, double tol, int max_iters, uint32_t flags, double alpha, double* fit, double* err,
                  int* iters, int* status, double* fit_history) {
  oracle_model* m = oracle_model_create(dims, R, U1, U2, U3, tol, max_iters, flags, alpha);
  if (!m) return -1;
  while (m->status == ORACLE_RUNNING) {
    oracle_model_iterate(m, T, normT2);
    if (fit_history && m->status != ORACLE_NUMERICAL) fit_history[m->iters - 1] = m->fit;
  }
  oracle_model_get(m, U1, U2, U3, lambda, fit, err, iters, status, NULL);
  oracle_model_destroy(m);
  return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* CALS, full algorithm (Alg. 3): queue in, lock-step iterations, queue out                    */
/* ------------------------------------------------------------------------------------------ */

/* Models are queued in index order 0..n_models-1.  inits[N*k + n] is model k's mode-(n+1)
 * starting factor; outs[N*k + n] receives its final factor (may be NULL).  A model fits if
 * the sum of active ranks plus its rank is at most max_total_rank and (max_slots == 0 or)
 * fewer than max_slots models are active.  retire_order receives the model indices in the
 * order they leave; total_rank_log (optional, one entry per round up to max_rounds) the
 * fused width of each round.  Returns the number of rounds, or -1 on a bad argument
 * (including a model that can never fit, which would block the queue for ever). */
int64_t oracle_cals_nd(const double* T, int N, const int64_t* dims, int n_models, const int32_t* ranks,
                       const double* const* inits, const double* tol, const int32_t* max_iters,
                       const uint32_t* flags, const double* alpha, int64_t max_total_rank, int max_slots,
                       double* const* outs, double* lambdas /* n_models x ORACLE_MAX_RANK */, double* fit, double* err,
                       int32_t* iters, int32_t* status, int32_t* retire_order, int32_t* total_rank_log,
                       int64_t max_rounds) {
  if (N < 3 || N > ORACLE_MAX_MODES) return -1;
  for (int k = 0; k < n_models; ++k)
    if (ranks[k] < 1 || ranks[k] > ORACLE_MAX_RANK || ranks[k] > max_total_rank) return -1;
  const double normT2 = (N == 3) ? oracle_norm_sq(T, dims) : oracle_norm_sq_nd(T, N, dims);
  oracle_model** slot = (oracle_model**)calloc((size_t)(n_models > 0 ? n_models : 1), sizeof(oracle_model*));
  int* slot_id = (int*)calloc((size_t)(n_models > 0 ? n_models : 1), sizeof(int));
  int n_active = 0, next = 0, n_retired = 0;
  int64_t rtot = 0, rounds = 0;
  while (next < n_models || n_active > 0) {
    /* fill the multi-matrices from the queue front; stop at the first model that does not fit */
    while (next < n_models) {
      const int r = ranks[next];
      if (rtot + r > max_total_rank || (max_slots > 0 && n_active >= max_slots)) break;
      slot[n_active] = oracle_model_create_nd(N, dims, r, inits + (size_t)N * next, tol[next], max_iters[next],
                                              flags[next], alpha[next]);
      slot_id[n_active] = next;
      n_active += 1; rtot += r; next += 1;
    }
    if (total_rank_log && rounds < max_rounds) total_rank_log[rounds] = (int32_t)rtot;
    /* advance all active instances one iteration (they are independent: Eq. (2)) */
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < n_active; ++s) oracle_model_iterate(slot[s], T, normT2);
    /* retire in slot order, survivors keep their order */
    int w = 0;
    for (int s = 0; s < n_active; ++s) {
      oracle_model* m = slot[s];
      const int k = slot_id[s];
      if (m->status != ORACLE_RUNNING) {
        oracle_model_get_nd(m, outs ? outs + (size_t)N * k : NULL,
                            lambdas ? lambdas + (size_t)k * ORACLE_MAX_RANK : NULL, fit ? fit + k : NULL,
                            err ? err + k : NULL, iters ? iters + k : NULL, status ? status + k : NULL, NULL);
        retire_order[n_retired++] = k;
        rtot -= m->R;
        oracle_model_destroy(m);
      } else {
        slot[w] = m; slot_id[w] = k; ++w;
      }
    }
    n_active = w;
    rounds += 1;
  }
  free(slot); free(slot_id);
  return rounds;
}

int64_t oracle_cals(const double* T, const int64_t* dims, int n_models, const int32_t* ranks,
                    const double* const* inits, const double* tol, const int32_t* max_iters,
                    const uint32_t* flags, const double* alpha, int64_t max_total_rank, int max_slots,
                    double* const* outs, double* lambdas /* n_models x ORACLE_MAX_RANK */, double* fit, double* err,
                    int32_t* iters, int32_t* status, int32_t* retire_order, int32_t* total_rank_log,
                    int64_t max_rounds) {
  return oracle_cals_nd(T, 3, dims, n_models, ranks, inits, tol, max_iters, flags, alpha, max_total_rank, max_slots,
                        outs, lambdas, fit, err, iters, status, retire_order, total_rank_log, max_rounds);
}
