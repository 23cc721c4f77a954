// Per-model steps of one CALS mode update (Alg. 2 inner loop; Alg. 1 Hadamard, update and error lines),
// one workgroup per active model (modes of more than 256 rows: one per model and row block, two launches):
//   H = product of the cached Gramians of all other modes        -- Hadamard product of Gramians
//   H = L L^T                                                    -- Cholesky, no pivoting
//   U[i,:] = M[i,:] H^-1 for every row i (two triangular solves) -- normal-equation update
//   (H numerically rank-deficient: U[i,:] = M[i,:] H^+ with H^+ from a Jacobi eigen-decomposition)
//   last mode only: inner = sum(U * M), normsq = sum(H * U^T U)  -- terms of the fast error formula
//   lambda_r = ||U[:,r]||_2, U[:,r] /= lambda_r, G = U^T U       -- unit columns, Gramian refresh
// plus the small utility kernels around it (initial Gramians, ||T||^2, column gather).
#include "cals_internal.h"

namespace cals {

constexpr int kRows = 256;             // rows staged per pass (= workgroup size)
constexpr int kXs = kRows + 1;         // padded stride of the staged block (conflict-free pair reads)

__device__ inline double block_sum(double v, double* red /* 256 doubles in LDS */) {
  const int tid = threadIdx.x;
  red[tid] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  const double r = red[0];
  __syncthreads();
  return r;
}

__device__ inline void pair_rs(int p, int& r, int& s) {   // p -> (r, s), r >= s, row-major lower triangle
  r = (int)((sqrt(8.0 * p + 1.0) - 1.0) * 0.5);
  while (r * (r + 1) / 2 > p) --r;
  while ((r + 1) * (r + 2) / 2 <= p) ++r;
  s = p - r * (r + 1) / 2;
}

// Accumulates the lower triangle of X^T X over the `nrows` staged rows.  Pair p (< R(R+1)/2 <= 528) is
// owned by thread p % 256, slot p / 256.  xs[r * kXs + j] holds X[row j][r].
__device__ inline void gram_accumulate(const double* xs, int R, int nrows, double (&gacc)[3]) {
  const int npairs = R * (R + 1) / 2;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const int p = threadIdx.x + 256 * q;
    if (p < npairs) {
      int r, s;
      pair_rs(p, r, s);
      const double* xr = xs + r * kXs;
      const double* xc = xs + s * kXs;
      double acc = gacc[q];
      for (int j = 0; j < nrows; ++j) acc += xr[j] * xc[j];
      gacc[q] = acc;
    }
  }
}

__device__ inline void gram_store(const double (&gacc)[3], int R, double* Gl /* LDS, R x R */) {
  const int npairs = R * (R + 1) / 2;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const int p = threadIdx.x + 256 * q;
    if (p < npairs) {
      int r, s;
      pair_rs(p, r, s);
      Gl[r * R + s] = gacc[q];
      Gl[s * R + r] = gacc[q];
    }
  }
}

// A pivot, or an eigenvalue, counts as zero below this fraction of the diagonal entry it started from, or of the
// largest eigenvalue: the normal equations are then rank-deficient and the update goes through the pseudo-inverse
// (Alg. 1 writes the update with the pseudo-inverse of H).
constexpr double kRankTol = 1e-12;

// In-place lower Cholesky of the R x R matrix A (LDS, row-major, ld = R; H0 = the untouched original).  The
// updates reach every element in the same order as the textbook column algorithm (k = 0,1,...).  Returns false
// (to all threads) when a pivot is not finite or not above kRankTol times its original diagonal entry.
__device__ inline bool block_cholesky(double* A, const double* H0, int R, int* flag /* LDS */) {
  const int tid = threadIdx.x;
  if (tid == 0) *flag = 1;
  __syncthreads();
  for (int j = 0; j < R; ++j) {
    if (tid == 0) {
      const double d = A[j * R + j];
      if (!(d > kRankTol * H0[j * R + j]) || !isfinite(d)) *flag = 0;
      else A[j * R + j] = sqrt(d);
    }
    __syncthreads();
    if (*flag == 0) return false;
    const double djj = A[j * R + j];
    for (int i = j + 1 + tid; i < R; i += 256) A[i * R + j] = A[i * R + j] / djj;
    __syncthreads();
    const int n = R - j - 1;                  // trailing block, lower triangle only
    for (int e = tid; e < n * n; e += 256) {
      const int i = j + 1 + e / n, c = j + 1 + e % n;
      if (c <= i) A[i * R + c] -= A[i * R + j] * A[c * R + j];
    }
    __syncthreads();
  }
  return true;
}

// Pseudo-inverse of the symmetric positive semi-definite R x R matrix H (LDS) by a two-sided Jacobi
// eigen-decomposition, all 256 threads of the workgroup: P = sum over eigenpairs with l_i > kRankTol * l_max of
// v_i v_i^T / l_i.  Rotations of one step act on disjoint index pairs (round-robin tournament over the indices), so
// a step is: angles from the 2 x 2 blocks, all column rotations (A and V), all row rotations (A).
// A (R*R; may be H itself), V (R*R), P (R*R), cs (>= 64 doubles; may be red), red (256 doubles) are LDS work areas.
// Returns false (to all threads) when H has a non-finite entry or no positive eigenvalue.
__device__ inline bool block_pinv(const double* H, int R, double* A, double* V, double* P, double* cs, double* red,
                                  int* flag /* LDS */) {
  const int tid = threadIdx.x;
  if (tid == 0) *flag = 1;
  __syncthreads();
  for (int e = tid; e < R * R; e += 256) {
    const double h = H[e];
    if (!isfinite(h)) *flag = 0;
    A[e] = h;
    V[e] = (e / R == e % R) ? 1.0 : 0.0;
  }
  __syncthreads();
  if (*flag == 0) return false;
  const int Re = (R + 1) & ~1;                 // even number of players; index R (when R is odd) sits out
  const int half = Re / 2;
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0.0, all = 0.0;
    for (int e = tid; e < R * R; e += 256) {
      const double v = A[e] * A[e];
      all += v;
      if (e / R != e % R) off += v;
    }
    off = block_sum(off, red);
    all = block_sum(all, red);
    if (!(off > 1e-34 * all)) break;
    for (int step = 0; step < Re - 1; ++step) {
      if (tid < half) {
        // circle method: player Re-1 stays, the others rotate
        int p = (tid == 0) ? Re - 1 : (step + tid) % (Re - 1);
        int q = (tid == 0) ? step : (step - tid + (Re - 1)) % (Re - 1);
        if (p > q) { const int t = p; p = q; q = t; }
        double c = 1.0, sn = 0.0;
        if (q < R) {
          const double apq = A[p * R + q];
          if (apq != 0.0) {
            const double tau = (A[q * R + q] - A[p * R + p]) / (2.0 * apq);
            const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
            c = 1.0 / sqrt(1.0 + t * t);
            sn = t * c;
          }
        } else {
          q = p;                                // sits out: identity on a valid index
        }
        cs[4 * tid + 0] = c;
        cs[4 * tid + 1] = sn;
        cs[4 * tid + 2] = (double)p;
        cs[4 * tid + 3] = (double)q;
      }
      __syncthreads();
      for (int w = tid; w < half * R; w += 256) {          // columns p, q of A and of V
        const int i = w / R, k = w % R;
        const double c = cs[4 * i], sn = cs[4 * i + 1];
        const int p = (int)cs[4 * i + 2], q = (int)cs[4 * i + 3];
        if (p != q) {
          const double akp = A[k * R + p], akq = A[k * R + q];
          A[k * R + p] = c * akp - sn * akq;
          A[k * R + q] = sn * akp + c * akq;
          const double vkp = V[k * R + p], vkq = V[k * R + q];
          V[k * R + p] = c * vkp - sn * vkq;
          V[k * R + q] = sn * vkp + c * vkq;
        }
      }
      __syncthreads();
      for (int w = tid; w < half * R; w += 256) {          // rows p, q of A
        const int i = w / R, k = w % R;
        const double c = cs[4 * i], sn = cs[4 * i + 1];
        const int p = (int)cs[4 * i + 2], q = (int)cs[4 * i + 3];
        if (p != q) {
          const double apk = A[p * R + k], aqk = A[q * R + k];
          A[p * R + k] = c * apk - sn * aqk;
          A[q * R + k] = sn * apk + c * aqk;
        }
      }
      __syncthreads();
    }
  }
  if (tid == 0) {
    double lmax = 0.0;
    for (int i = 0; i < R; ++i) lmax = A[i * R + i] > lmax ? A[i * R + i] : lmax;
    red[0] = lmax;
    if (!(lmax > 0.0)) *flag = 0;
  }
  __syncthreads();
  const double cut = kRankTol * red[0];
  const bool ok = *flag != 0;
  for (int e = tid; e < R * R; e += 256) {
    const int r = e / R, c = e % R;
    double acc = 0.0;
    for (int i = 0; i < R; ++i) {
      const double l = A[i * R + i];
      if (l > cut) acc += V[r * R + i] * V[c * R + i] / l;
    }
    P[e] = acc;
  }
  __syncthreads();
  return ok;
}

// ---- modes of at most 256 rows: one workgroup per model, one row per thread, everything in one pass ----------
// The two latency chains of the update are kept out of LDS: the Cholesky factorisation runs in ONE wavefront with
// row i of the working matrix in lane i's registers (pivot column broadcast through v_readlane; right-looking, so
// every element sees its subtractions in the order of the textbook column algorithm), and a thread solves its row
// with the right-hand side in registers (the factor is read from LDS at wave-uniform addresses, which do not depend
// on the data: the dependent chain is the FMA latency only).  RM = rank rounded up to a multiple of 4; the factor
// is stored RM x RM with zero padding and unit diagonal beyond the rank, so the unrolled loops need no guards.
template <int RM>
__device__ __forceinline__ bool wave_cholesky(const double* H, double* L, int R, int lane) {
  double arow[RM];
#pragma unroll
  for (int k = 0; k < RM; ++k) arow[k] = (lane < R && k < R) ? H[lane * R + k] : 0.0;
  const double diag0 = (lane < R) ? H[lane * R + lane] : 1.0;
  bool ok = true;
#pragma unroll
  for (int j = 0; j < RM; ++j) {
    if (ok && j < R) {
      const double djj = readlane_f64(arow[j], j);
      if (!(djj > kRankTol * readlane_f64(diag0, j)) || !isfinite(djj)) {
        ok = false;
      } else {
        const double ljj = sqrt(djj);
        const double lcol = (lane > j) ? arow[j] / ljj : (lane == j ? ljj : 0.0);
        if (lane >= j && lane < R) L[lane * RM + j] = lcol;
#pragma unroll
        for (int k = j + 1; k < RM; ++k) arow[k] = fma(-lcol, readlane_f64(lcol, k), arow[k]);
      }
    }
  }
  return ok;
}

__device__ inline double fast_block_sum(double v, double* red /* >= 4 doubles in LDS */) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// Solves (L L^T) x = m for one row with x in registers; L is RM x RM in LDS, zero padded with unit diagonal.
template <int RM>
__device__ __forceinline__ void solve_row_in_registers(const double* L, double (&x)[RM]) {
#pragma unroll
  for (int r = 0; r < RM; ++r) {              // L y = m
    double v = x[r];
#pragma unroll
    for (int k = 0; k < r; ++k) v = fma(-L[r * RM + k], x[k], v);
    x[r] = v / L[r * RM + r];
    __builtin_amdgcn_sched_barrier(0);        // keeps the factor reads of later rows from being hoisted (registers)
  }
#pragma unroll
  for (int r = RM - 1; r >= 0; --r) {         // L^T x = y
    double v = x[r];
#pragma unroll
    for (int k = r + 1; k < RM; ++k) v = fma(-L[k * RM + r], x[k], v);
    x[r] = v / L[r * RM + r];
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Tall modes, ranks up to 16: the rows [r0, r1) of one model, 256 at a time -- solve in registers, store the
// (not yet normalised) rows, stage them for the Gramian, accumulate Gramian and inner product.
template <int RM>
__device__ __forceinline__ void solve_rows_small(const UpdateArgs& a, const ModelDesc& d, const double* L, double* xs,
                                                 bool nonneg, int r0, int r1, double (&gacc)[3], double& inner) {
  const int tid = threadIdx.x, R = d.rank;
  for (int base = r0; base < r1; base += kRows) {
    const int i = base + tid;
    const int nrows = (r1 - base < kRows) ? (r1 - base) : kRows;
    if (i < r1) {
      const double* mrow = a.M + (int64_t)i * a.ld + d.col;
      const double* src = nonneg ? a.X + (int64_t)i * a.ld + d.col : mrow;
      double x[RM];
#pragma unroll
      for (int r = 0; r < RM; ++r) x[r] = (r < R) ? src[r] : 0.0;
      if (!nonneg) solve_row_in_registers<RM>(L, x);
      double* urow = a.U + (int64_t)i * a.ld + d.col;
#pragma unroll
      for (int r = 0; r < RM; ++r)
        if (r < R) {
          xs[r * kXs + tid] = x[r];
          urow[r] = x[r];
          inner = fma(x[r], mrow[r], inner);
        }
    }
    __syncthreads();
    gram_accumulate(xs, R, nrows, gacc);
    __syncthreads();
  }
}

// x = m P for this thread's row (P symmetric R x R in LDS): x is built in the output row (scratch use of memory the
// caller overwrites anyway) and then staged in xs[. * kXs + tid] like every other solved row.
__device__ inline void row_times_matrix(const double* P, int R, const double* mrow, double* urow, double* xs) {
  const int tid = threadIdx.x;
  for (int r = 0; r < R; ++r) xs[r * kXs + tid] = mrow[r];
  for (int c = 0; c < R; ++c) {
    double v = 0.0;
    for (int k = 0; k < R; ++k) v += xs[k * kXs + tid] * P[k * R + c];
    urow[c] = v;
  }
  for (int r = 0; r < R; ++r) xs[r * kXs + tid] = urow[r];
}

__device__ __noinline__ void update_wide(const UpdateArgs& a, const ModelDesc& d, double* lds, int* flagp);

template <int RM>
__device__ __forceinline__ void update_small(const UpdateArgs& a, const ModelDesc& d, int slot, double* lds, int* flag) {
  ModelState* st = a.state + d.sid;
  ModelOut* out = a.out + d.sid;
  const int tid = threadIdx.x;
  const int R = d.rank;
  double* xs = lds;                           // R * kXs: the solved rows, staged for the Gramian
  double* H = xs + kMaxRank * kXs;            // R*R, Hadamard of Gramians
  double* L = H + kGramStride;                // RM*RM, Cholesky factor (zero padded, unit diagonal beyond R)
  double* Gl = L + kGramStride;               // R*R, Gramian of the updated factor
  double* red = Gl + kGramStride;             // 256
  double* lam = red + 256;                    // R

  for (int e = tid; e < R * R; e += 256) H[e] = hadamard_of_others(st, a.nmodes, a.mode, e);
  for (int e = tid; e < RM * RM; e += 256) L[e] = (e / RM == e % RM && e / RM >= R) ? 1.0 : 0.0;
  __syncthreads();
  // NONNEG models: the rows were solved by the non-negative update already (a.X); only its outcome is read
  const bool nonneg = (d.flags & 1u) != 0;
  if (nonneg) {
    if (tid == 0) {
      *flag = a.nn_fail[slot] == 0;
      a.nn_fail[slot] = 0;
    }
  } else if (tid < 64) {
    const bool ok = wave_cholesky<RM>(H, L, R, tid);
    if (tid == 0) *flag = ok;
  }
  __syncthreads();
  if (*flag == 0) {
    if (nonneg) {
      if (tid == 0) out->status = 3;          // CALS_NUMERICAL; factors of this mode stay untouched
    } else {
      __syncthreads();
      update_wide(a, d, lds, flag);           // rank-deficient normal equations: the general path applies H^+
    }
    return;
  }

  const int i = tid;
  const bool live = i < a.In;
  double x[RM];
  double inner = 0.0;
  if (live) {
    const double* mrow = a.M + (int64_t)i * a.ld + d.col;
    if (nonneg) {
      const double* xrow = a.X + (int64_t)i * a.ld + d.col;
#pragma unroll
      for (int r = 0; r < RM; ++r) x[r] = (r < R) ? xrow[r] : 0.0;
    } else {
#pragma unroll
      for (int r = 0; r < RM; ++r) x[r] = (r < R) ? mrow[r] : 0.0;
      solve_row_in_registers<RM>(L, x);
    }
#pragma unroll
    for (int r = 0; r < RM; ++r)
      if (r < R) {
        xs[r * kXs + tid] = x[r];
        inner = fma(x[r], mrow[r], inner);
      }
  }
  __syncthreads();
  double gacc[3] = {0.0, 0.0, 0.0};
  gram_accumulate(xs, R, a.In, gacc);
  gram_store(gacc, R, Gl);
  __syncthreads();

  if (a.mode == a.nmodes - 1) {
    double part = 0.0;
    for (int e = tid; e < R * R; e += 256) part += H[e] * Gl[e];
    const double normsq = fast_block_sum(part, red);
    const double in = fast_block_sum(inner, red);
    if (tid == 0) {
      st->inner = in;
      st->normsq = normsq;
      const double err = a.normT2 + normsq - 2.0 * in;
      out->err = err;
      out->fit = 1.0 - sqrt(err > 0.0 ? err : 0.0) / sqrt(a.normT2);
      out->iters += 1;
    }
  }
  if (tid < R) {
    const double l = sqrt(Gl[tid * R + tid]);
    lam[tid] = l;
    a.lambda[d.sid * kMaxRank + tid] = l;
  }
  __syncthreads();
  for (int e = tid; e < R * R; e += 256) {
    const int r = e / R, s = e % R;
    const double lr = lam[r] > 0.0 ? lam[r] : 1.0, ls = lam[s] > 0.0 ? lam[s] : 1.0;
    st->G[a.mode][e] = (Gl[e] / lr) / ls;
  }
  if (live) {
    double* urow = a.U + (int64_t)i * a.ld + d.col;
#pragma unroll
    for (int r = 0; r < RM; ++r)
      if (r < R) {
        const double l = lam[r];
        urow[r] = l > 0.0 ? x[r] / l : x[r];
      }
  }
}

// Ranks above 20: the same steps with the factor and the row vectors in LDS (the register arrays of the path above
// would not fit next to each other for every rank in one kernel).
__device__ __noinline__ void update_wide(const UpdateArgs& a, const ModelDesc& d, double* lds, int* flagp) {
  ModelState* st = a.state + d.sid;
  ModelOut* out = a.out + d.sid;
  const int tid = threadIdx.x;
  const int R = d.rank;
  double* xs = lds;                           // R * kXs
  double* H = xs + kMaxRank * kXs;            // R*R, Hadamard of Gramians
  double* L = H + kGramStride;                // R*R, Cholesky factor
  double* Gl = L + kGramStride;               // R*R, Gramian of the updated factor
  double* red = Gl + kGramStride;             // 256
  double* lam = red + 256;                    // R
  int& flag = *flagp;

  for (int e = tid; e < R * R; e += 256) {
    const double h = hadamard_of_others(st, a.nmodes, a.mode, e);
    H[e] = h;
    L[e] = h;
  }
  __syncthreads();
  // NONNEG models: the rows were solved by the non-negative update already (a.X); only its outcome is read
  const bool nonneg = (d.flags & 1u) != 0;
  bool pinv = false;
  if (nonneg) {
    if (tid == 0) {
      flag = a.nn_fail[blockIdx.x];
      a.nn_fail[blockIdx.x] = 0;
    }
    __syncthreads();
    if (flag != 0) {
      if (tid == 0) out->status = 3;
      return;
    }
  } else if (!block_cholesky(L, H, R, &flag)) {
    // rank-deficient: P = H^+ takes the factor's place (work areas: Gl and the row staging block, both free now)
    if (!block_pinv(H, R, Gl, xs, L, red, red, &flag)) {
      if (tid == 0) out->status = 3;          // CALS_NUMERICAL; factors of this mode stay untouched
      return;
    }
    pinv = true;
  }

  double gacc[3] = {0.0, 0.0, 0.0};
  double inner = 0.0;
  const double* Mb = a.M + d.col;
  double* Ub = a.U + d.col;
  for (int base = 0; base < a.In; base += kRows) {
    const int i = base + tid;
    const int nrows = (a.In - base < kRows) ? (a.In - base) : kRows;
    if (i < a.In) {
      const double* mrow = Mb + (int64_t)i * a.ld;
      double* urow = Ub + (int64_t)i * a.ld;
      if (nonneg) {
        const double* xrow = a.X + (int64_t)i * a.ld + d.col;
        for (int r = 0; r < R; ++r) xs[r * kXs + tid] = xrow[r];
      } else if (pinv) {
        row_times_matrix(L, R, mrow, urow, xs);
      } else {
        for (int r = 0; r < R; ++r) xs[r * kXs + tid] = mrow[r];
        // L y = m
        for (int r = 0; r < R; ++r) {
          double v = xs[r * kXs + tid];
          for (int k = 0; k < r; ++k) v -= L[r * R + k] * xs[k * kXs + tid];
          xs[r * kXs + tid] = v / L[r * R + r];
        }
        // L^T x = y
        for (int r = R - 1; r >= 0; --r) {
          double v = xs[r * kXs + tid];
          for (int k = r + 1; k < R; ++k) v -= L[k * R + r] * xs[k * kXs + tid];
          xs[r * kXs + tid] = v / L[r * R + r];
        }
      }
      double part = 0.0;
      for (int r = 0; r < R; ++r) {
        const double x = xs[r * kXs + tid];
        urow[r] = x;
        part += x * mrow[r];
      }
      inner += part;
    }
    __syncthreads();
    gram_accumulate(xs, R, nrows, gacc);
    __syncthreads();
  }
  gram_store(gacc, R, Gl);
  __syncthreads();

  if (a.mode == a.nmodes - 1) {
    double part = 0.0;
    for (int e = tid; e < R * R; e += 256) part += H[e] * Gl[e];
    const double normsq = block_sum(part, red);
    const double in = block_sum(inner, red);
    if (tid == 0) {
      st->inner = in;
      st->normsq = normsq;
      const double err = a.normT2 + normsq - 2.0 * in;
      out->err = err;
      out->fit = 1.0 - sqrt(err > 0.0 ? err : 0.0) / sqrt(a.normT2);
      out->iters += 1;
    }
  }
  if (tid < R) {
    const double l = sqrt(Gl[tid * R + tid]);
    lam[tid] = l;
    a.lambda[d.sid * kMaxRank + tid] = l;
  }
  __syncthreads();
  for (int e = tid; e < R * R; e += 256) {
    const int r = e / R, s = e % R;
    const double lr = lam[r] > 0.0 ? lam[r] : 1.0, ls = lam[s] > 0.0 ? lam[s] : 1.0;
    st->G[a.mode][e] = (Gl[e] / lr) / ls;
  }
  for (int i = tid; i < a.In; i += 256) {
    double* urow = Ub + (int64_t)i * a.ld;
    for (int r = 0; r < R; ++r) {
      const double l = lam[r];
      if (l > 0.0) urow[r] = urow[r] / l;
    }
  }
}

__global__ void __launch_bounds__(256) update_kernel(UpdateArgs a) {
  extern __shared__ double lds[];
  __shared__ int flag;
  const ModelDesc d = a.desc[blockIdx.x];
  if (a.out[d.sid].status != 0) return;       // stopped earlier in this iteration (uniform)
  switch ((d.rank + 3) / 4) {
    case 1: update_small<4>(a, d, blockIdx.x, lds, &flag); break;
    case 2: update_small<8>(a, d, blockIdx.x, lds, &flag); break;
    case 3: update_small<12>(a, d, blockIdx.x, lds, &flag); break;
    case 4: update_small<16>(a, d, blockIdx.x, lds, &flag); break;
    case 5: update_small<20>(a, d, blockIdx.x, lds, &flag); break;
    default: update_wide(a, d, lds, &flag); break;
  }
}

// ---- tall modes: the same update cut into row blocks, two launches -------------------------------------
// update_solve_kernel, grid (models, row blocks): every workgroup factorises H itself (identical results),
// solves its rows and leaves its partial Gramian and inner product in a.part.  update_finish_kernel, same
// grid: every workgroup adds the partials in block order (fixed order: reproducible), derives lambda and
// scales its rows; row block 0 also writes the model's Gramian, lambda and error terms.
__device__ inline int rows_per_block(int In, int nblk) { return ((In + nblk - 1) / nblk + kRows - 1) / kRows * kRows; }

__global__ void __launch_bounds__(256) update_solve_kernel(UpdateArgs a) {
  extern __shared__ double lds[];
  const ModelDesc d = a.desc[blockIdx.x];
  const ModelState* st = a.state + d.sid;
  ModelOut* out = a.out + d.sid;
  if (out->status != 0) return;               // stopped earlier in this iteration (uniform over the model's blocks:
                                              // this launch only ever stores the value every block computes alike)
  const int tid = threadIdx.x;
  const int R = d.rank;
  double* xs = lds;                           // R * kXs
  double* L = xs + kMaxRank * kXs;            // Cholesky factor: R*R in place of H, or RM*RM padded (ranks <= 16)
  double* red = L + kGramStride;              // 256
  double* H = red + 256;                      // R*R (ranks <= 16: the factorisation reads H and writes L)
  __shared__ int flag;
  const bool small = R <= 16;
  const int RMs = (R + 3) / 4 * 4;

  if (small) {
    for (int e = tid; e < R * R; e += 256) H[e] = hadamard_of_others(st, a.nmodes, a.mode, e);
    for (int e = tid; e < RMs * RMs; e += 256) L[e] = (e / RMs == e % RMs && e / RMs >= R) ? 1.0 : 0.0;
  } else {
    for (int e = tid; e < R * R; e += 256) {
      const double h = hadamard_of_others(st, a.nmodes, a.mode, e);
      H[e] = h;
      L[e] = h;
    }
  }
  __syncthreads();
  const bool nonneg = (d.flags & 1u) != 0;
  bool pinv = false;
  bool failed;
  if (nonneg) {
    if (tid == 0) flag = a.nn_fail[blockIdx.x];   // cleared by update_finish_kernel
    __syncthreads();
    failed = flag != 0;
  } else if (small) {
    if (tid < 64) {
      bool ok;
      switch (RMs) {
        case 4: ok = wave_cholesky<4>(H, L, R, tid); break;
        case 8: ok = wave_cholesky<8>(H, L, R, tid); break;
        case 12: ok = wave_cholesky<12>(H, L, R, tid); break;
        default: ok = wave_cholesky<16>(H, L, R, tid); break;
      }
      if (tid == 0) flag = ok;
    }
    __syncthreads();
    failed = flag == 0;
  } else {
    failed = !block_cholesky(L, H, R, &flag);
  }
  if (failed && !nonneg) {
    // rank-deficient: every row block computes the same P = H^+ (in the factor's place; H is used up as work area)
    __syncthreads();
    failed = !block_pinv(H, R, H, xs, L, red, red, &flag);
    pinv = !failed;
  }
  if (failed) {
    if (tid == 0 && blockIdx.y == 0) out->status = 3;   // CALS_NUMERICAL; factors of this mode stay untouched
    return;
  }

  const int nblk = gridDim.y;
  const int rpb = rows_per_block(a.In, nblk);
  const int r0 = blockIdx.y * rpb;
  const int r1 = (r0 + rpb < a.In) ? (r0 + rpb) : a.In;
  double gacc[3] = {0.0, 0.0, 0.0};
  double inner = 0.0;
  const double* Mb = a.M + d.col;
  double* Ub = a.U + d.col;
  if (small && !pinv) {
    switch (RMs) {
      case 4: solve_rows_small<4>(a, d, L, xs, nonneg, r0, r1, gacc, inner); break;
      case 8: solve_rows_small<8>(a, d, L, xs, nonneg, r0, r1, gacc, inner); break;
      case 12: solve_rows_small<12>(a, d, L, xs, nonneg, r0, r1, gacc, inner); break;
      default: solve_rows_small<16>(a, d, L, xs, nonneg, r0, r1, gacc, inner); break;
    }
  }
  for (int base = (small && !pinv) ? r1 : r0; base < r1; base += kRows) {
    const int i = base + tid;
    const int nrows = (r1 - base < kRows) ? (r1 - base) : kRows;
    if (i < r1) {
      const double* mrow = Mb + (int64_t)i * a.ld;
      if (nonneg) {
        const double* xrow = a.X + (int64_t)i * a.ld + d.col;
        for (int r = 0; r < R; ++r) xs[r * kXs + tid] = xrow[r];
      } else if (pinv) {
        row_times_matrix(L, R, mrow, Ub + (int64_t)i * a.ld, xs);
      } else {
        for (int r = 0; r < R; ++r) xs[r * kXs + tid] = mrow[r];
        for (int r = 0; r < R; ++r) {          // L y = m
          double v = xs[r * kXs + tid];
          for (int k = 0; k < r; ++k) v -= L[r * R + k] * xs[k * kXs + tid];
          xs[r * kXs + tid] = v / L[r * R + r];
        }
        for (int r = R - 1; r >= 0; --r) {     // L^T x = y
          double v = xs[r * kXs + tid];
          for (int k = r + 1; k < R; ++k) v -= L[k * R + r] * xs[k * kXs + tid];
          xs[r * kXs + tid] = v / L[r * R + r];
        }
      }
      double* urow = Ub + (int64_t)i * a.ld;
      double part = 0.0;
      for (int r = 0; r < R; ++r) {
        const double x = xs[r * kXs + tid];
        urow[r] = x;
        part += x * mrow[r];
      }
      inner += part;
    }
    __syncthreads();
    gram_accumulate(xs, R, nrows, gacc);
    __syncthreads();
  }
  double* part = a.part + ((size_t)blockIdx.x * nblk + blockIdx.y) * kUpdatePartStride;
  const int npairs = R * (R + 1) / 2;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const int p = tid + 256 * q;
    if (p < npairs) part[p] = gacc[q];
  }
  const double in = block_sum(inner, red);
  if (tid == 0) part[528] = in;
}

__global__ void __launch_bounds__(256) update_finish_kernel(UpdateArgs a) {
  extern __shared__ double lds[];
  const ModelDesc d = a.desc[blockIdx.x];
  ModelState* st = a.state + d.sid;
  ModelOut* out = a.out + d.sid;
  const int tid = threadIdx.x;
  if ((d.flags & 1u) && blockIdx.y == 0 && tid == 0) a.nn_fail[blockIdx.x] = 0;
  if (out->status != 0) return;               // this launch never changes a status
  const int R = d.rank;
  const int nblk = gridDim.y;
  double* Gl = lds;                           // R*R, Gramian of the updated factor
  double* red = Gl + kGramStride;             // 256
  double* lam = red + 256;                    // R
  const double* part = a.part + (size_t)blockIdx.x * nblk * kUpdatePartStride;
  const int npairs = R * (R + 1) / 2;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const int p = tid + 256 * q;
    if (p < npairs) {
      double g = 0.0;
      for (int b = 0; b < nblk; ++b) g += part[(size_t)b * kUpdatePartStride + p];
      int r, s;
      pair_rs(p, r, s);
      Gl[r * R + s] = g;
      Gl[s * R + r] = g;
    }
  }
  __syncthreads();
  if (blockIdx.y == 0 && a.mode == a.nmodes - 1) {
    double v = 0.0;
    for (int e = tid; e < R * R; e += 256) v += (hadamard_of_others(st, a.nmodes, a.mode, e)) * Gl[e];
    const double normsq = block_sum(v, red);
    if (tid == 0) {
      double in = 0.0;
      for (int b = 0; b < nblk; ++b) in += part[(size_t)b * kUpdatePartStride + 528];
      st->inner = in;
      st->normsq = normsq;
      const double err = a.normT2 + normsq - 2.0 * in;
      out->err = err;
      out->fit = 1.0 - sqrt(err > 0.0 ? err : 0.0) / sqrt(a.normT2);
      out->iters += 1;
    }
  }
  if (tid < R) {
    const double l = sqrt(Gl[tid * R + tid]);
    lam[tid] = l;
    if (blockIdx.y == 0) a.lambda[d.sid * kMaxRank + tid] = l;
  }
  __syncthreads();
  if (blockIdx.y == 0)
    for (int e = tid; e < R * R; e += 256) {
      const int r = e / R, s = e % R;
      const double lr = lam[r] > 0.0 ? lam[r] : 1.0, ls = lam[s] > 0.0 ? lam[s] : 1.0;
      st->G[a.mode][e] = (Gl[e] / lr) / ls;
    }
  const int rpb = rows_per_block(a.In, nblk);
  const int r0 = blockIdx.y * rpb;
  const int r1 = (r0 + rpb < a.In) ? (r0 + rpb) : a.In;
  double* Ub = a.U + d.col;
  for (int i = r0 + tid; i < r1; i += 256) {
    double* urow = Ub + (int64_t)i * a.ld;
    for (int r = 0; r < R; ++r) {
      const double l = lam[r];
      if (l > 0.0) urow[r] = urow[r] / l;
    }
  }
}

static constexpr size_t kUpdateLds = sizeof(double) * (kMaxRank * kXs + 3 * kGramStride + 256 + kMaxRank);
static constexpr size_t kSolveLds = sizeof(double) * (kMaxRank * kXs + 2 * kGramStride + 256);
static constexpr size_t kFinishLds = sizeof(double) * (kGramStride + 256 + kMaxRank);

hipError_t launch_update(const UpdateArgs& a, hipStream_t stream) {
  static std::atomic<unsigned long long> attr_seen{0};
  if (first_use_on_current_device(attr_seen)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(update_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kUpdateLds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(update_solve_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSolveLds);
    if (e != hipSuccess) return e;
  }
  if (a.n_models < 1) return hipSuccess;
  const int nblk = update_row_blocks(a.In);
  if (nblk == 1) {
    hipLaunchKernelGGL(update_kernel, dim3(a.n_models), dim3(256), kUpdateLds, stream, a);
    return hipGetLastError();
  }
  if (!a.part) return hipErrorInvalidValue;
  hipLaunchKernelGGL(update_solve_kernel, dim3(a.n_models, nblk), dim3(256), kSolveLds, stream, a);
  hipLaunchKernelGGL(update_finish_kernel, dim3(a.n_models, nblk), dim3(256), kFinishLds, stream, a);
  return hipGetLastError();
}

// ---- Gramians of freshly inserted models: one workgroup per (model, mode) -------------------------
struct GramInitArgs {
  const ModelDesc* desc;
  ModelState* state;
  ModelOut* out;
  double* lambda;
  uint32_t* passive[kMaxModes];
  int capacity;
  int reset_out;
  const double* U[kMaxModes];
  int In[kMaxModes];
  int ld, first;
};

__global__ void __launch_bounds__(256) gram_init_kernel(GramInitArgs a) {
  extern __shared__ double lds[];
  const ModelDesc d = a.desc[a.first + blockIdx.x];
  const int mode = blockIdx.y;
  ModelState* st = a.state + d.sid;
  const int tid = threadIdx.x, R = d.rank, In = a.In[mode];
  double* xs = lds;
  double* Gl = xs + kMaxRank * kXs;
  double gacc[3] = {0.0, 0.0, 0.0};
  const double* Ub = a.U[mode] + d.col;
  for (int base = 0; base < In; base += kRows) {
    const int i = base + tid;
    const int nrows = (In - base < kRows) ? (In - base) : kRows;
    if (i < In)
      for (int r = 0; r < R; ++r) xs[r * kXs + tid] = Ub[(int64_t)i * a.ld + r];
    __syncthreads();
    gram_accumulate(xs, R, nrows, gacc);
    __syncthreads();
  }
  gram_store(gacc, R, Gl);
  __syncthreads();
  for (int e = tid; e < R * R; e += 256) st->G[mode][e] = Gl[e];
  if (a.reset_out && mode == 0 && tid == 0) {
    ModelOut o;
    o.err = 0.0; o.fit = 0.0; o.status = 0; o.iters = 0; o.ls_accepted = 0; o.pad = 0;
    a.out[d.sid] = o;
  }
  if (a.reset_out && mode == 0 && tid < kMaxRank) a.lambda[d.sid * kMaxRank + tid] = 1.0;
  if (a.reset_out && a.passive[mode])          // a fresh model starts with empty passive sets
    for (int i = tid; i < In; i += 256) a.passive[mode][(int64_t)i * a.capacity + d.sid] = 0u;
}

hipError_t launch_gram_init(const ModelDesc* desc, ModelState* state, ModelOut* out, double* lambda, bool reset_out,
                            uint32_t* const* passive, int capacity, const double* const* U, const int* In, int nmodes,
                            int ld, int first, int count, hipStream_t stream) {
  static std::atomic<unsigned long long> attr_seen{0};
  const size_t lds = sizeof(double) * (kMaxRank * kXs + kGramStride);
  if (first_use_on_current_device(attr_seen)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gram_init_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  if (count < 1) return hipSuccess;
  if (nmodes < 1 || nmodes > kMaxModes) return hipErrorInvalidValue;
  GramInitArgs a{};
  a.desc = desc; a.state = state; a.out = out; a.lambda = lambda; a.reset_out = reset_out ? 1 : 0; a.ld = ld; a.first = first;
  a.capacity = capacity;
  for (int n = 0; n < nmodes; ++n) { a.U[n] = U[n]; a.In[n] = In[n]; a.passive[n] = passive ? passive[n] : nullptr; }
  hipLaunchKernelGGL(gram_init_kernel, dim3(count, nmodes), dim3(256), lds, stream, a);
  return hipGetLastError();
}

// ---- ||T||^2 with a fixed reduction tree ----------------------------------------------------------
constexpr int kNormBlocks = 1024;

__global__ void __launch_bounds__(256) norm_sq_partial_kernel(const double* __restrict__ T, int64_t n,
                                                              double* __restrict__ partial, int* __restrict__ flag) {
  __shared__ double red[256];
  const int64_t per = (n + kNormBlocks - 1) / kNormBlocks;
  const int64_t b0 = (int64_t)blockIdx.x * per;
  const int64_t b1 = (b0 + per < n) ? (b0 + per) : n;
  double s = 0.0;
  bool bad = false;
  for (int64_t i = b0 + threadIdx.x; i < b1; i += 256) {
    const double v = T[i];
    bad |= !isfinite(v);
    s += v * v;
  }
  if (bad) atomicOr(flag, 1);
  const double tot = block_sum(s, red);
  if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

__global__ void __launch_bounds__(256) norm_sq_final_kernel(const double* __restrict__ partial, double* __restrict__ out) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < kNormBlocks; i += 256) s += partial[i];
  const double tot = block_sum(s, red);
  if (threadIdx.x == 0) out[0] = tot;
}

hipError_t launch_norm_sq(const double* T, int64_t n, double* partial, double* out, int* flag, hipStream_t stream) {
  hipLaunchKernelGGL(norm_sq_partial_kernel, dim3(kNormBlocks), dim3(256), 0, stream, T, n, partial, flag);
  hipLaunchKernelGGL(norm_sq_final_kernel, dim3(1), dim3(256), 0, stream, (const double*)partial, out);
  return hipGetLastError();
}

// ---- column gather (compaction of the multi-matrices after retirements; Sec. 4) -------------------
__global__ void __launch_bounds__(256) gather_columns_kernel(const double* __restrict__ src, double* __restrict__ dst,
                                                             const int32_t* __restrict__ map, int rows, int ncols, int ld) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)rows * ncols;
  if (idx >= total) return;
  const int i = (int)(idx / ncols), c = (int)(idx % ncols);
  dst[(int64_t)i * ld + c] = src[(int64_t)i * ld + map[c]];
}

hipError_t launch_gather_columns(const double* src, double* dst, const int32_t* map, int rows, int ncols, int ld,
                                 hipStream_t stream) {
  if (rows < 1 || ncols < 1) return hipSuccess;
  const int64_t total = (int64_t)rows * ncols;
  hipLaunchKernelGGL(gather_columns_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, src, dst, map,
                     rows, ncols, ld);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256) copy_block_kernel(const double* __restrict__ src, int64_t src_ld,
                                                         double* __restrict__ dst, int64_t dst_ld,
                                                         const int32_t* __restrict__ map, int rows, int cols) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)rows * cols) return;
  const int i = (int)(idx / cols), c = (int)(idx % cols);
  dst[(int64_t)i * dst_ld + c] = src[(int64_t)i * src_ld + (map ? map[c] : c)];
}

hipError_t launch_copy_block(const double* src, int64_t src_ld, double* dst, int64_t dst_ld, int rows, int cols,
                             hipStream_t stream) {
  return launch_gather_block(src, src_ld, dst, dst_ld, nullptr, rows, cols, stream);
}

hipError_t launch_gather_block(const double* src, int64_t src_ld, double* dst, int64_t dst_ld, const int32_t* map,
                               int rows, int cols, hipStream_t stream) {
  if (rows < 1 || cols < 1) return hipSuccess;
  const int64_t total = (int64_t)rows * cols;
  hipLaunchKernelGGL(copy_block_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, src, src_ld, dst,
                     dst_ld, map, rows, cols);
  return hipGetLastError();
}

}  // namespace cals
