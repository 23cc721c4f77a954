// Non-negative update for CALS (Sec. 5 of the paper, "Non-negativity constraints"): after the fused MTTKRP the
// normal-equation solve of a NONNEG model is replaced, row by row, by
//     minimise 1/2 x^T H x - m^T x   subject to x >= 0,
// with an active-set (Lawson-Hanson) search on (H, m); the passive set a row ends with is kept for the next
// iteration (warm start; dropped if its sub-block of H is not positive definite).  H and the MTTKRP are computed
// once per mode update, exactly as for plain ALS.
//
// One wavefront per row, lane r = component r.  The search is a chain of small dense solves; spreading a row
// over the lanes turns each solve from O(R^3) dependent steps into O(R^2) register operations:
//   - lane i keeps row i of H in registers (loaded once per model and wavefront) and, per solve, row i of the
//     working matrix; the passive sub-system is solved by symmetric Gaussian elimination without pivoting
//     (pivot j is broadcast from lane j with v_readlane, every lane below updates its own row and right-hand
//     side) and column-oriented back-substitution.  A pivot that is not positive and finite is the same outcome
//     as a failed Cholesky factorisation;
//   - feasibility, the step length and the choice of the entering variable are wavefront votes and reductions;
//     ties in the gradient test go to the lowest index, as in a scalar left-to-right scan;
//   - all control flow is uniform over the wavefront, so the search needs no barrier.
// The chains of dependent register operations make the kernel latency-bound, so what counts is how many wavefronts
// a SIMD holds: H sits in LDS (one copy per workgroup; a wavefront reloads its working rows from there for every
// solve), the pivots' reciprocals share one lane-indexed register, and the kernel is instantiated per largest rank
// class of the launch, so that a queue of low-rank models does not run with the register budget of rank 32.
#include <cfloat>
#include <cmath>
#include <cstdlib>

#include "cals_internal.h"

namespace cals {

__device__ inline double wave_max(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o));
  return v;
}
__device__ inline double wave_min(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmin(v, __shfl_xor(v, o));
  return v;
}

constexpr int kNnlsRowsPerBlock = 4;    // default: 4 wavefronts x 1 row (short critical path per wavefront)

// All rows [row0, row1) with stride 4 from row0 + wave, for one model of rank R <= RM.
template <int RM>
__device__ __forceinline__ void nnls_rows(const NnlsArgs& a, const ModelDesc& d, int slot, int row0, int row1, int lane,
                                          int wave, const double* Hs /* LDS: (RM+1) rows of RM+1, zero outside R x R */) {
  const int R = d.rank;
  const bool live = lane < R;
  // row `lane` of H; lanes beyond the rank read the zero row.  (volatile: every use is a fresh LDS read -- the
  // compiler would otherwise keep the whole row in registers for the lifetime of the wavefront)
  const double* hrow = Hs + (live ? lane : RM) * (RM + 1);
  double cs = 0.0;                       // H is symmetric: row sums are column sums
#pragma unroll
  for (int k = 0; k < RM; ++k) cs += fabs(hrow[k]);
  const double h1 = wave_max(cs);        // ||H||_1
  const double tau = 10.0 * DBL_EPSILON * h1 * (double)R;
  const int cap = 30 * R;
  const uint32_t full = (R >= 32) ? 0xffffffffu : ((1u << R) - 1u);

  for (int i = row0 + wave; i < row1; i += 4) {
    uint32_t* pslot = a.passive + (int64_t)i * a.capacity + d.sid;
    uint32_t P = (uint32_t)__builtin_amdgcn_readfirstlane((int)*pslot) & full;
    const double m = live ? a.M[(int64_t)i * a.ld + d.col + lane] : 0.0;
    double x = 0.0;                      // component `lane` of the iterate; zero outside the passive set
    int steps = 0;
    bool bad = false;
    bool from_warm = (P != 0);           // the passive set still derives from the warm start
    for (;;) {
      while (P) {
        // ---- solve H_PP s_P = m_P: elimination on the passive rows and columns, in ascending index order
        double arow[RM];
#pragma unroll
        for (int k = 0; k < RM; ++k) arow[k] = hrow[k];
        double b = m;
        double rpiv = 0.0;                 // lane j: reciprocal of pivot j, reused by the back-substitution
        bool ok = true;
#pragma unroll
        for (int j = 0; j < RM; ++j) {
          if (ok && ((P >> j) & 1u)) {         // P has no bits at or above R
            const double dj = readlane_f64(arow[j], j);
            if (!(dj > 0.0) || !isfinite(dj)) {
              ok = false;
            } else {
              const double rp = 1.0 / dj;
              rpiv = (lane == j) ? rp : rpiv;
              const double mult = (lane > j) ? arow[j] * rp : 0.0;
              const double bj = readlane_f64(b, j);
              b = fma(-mult, bj, b);
#pragma unroll
              for (int k = j + 1; k < RM; ++k) arow[k] = fma(-mult, readlane_f64(arow[k], j), arow[k]);
            }
          }
        }
        if (!ok) {
          if (!from_warm) { bad = true; break; }
          // a warm start whose sub-block cannot be factorised is dropped: restart from the empty set
          from_warm = false;
          P = 0;
          x = 0.0;
          break;
        }
        double s = 0.0;
#pragma unroll
        for (int k = RM - 1; k >= 0; --k) {
          if ((P >> k) & 1u) {
            const double sk = readlane_f64(b, k) * readlane_f64(rpiv, k);
            s = (lane == k) ? sk : s;
            b = (lane < k) ? fma(-arow[k], sk, b) : b;
          }
        }
        // ---- feasible: take it; else step towards it until the first component reaches zero
        const bool inP = live && ((P >> lane) & 1u);
        const bool nonpos = inP && !(s > 0.0);
        if (__ballot(nonpos) == 0) {
          x = inP ? s : 0.0;
          break;
        }
        const double q = nonpos ? x / (x - s) : 1.0;
        const double beta = wave_min(q);                            // fmin drops the NaN of 0/0
        const double xn = x + beta * (s - x);
        // a variable that bounds the step has reached zero and leaves the passive set, whatever rounding makes of
        // x + beta (s - x) for it (a tiny positive result would stall the search)
        const bool keep = inP && (xn > 0.0) && !(nonpos && q == beta);
        x = keep ? xn : 0.0;
        P = (uint32_t)__ballot(keep);
        if (++steps > cap) break;
      }
      if (bad || steps > cap) break;
      // ---- gradient test: move the most violating variable into the passive set
      double w = m;
#pragma unroll
      for (int k = 0; k < RM; ++k) w = fma(-hrow[k], readlane_f64(x, k), w);   // x and hrow are zero beyond R
      const bool cand = live && !((P >> lane) & 1u) && (w > tau);
      if (__ballot(cand) == 0) break;
      const double wmax = wave_max(cand ? w : -INFINITY);
      const unsigned long long winners = __ballot(cand && w == wmax);
      P |= 1u << __builtin_ctzll(winners);
      from_warm = false;
      if (++steps > cap) break;
    }
    if (bad) {
      if (lane == 0) atomicOr(a.fail + slot, 1);
      continue;
    }
    if (lane == 0) *pslot = P;
    if (live) a.X[(int64_t)i * a.ld + d.col + lane] = x;
  }
}

// RMAX = the largest rank class among the NONNEG models of the launch: the kernel's register budget is that of
// its widest instantiation, so a queue of low-rank models runs with many more wavefronts per SIMD.
template <int RM, int RMAX>
__device__ __forceinline__ void nnls_class(const NnlsArgs& a, const ModelDesc& d, int slot, int row0, int row1, double* Hs) {
  if constexpr (RM <= RMAX) {
    const ModelState* st = a.state + d.sid;
    const int R = d.rank;
    for (int e = threadIdx.x; e < (RM + 1) * (RM + 1); e += 256) {
      const int r = e / (RM + 1), k = e % (RM + 1);
      Hs[e] = (r < R && k < R) ? hadamard_of_others(st, a.nmodes, a.mode, r * R + k) : 0.0;
    }
    __syncthreads();
    nnls_rows<RM>(a, d, slot, row0, row1, threadIdx.x & 63, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), Hs);
  }
}

template <int RMAX>
__global__ void __launch_bounds__(256) nnls_kernel(NnlsArgs a) {
  __shared__ double Hs[(RMAX + 1) * (RMAX + 1)];
  // grid: x = row blocks (a mode can have millions of rows), y = slot positions (at most a few thousand), taken in
  // the order the host gives: workgroups are handed out y by y, and a launch ends with its last workgroup, so the
  // models whose rows take longest (the highest ranks) go first
  const int slot = a.order[blockIdx.y];
  const ModelDesc d = a.desc[slot];
  if (!(d.flags & 1u)) return;
  if (a.out[d.sid].status != 0) return;
  const int row0 = blockIdx.x * a.rows_per_block;
  if (row0 >= a.In) return;
  const int row1 = (row0 + a.rows_per_block < a.In) ? (row0 + a.rows_per_block) : a.In;
  switch ((d.rank + 3) / 4) {           // register arrays sized to the rank rounded up to a multiple of 4
    case 1: nnls_class<4, RMAX>(a, d, slot, row0, row1, Hs); break;
    case 2: nnls_class<8, RMAX>(a, d, slot, row0, row1, Hs); break;
    case 3: nnls_class<12, RMAX>(a, d, slot, row0, row1, Hs); break;
    case 4: nnls_class<16, RMAX>(a, d, slot, row0, row1, Hs); break;
    case 5: nnls_class<20, RMAX>(a, d, slot, row0, row1, Hs); break;
    case 6: nnls_class<24, RMAX>(a, d, slot, row0, row1, Hs); break;
    case 7: nnls_class<28, RMAX>(a, d, slot, row0, row1, Hs); break;
    default: nnls_class<32, RMAX>(a, d, slot, row0, row1, Hs); break;
  }
}

hipError_t launch_nnls(const NnlsArgs& a0, hipStream_t stream) {
  if (a0.n_models < 1 || a0.In < 1) return hipSuccess;
  if (!a0.order) return hipErrorInvalidValue;
  NnlsArgs a = a0;
  a.rows_per_block = kNnlsRowsPerBlock;
  if (a.n_models > 65535) return hipErrorInvalidValue;
  const dim3 grid((a.In + a.rows_per_block - 1) / a.rows_per_block, a.n_models);
  const int rmax = a.max_rank < 1 ? 1 : a.max_rank;
  if (rmax <= 8) hipLaunchKernelGGL(nnls_kernel<8>, grid, dim3(256), 0, stream, a);
  else if (rmax <= 12) hipLaunchKernelGGL(nnls_kernel<12>, grid, dim3(256), 0, stream, a);
  else if (rmax <= 16) hipLaunchKernelGGL(nnls_kernel<16>, grid, dim3(256), 0, stream, a);
  else if (rmax <= 20) hipLaunchKernelGGL(nnls_kernel<20>, grid, dim3(256), 0, stream, a);
  else if (rmax <= 24) hipLaunchKernelGGL(nnls_kernel<24>, grid, dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(nnls_kernel<32>, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace cals
