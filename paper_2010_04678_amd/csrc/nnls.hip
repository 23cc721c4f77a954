// Non-negative update for CALS (Sec. 5 of the paper, "Non-negativity constraints"): after the fused MTTKRP the
// normal-equation solve of a NONNEG model is replaced, row by row, by
//     minimise 1/2 x^T H x - m^T x   subject to x >= 0,
// with an active-set (Lawson-Hanson) search on (H, m); the passive set a row ends with is kept for the next
// iteration (warm start; dropped if its sub-block of H is not positive definite).  H and the MTTKRP are computed once per mode update, exactly as for plain ALS.
//
// One lane per row, one wavefront per workgroup.  Every lane runs the textbook sequence (factorise the passive
// sub-block of H, solve, step towards feasibility, gradient test) in the same order of operations as a scalar
// implementation; loops run over the full index range with the lane's passive mask as predicate, so all lanes
// read H at the same (broadcast) address.  Per-lane vectors and the packed Cholesky factor live in LDS,
// element-major ([element][lane]), which is bank-conflict free.
#include <cfloat>

#include "cals_internal.h"

namespace cals {

// Rows per workgroup: few, so that the per-lane LDS arrays stay small and several wavefronts share a CU (the
// search is a chain of dependent LDS reads: it needs occupancy, not lanes).
__host__ __device__ inline int nnls_rows_per_block(int R) { return R <= 24 ? 16 : 8; }
__host__ __device__ inline size_t nnls_lds_doubles(int R) {
  return (size_t)kGramStride + (size_t)(R * (R + 1) / 2 + 3 * R) * nnls_rows_per_block(R);
}

__global__ void __launch_bounds__(64) nnls_kernel(NnlsArgs a) {
  extern __shared__ double lds[];
  const ModelDesc d = a.desc[blockIdx.x];
  if (!(d.flags & 1u)) return;
  if (a.out[d.sid].status != 0) return;
  const int R = d.rank;
  const int RPB = nnls_rows_per_block(R);
  const int base = blockIdx.y * RPB;
  if (base >= a.In) return;
  const int lane = threadIdx.x;
  const ModelState* st = a.state + d.sid;
  const int ma = (a.mode == 0) ? 1 : 0, mb = (a.mode == 2) ? 1 : 2;
  const int npack = R * (R + 1) / 2;
  double* H = lds;                       // R*R (symmetric), shared by the lanes
  double* Lp = H + kGramStride;          // [npack][RPB]  packed lower Cholesky factor, indexed by original indices
  double* xv = Lp + npack * RPB;         // [R][RPB]
  double* sv = xv + R * RPB;             // [R][RPB]
  double* mv = sv + R * RPB;             // [R][RPB]
  for (int e = lane; e < R * R; e += 64) H[e] = st->G[ma][e] * st->G[mb][e];
  __syncthreads();
  double h1 = 0.0;                       // ||H||_1 (same for all lanes)
  for (int j = 0; j < R; ++j) {
    double cs = 0.0;
    for (int i = 0; i < R; ++i) cs += fabs(H[i * R + j]);
    if (cs > h1) h1 = cs;
  }
  const double tau = 10.0 * DBL_EPSILON * h1 * (double)R;
  const int cap = 30 * R;
  const int i = base + lane;
  if (lane >= RPB || i >= a.In) return;  // no barrier below this point

#define LP(r, c) Lp[((r) * ((r) + 1) / 2 + (c)) * RPB + lane]
#define XV(r) xv[(r) * RPB + lane]
#define SV(r) sv[(r) * RPB + lane]
#define MV(r) mv[(r) * RPB + lane]
// loops over the members of a bit set in ascending order (the order a scalar implementation visits them)
#define FOR_BITS(var, set) for (uint32_t var##_s = (set); var##_s; var##_s &= var##_s - 1) { const int var = __builtin_ctz(var##_s);
#define END_BITS }
  const uint32_t full = (R >= 32) ? 0xffffffffu : ((1u << R) - 1u);
  uint32_t* pslot = a.passive + (int64_t)i * a.capacity + d.sid;
  uint32_t P = *pslot & full;
  const double* mrow = a.M + (int64_t)i * a.ld + d.col;
  for (int r = 0; r < R; ++r) { MV(r) = mrow[r]; XV(r) = 0.0; }
  int steps = 0;
  bool bad = false;
  bool from_warm = (P != 0);             // the passive set still derives from the warm start
  for (;;) {
    while (P) {
      // Cholesky of H restricted to the passive set (columns in ascending index order)
      FOR_BITS(j, P)
        const uint32_t below = P & ((1u << j) - 1u);
        double dj = H[j * R + j];
        FOR_BITS(k, below) dj -= LP(j, k) * LP(j, k); END_BITS
        if (!(dj > 0.0) || !isfinite(dj)) { bad = true; break; }
        dj = sqrt(dj);
        LP(j, j) = dj;
        const uint32_t above = (j >= 31) ? 0u : (P & ~((2u << j) - 1u));
        FOR_BITS(r, above)
          double v = H[r * R + j];
          FOR_BITS(k, below) v -= LP(r, k) * LP(j, k); END_BITS
          LP(r, j) = v / dj;
        END_BITS
      END_BITS
      if (bad) {
        if (!from_warm) break;
        // a warm start whose sub-block cannot be factorised is dropped: restart from the empty set
        bad = false;
        from_warm = false;
        P = 0;
        for (int r = 0; r < R; ++r) XV(r) = 0.0;
        break;
      }
      // solve (L L^T) s = m on the passive set
      FOR_BITS(r, P)
        double v = MV(r);
        FOR_BITS(k, P & ((1u << r) - 1u)) v -= LP(r, k) * SV(k); END_BITS
        SV(r) = v / LP(r, r);
      END_BITS
      for (int r = R - 1; r >= 0; --r) {
        if (!(P & (1u << r))) continue;
        double v = SV(r);
        const uint32_t above = (r >= 31) ? 0u : (P & ~((2u << r) - 1u));
        FOR_BITS(k, above) v -= LP(k, r) * SV(k); END_BITS
        SV(r) = v / LP(r, r);
      }
      bool feasible = true;
      FOR_BITS(r, P) if (!(SV(r) > 0.0)) feasible = false; END_BITS
      if (feasible) {
        for (int r = 0; r < R; ++r) XV(r) = (P & (1u << r)) ? SV(r) : 0.0;
        break;
      }
      double beta = 1.0;
      FOR_BITS(r, P)
        if (!(SV(r) > 0.0)) {
          const double xa = XV(r);
          const double q = xa / (xa - SV(r));
          if (q < beta) beta = q;
        }
      END_BITS
      const uint32_t Pold = P;
      FOR_BITS(r, Pold)
        const double xn = XV(r) + beta * (SV(r) - XV(r));
        if (!(xn > 0.0)) { XV(r) = 0.0; P &= ~(1u << r); }
        else XV(r) = xn;
      END_BITS
      if (++steps > cap) break;
    }
    if (bad || steps > cap) break;
    // gradient test: move the most violating variable into the passive set (x is zero outside P)
    int best = -1;
    double wbest = tau;
    FOR_BITS(j, full & ~P)
      double w = MV(j);
      FOR_BITS(k, P) w -= H[j * R + k] * XV(k); END_BITS
      if (w > wbest) { wbest = w; best = j; }
    END_BITS
    if (best < 0) break;
    P |= (1u << best);
    from_warm = false;
    if (++steps > cap) break;
  }
  if (bad) {
    atomicOr(a.fail + blockIdx.x, 1);
    return;
  }
  *pslot = P;
  double* xrow = a.X + (int64_t)i * a.ld + d.col;
  for (int r = 0; r < R; ++r) xrow[r] = XV(r);
#undef LP
#undef XV
#undef SV
#undef MV
#undef FOR_BITS
#undef END_BITS
}

hipError_t launch_nnls(const NnlsArgs& a, hipStream_t stream) {
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(nnls_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(sizeof(double) * nnls_lds_doubles(kMaxRank)));
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  if (a.n_models < 1) return hipSuccess;
  const int rmax = a.max_rank < 1 ? 1 : (a.max_rank > kMaxRank ? kMaxRank : a.max_rank);
  size_t doubles = 0;
  for (int r = 1; r <= rmax; ++r) doubles = nnls_lds_doubles(r) > doubles ? nnls_lds_doubles(r) : doubles;
  hipLaunchKernelGGL(nnls_kernel, dim3(a.n_models, (a.In + 7) / 8), dim3(64), sizeof(double) * doubles, stream, a);
  return hipGetLastError();
}

}  // namespace cals
