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

__device__ inline int nnls_rows_per_block(int R) { return R <= 20 ? 64 : (R <= 27 ? 32 : 16); }

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
      for (int j = 0; j < R && !bad; ++j) {
        if (!(P & (1u << j))) continue;
        double dj = H[j * R + j];
        for (int k = 0; k < j; ++k)
          if (P & (1u << k)) dj -= LP(j, k) * LP(j, k);
        if (!(dj > 0.0) || !isfinite(dj)) { bad = true; break; }
        dj = sqrt(dj);
        LP(j, j) = dj;
        for (int r = j + 1; r < R; ++r) {
          if (!(P & (1u << r))) continue;
          double v = H[r * R + j];
          for (int k = 0; k < j; ++k)
            if (P & (1u << k)) v -= LP(r, k) * LP(j, k);
          LP(r, j) = v / dj;
        }
      }
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
      for (int r = 0; r < R; ++r) {
        if (!(P & (1u << r))) continue;
        double v = MV(r);
        for (int k = 0; k < r; ++k)
          if (P & (1u << k)) v -= LP(r, k) * SV(k);
        SV(r) = v / LP(r, r);
      }
      for (int r = R - 1; r >= 0; --r) {
        if (!(P & (1u << r))) continue;
        double v = SV(r);
        for (int k = r + 1; k < R; ++k)
          if (P & (1u << k)) v -= LP(k, r) * SV(k);
        SV(r) = v / LP(r, r);
      }
      bool feasible = true;
      for (int r = 0; r < R; ++r)
        if ((P & (1u << r)) && !(SV(r) > 0.0)) feasible = false;
      if (feasible) {
        for (int r = 0; r < R; ++r) XV(r) = (P & (1u << r)) ? SV(r) : 0.0;
        break;
      }
      double beta = 1.0;
      for (int r = 0; r < R; ++r)
        if ((P & (1u << r)) && !(SV(r) > 0.0)) {
          const double xa = XV(r);
          const double q = xa / (xa - SV(r));
          if (q < beta) beta = q;
        }
      for (int r = 0; r < R; ++r) {
        if (!(P & (1u << r))) continue;
        const double xn = XV(r) + beta * (SV(r) - XV(r));
        if (!(xn > 0.0)) { XV(r) = 0.0; P &= ~(1u << r); }
        else XV(r) = xn;
      }
      if (++steps > cap) break;
    }
    if (bad || steps > cap) break;
    // gradient test: move the most violating variable into the passive set
    int best = -1;
    double wbest = tau;
    for (int j = 0; j < R; ++j) {
      if (P & (1u << j)) continue;
      double w = MV(j);
      for (int k = 0; k < R; ++k) w -= H[j * R + k] * XV(k);
      if (w > wbest) { wbest = w; best = j; }
    }
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
}

hipError_t launch_nnls(const NnlsArgs& a, hipStream_t stream) {
  static bool attr_done = false;
  // worst case over the three row-block sizes: R = 20 with 64 rows
  const size_t lds = sizeof(double) * (kGramStride + (size_t)(210 + 60) * 64 + 64);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(nnls_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  if (a.n_models < 1) return hipSuccess;
  hipLaunchKernelGGL(nnls_kernel, dim3(a.n_models, (a.In + 15) / 16), dim3(64), lds, stream, a);
  return hipGetLastError();
}

}  // namespace cals
