// Fused multi-model MTTKRP for a dense 3-way fp64 tensor on gfx950 (Eq. (2) of the paper):
//   M[m, c] = sum_{ia, ib} T[m, ia, ib] * (Ua[ia, c] * Ub[ib, c])      for every fused column c.
//
// Work decomposition
//   grid.x : blocks of 64 output rows (4 wavefronts x one 16-row MFMA tile each)
//   grid.y : blocks of 16*WN fused columns (normally a single block holding every column, so the
//            tensor is streamed from HBM exactly once)
//   grid.z : split of the contraction range K = Ia*Ib; partial results go to a workspace and are
//            added in split order by a second kernel (fixed order => bit-reproducible results).
//
// Per workgroup and per stage of KA contraction indices
//   - the KRP tile (KA x 16*WN) is formed ONCE in LDS from factor rows (one fp64 multiply per
//     element, shared by all four wavefronts) -- it never exists in HBM;
//   - every wavefront loads its own 16 x KA tensor fragment straight from global memory into the
//     register layout of v_mfma_f64_16x16x4_f64 (lane l holds A[l%16][l/16]), one stage ahead;
//   - WN accumulator tiles (16x16, 4 doubles per lane) stay in registers for the whole K range.
// The LDS tile is double-buffered: the next stage's tile is produced piecewise between the MFMAs of
// the current stage, so one barrier per stage is enough.
#include "cals_internal.h"

namespace cals {

typedef double double4_t __attribute__((ext_vector_type(4)));

struct MttkrpKernelArgs {
  const double* T;
  const double* Ua;
  const double* Ub;
  double* P;          // output: partials [split][In][ld] or M itself when splits == 1
  int64_t sm, sa, sb;
  int64_t K, chunk;
  int64_t pstride;    // In * ld
  int In, Ia, Ib;
  int ncols, ld;
  int ntile16;        // ceil(ncols / 16)
};

// WRAPLOOP = false requires Ia >= KA (an index advanced by at most KA wraps at most once).
template <int WN, int KA, bool WRAPLOOP>
__global__ void __launch_bounds__(256) mttkrp_kernel(MttkrpKernelArgs a) {
  constexpr int NC = 16 * WN;                 // columns of the LDS tile
  constexpr int KS = KA / 4;                  // MFMA k-steps per stage
  constexpr int PIECE = 4 * NC;               // KRP elements produced per k-step (4 rows)
  constexpr int EPP = (PIECE + 255) / 256;    // ... per thread
  extern __shared__ double smem[];            // [2][KA][NC]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;                   // A: row within the tile / B,D: column within the tile
  const int lq = lane >> 4;                   // A,B: k within the k-step / D: row group
  const int m0 = blockIdx.x * 64 + wave * 16;
  const int n0 = blockIdx.y * NC;
  const int64_t kb = (int64_t)blockIdx.z * a.chunk;
  const int64_t ke = (kb + a.chunk < a.K) ? (kb + a.chunk) : a.K;
  const int nstage = (int)((ke - kb + KA - 1) / KA);
  const int row = m0 + li;
  const int Ia = a.Ia;

  double4_t acc[WN];
#pragma unroll
  for (int j = 0; j < WN; ++j) acc[j] = double4_t{0.0, 0.0, 0.0, 0.0};

  // ---- this lane's walk through the contraction range: k = kb + lq, then +4 per k-step.
  // a_off is the tensor offset of (row, ia, ib); a wrap of ia into the next ib adds `a_wrap`.
  // Rows past the end of the matrix are clamped to the last row (their results are never stored).
  int a_ia;
  int64_t a_off;
  int a_left;                                 // contraction indices left before ke, from this lane's k
  {
    const int64_t k = kb + lq;
    const int64_t ib = k / Ia;
    a_ia = (int)(k - ib * Ia);
    a_off = (int64_t)(row < a.In ? row : a.In - 1) * a.sm + (int64_t)a_ia * a.sa + ib * a.sb;
    a_left = (int)(ke - k);                   // <= chunk < 2^31 (checked on the host)
  }
  const int64_t a_step = 4 * a.sa;
  const int64_t a_wrap = a.sb - (int64_t)Ia * a.sa;

  double areg0[KS], areg1[KS];

  // The load is unconditional from a clamped (always valid) offset and the value is masked afterwards:
  // no divergent control flow, so the scheduler is free to hoist it.
  auto load_a_stage = [&](double* dst) {
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bool ok = a_left > 0;
      const double v = a.T[ok ? a_off : 0];
      dst[s] = ok ? v : 0.0;
      a_left -= 4;
      a_ia += 4;
      a_off += a_step;
      if (WRAPLOOP) {
        while (a_ia >= Ia) { a_ia -= Ia; a_off += a_wrap; }
      } else {
        if (a_ia >= Ia) { a_ia -= Ia; a_off += a_wrap; }
      }
    }
  };

  // ---- KRP tile production.  Thread t owns tile column(s) ptc[u] and the rows pr, pr+G, pr+2G, ...
  // (G row groups when the tile is narrower than the workgroup).  Rows and columns outside the problem
  // are clamped to valid ones instead of being zeroed: such a row meets a zero tensor fragment (a_left
  // <= 0), such a column only feeds output columns that are never stored.
  constexpr int G = (NC >= 256) ? 1 : (NC > 128 ? 1 : (NC > 64 ? 2 : (NC > 32 ? 4 : (NC > 16 ? 8 : 16))));
  constexpr int CU = (NC + 255) / 256;                     // columns per thread
  constexpr int RPT = KA / G;                              // rows per thread
  constexpr int X = RPT * CU;                              // elements per thread per stage
  constexpr int LSTEPS = (KS > 1) ? (KS - 1) : 1;          // k-steps that issue loads
  constexpr int XG = (X + LSTEPS - 1) / LSTEPS;            // elements per thread per k-step
  static_assert(KA % G == 0, "row groups must divide the stage");
  // Surplus threads (tile narrower than the workgroup, or second column past the tile edge) repeat
  // another thread's element: same address, same value, so every store is unconditional.
  const int pr = (NC < 256) ? (tid / NC) % G : 0;
  const int pc = (NC < 256) ? (tid % NC) : tid;
  int ptc[CU], pcg[CU];                                    // tile column, clamped global column
#pragma unroll
  for (int u = 0; u < CU; ++u) {
    const int tc = pc + 256 * u;
    ptc[u] = tc < NC ? tc : NC - 1;
    const int c = n0 + ptc[u];
    pcg[u] = c < a.ld ? c : a.ld - 1;
  }
  // block-uniform position of the stage being produced
  int p_ia, p_ib;
  {
    const int64_t ib = kb / Ia;
    p_ib = (int)ib;
    p_ia = (int)(kb - ib * Ia);
  }
  double pua[XG], pub[XG];

  auto fetch_group = [&](int g) {                          // issue the loads of elements [g*XG, g*XG+XG)
#pragma unroll
    for (int y = 0; y < XG; ++y) {
      const int x = g * XG + y;
      if (x < X) {
        const int r = pr + G * (x / CU);
        const int u = x % CU;
        int ia = p_ia + r, ib = p_ib;
        if (WRAPLOOP) {
          while (ia >= Ia) { ia -= Ia; ib += 1; }
        } else {
          if (ia >= Ia) { ia -= Ia; ib += 1; }
        }
        ib = ib < a.Ib ? ib : a.Ib - 1;
        pua[y] = a.Ua[ia * a.ld + pcg[u]];
        pub[y] = a.Ub[ib * a.ld + pcg[u]];
      }
    }
  };
  auto commit_group = [&](double* tile, int g) {           // multiply and store what fetch_group(g) fetched
#pragma unroll
    for (int y = 0; y < XG; ++y) {
      const int x = g * XG + y;
      if (x < X) {
        const int r = pr + G * (x / CU);
        tile[r * NC + ptc[x % CU]] = pua[y] * pub[y];
      }
    }
  };
  auto advance_producer = [&]() {
    p_ia += KA;
    if (WRAPLOOP) {
      while (p_ia >= Ia) { p_ia -= Ia; p_ib += 1; }
    } else {
      if (p_ia >= Ia) { p_ia -= Ia; p_ib += 1; }
    }
  };

  // one stage: MFMAs on (acur, tile `cur`) while the next fragment is fetched and the next tile produced
  auto run_stage = [&](const double* acur, double* anext, int cur) {
    const double* tile = smem + cur * (KA * NC);
    double* next_tile = smem + (cur ^ 1) * (KA * NC);
    load_a_stage(anext);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (KS > 1) {
        if (s >= 1) commit_group(next_tile, s - 1);
        if (s < KS - 1) fetch_group(s);
      } else {
        fetch_group(0);
      }
      const double av = acur[s];
      const double* brow = tile + (4 * s + lq) * NC + li;
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        const double bv = brow[16 * j];
        acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[j], 0, 0, 0);
      }
      if (KS == 1) commit_group(next_tile, 0);
    }
    advance_producer();
    __syncthreads();
  };

  // ---- prologue: tile 0 and fragment 0
#pragma unroll
  for (int g = 0; g < LSTEPS; ++g) { fetch_group(g); commit_group(smem, g); }
  advance_producer();
  load_a_stage(areg0);
  __syncthreads();

  for (int st = 0; st < nstage; st += 2) {
    run_stage(areg0, areg1, 0);
    if (st + 1 < nstage) run_stage(areg1, areg0, 1);
  }

  // ---- epilogue: D[4*v + lq][li] of every tile -> P[split][row][col]
  if (m0 < a.In) {
    double* P = a.P + (int64_t)blockIdx.z * a.pstride;
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int col = n0 + 16 * j + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = m0 + 4 * v + lq;
        if (r < a.In && col < a.ncols) P[(int64_t)r * a.ld + col] = acc[j][v];
      }
    }
  }
}

// Adds the split-K partials in split order: M[r][c] = ((P0 + P1) + P2) + ...
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const double* __restrict__ P, double* __restrict__ M,
                                                            int64_t n_rows_ld, int ld, int ncols, int splits) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n_rows_ld) return;
  const int c = (int)(idx % ld);
  if (c >= ncols) return;
  double s = P[idx];
  for (int z = 1; z < splits; ++z) s += P[idx + (int64_t)z * n_rows_ld];
  M[idx] = s;
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------

typedef void (*mttkrp_fn)(MttkrpKernelArgs);
struct Variant { int wn, ka; mttkrp_fn fast, general; };

#define CALS_VARIANT(WN_, KA_) { WN_, KA_, mttkrp_kernel<WN_, KA_, false>, mttkrp_kernel<WN_, KA_, true> }
static const Variant kVariants[] = {
    CALS_VARIANT(1, 64),  CALS_VARIANT(2, 32),  CALS_VARIANT(3, 32),  CALS_VARIANT(4, 32),  CALS_VARIANT(5, 16),
    CALS_VARIANT(6, 16),  CALS_VARIANT(7, 16),  CALS_VARIANT(8, 16),  CALS_VARIANT(9, 16),  CALS_VARIANT(10, 16),
    CALS_VARIANT(11, 16), CALS_VARIANT(12, 16), CALS_VARIANT(13, 16), CALS_VARIANT(14, 16), CALS_VARIANT(15, 16),
    CALS_VARIANT(16, 16), CALS_VARIANT(17, 16), CALS_VARIANT(18, 16), CALS_VARIANT(19, 16), CALS_VARIANT(20, 16),
    CALS_VARIANT(21, 16), CALS_VARIANT(22, 16), CALS_VARIANT(23, 16), CALS_VARIANT(24, 16), CALS_VARIANT(25, 16),
    CALS_VARIANT(26, 16), CALS_VARIANT(27, 16),
};
static constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
static constexpr int kMaxWn = 27;

static size_t variant_lds_bytes(const Variant& v) { return (size_t)2 * v.ka * 16 * v.wn * sizeof(double); }

hipError_t mttkrp_init() {
  for (int i = 0; i < kNumVariants; ++i) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kVariants[i].fast),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)variant_lds_bytes(kVariants[i]));
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kVariants[i].general),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)variant_lds_bytes(kVariants[i]));
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

static const Variant* pick_variant(int tiles_per_block) {
  for (int i = 0; i < kNumVariants; ++i)
    if (kVariants[i].wn >= tiles_per_block) return &kVariants[i];
  return &kVariants[kNumVariants - 1];
}

MttkrpPlan mttkrp_plan(const MttkrpProblem& p, int num_cus) {
  MttkrpPlan pl{};
  const int ntile16 = (p.ncols + 15) / 16;
  pl.ny = (ntile16 + kMaxWn - 1) / kMaxWn;
  const int per_block = (ntile16 + pl.ny - 1) / pl.ny;
  const Variant* v = pick_variant(per_block);
  pl.wn = v->wn;
  pl.ka = v->ka;
  pl.mtiles = (p.In + 63) / 64;
  const int64_t K = (int64_t)p.Ia * p.Ib;
  // resident workgroups per CU: bounded by registers (accumulators) and LDS
  int per_cu = (pl.wn >= 14) ? 1 : (pl.wn >= 6 ? 2 : (pl.wn >= 3 ? 4 : 8));
  const int64_t target = (int64_t)num_cus * per_cu;
  int64_t base = (int64_t)pl.mtiles * pl.ny;
  int64_t splits = (target + base - 1) / base;
  const int64_t max_splits = (K + 4 * pl.ka - 1) / (4 * pl.ka);   // at least four stages per split
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  int64_t chunk = (K + splits - 1) / splits;
  chunk = (chunk + pl.ka - 1) / pl.ka * pl.ka;
  splits = (K + chunk - 1) / chunk;
  pl.splits = (int)splits;
  pl.chunk = chunk;
  pl.workspace_bytes = (pl.splits > 1) ? (size_t)pl.splits * p.In * p.ld * sizeof(double) : 0;
  return pl;
}

hipError_t mttkrp_launch(const MttkrpProblem& p, const MttkrpPlan& pl, double* workspace, hipStream_t stream,
                         hipEvent_t* ev) {
  const Variant* v = nullptr;
  for (int i = 0; i < kNumVariants; ++i)
    if (kVariants[i].wn == pl.wn && kVariants[i].ka == pl.ka) v = &kVariants[i];
  if (!v) return hipErrorInvalidValue;
  if (p.ncols < 1 || p.ncols > p.ld || p.In < 1 || p.Ia < 1 || p.Ib < 1) return hipErrorInvalidValue;
  if ((int64_t)pl.ny * 16 * pl.wn < p.ncols) return hipErrorInvalidValue;
  if (pl.splits > 1 && !workspace) return hipErrorInvalidValue;
  MttkrpKernelArgs a;
  a.T = p.T; a.Ua = p.Ua; a.Ub = p.Ub;
  a.P = (pl.splits > 1) ? workspace : p.M;
  a.sm = p.sm; a.sa = p.sa; a.sb = p.sb;
  a.K = (int64_t)p.Ia * p.Ib; a.chunk = pl.chunk;
  a.pstride = (int64_t)p.In * p.ld;
  a.In = p.In; a.Ia = p.Ia; a.Ib = p.Ib;
  a.ncols = p.ncols; a.ld = p.ld;
  a.ntile16 = (p.ncols + 15) / 16;
  dim3 grid(pl.mtiles, pl.ny, pl.splits);
  if (ev) (void)hipEventRecord(ev[0], stream);
  hipLaunchKernelGGL((p.Ia >= pl.ka ? v->fast : v->general), grid, dim3(256), variant_lds_bytes(*v), stream, a);
  if (ev) (void)hipEventRecord(ev[1], stream);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (pl.splits > 1) {
    const int64_t n = a.pstride;
    if (ev) (void)hipEventRecord(ev[2], stream);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       (const double*)workspace, p.M, n, p.ld, p.ncols, pl.splits);
    if (ev) (void)hipEventRecord(ev[3], stream);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace cals
