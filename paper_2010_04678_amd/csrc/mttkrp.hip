// Host side of the fused multi-model MTTKRP (Eq. (2) of the paper): choice of tile shape and split of the
// contraction range, kernel launch, and the ordered reduction of the split-K partials.
#include <algorithm>
#include <cstdlib>

#include "mttkrp_kernel.h"
#include "mttkrp_rows_kernel.h"

namespace cals {

// Adds the split-K partials in a fixed order (so results are bit-reproducible): the splits are cut into G
// consecutive groups, each group is summed in split order by its own part of the workgroup, and the group sums are
// added left to right.  G = 8 (32 elements per workgroup) keeps many loads in flight and the grid several times the
// CU count even when the output is small and the split count large; with few splits fewer groups are used, so
// that every thread has loads to issue (G = 1: 256 elements per workgroup, each thread sums its element's splits).
template <int G>
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const double* __restrict__ P, double* __restrict__ M,
                                                            int64_t n_rows_ld, int ld, int ncols, int splits) {
  constexpr int E = 256 / G;     // elements per workgroup
  __shared__ double part[G][E];
  const int e = threadIdx.x % E, g = threadIdx.x / E;
  const int64_t idx = (int64_t)blockIdx.x * E + e;
  const bool live = idx < n_rows_ld && (int)(idx % ld) < ncols;
  const int per = (splits + G - 1) / G;
  const int z0 = g * per, z1 = (z0 + per < splits) ? (z0 + per) : splits;
  double s = 0.0;
  if (live) {
    const double* p = P + idx + (int64_t)z0 * n_rows_ld;
    int z = z0;
    for (; z + 4 <= z1; z += 4, p += 4 * n_rows_ld) {      // four loads in flight; added in split order
      const double v0 = p[0], v1 = p[n_rows_ld], v2 = p[2 * n_rows_ld], v3 = p[3 * n_rows_ld];
      s = (((s + v0) + v1) + v2) + v3;
    }
    for (; z < z1; ++z, p += n_rows_ld) s += *p;
  }
  if (G == 1) {
    if (live) M[idx] = s;
    return;
  }
  part[g][e] = s;
  __syncthreads();
  if (g == 0 && live) {
    double t = part[0][e];
#pragma unroll
    for (int q = 1; q < G; ++q) t += part[q][e];
    M[idx] = t;
  }
}

hipError_t launch_splitk_reduce(const double* P, double* M, int64_t n_rows_ld, int ld, int ncols, int splits, hipStream_t stream) {
  if (!P || !M || n_rows_ld < 1 || splits < 1) return hipErrorInvalidValue;
  // the group count depends on the split count alone, so a given launch shape always adds in the same order
  if (splits <= 4) {
    hipLaunchKernelGGL(splitk_reduce_kernel<1>, dim3((unsigned)((n_rows_ld + 255) / 256)), dim3(256), 0, stream, P, M, n_rows_ld, ld, ncols, splits);
  } else if (splits <= 8) {
    hipLaunchKernelGGL(splitk_reduce_kernel<2>, dim3((unsigned)((n_rows_ld + 127) / 128)), dim3(256), 0, stream, P, M, n_rows_ld, ld, ncols, splits);
  } else if (splits <= 16) {
    hipLaunchKernelGGL(splitk_reduce_kernel<4>, dim3((unsigned)((n_rows_ld + 63) / 64)), dim3(256), 0, stream, P, M, n_rows_ld, ld, ncols, splits);
  } else {
    hipLaunchKernelGGL(splitk_reduce_kernel<8>, dim3((unsigned)((n_rows_ld + 31) / 32)), dim3(256), 0, stream, P, M, n_rows_ld, ld, ncols, splits);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// variants, plan, launch
// ---------------------------------------------------------------------------------------------------

static constexpr int kMaxWnTiles = 14;

static size_t variant_lds_bytes(const Variant& v) { return (size_t)2 * v.ka * 16 * v.wn * sizeof(double); }

static const Variant* find_variant(int wm, int wn) {
  int n = 0;
  const Variant* t = (wm == 1) ? mttkrp_variants_wm1(&n) : (wm == 2 ? mttkrp_variants_wm2(&n) : (wm == 3 ? mttkrp_variants_wm3(&n) : mttkrp_variants_wm4(&n)));
  for (int i = 0; i < n; ++i)
    if (t[i].wn == wn) return &t[i];
  return nullptr;
}

hipError_t mttkrp_init() {
  // The tile kernel's variants need at most 14 x 4 KiB of dynamic LDS, within the default limit of 64 KiB: no
  // attribute to set.  The rows kernel's exchange buffers go beyond it.
  static_assert((size_t)2 * 16 * 16 * kMaxWnTiles * sizeof(double) <= 64 * 1024, "tile kernel LDS within the default limit");
  for (int grp = 0; grp < 2; ++grp) {
    int n = 0;
    const RowsVariant* t = grp == 0 ? mttkrp_rows_variants_a(&n) : mttkrp_rows_variants_b(&n);
    for (int i = 0; i < n; ++i)
      for (int m = 0; m < 2; ++m) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(t[i].fn[m]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)rows_lds_bytes(t[i].wmb, t[i].wnb));
        if (e != hipSuccess) return e;
      }
  }
  return hipSuccess;
}

static int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
}

MttkrpTuning mttkrp_tuning_from_env() {
  MttkrpTuning t;
  t.wn_max = env_int("CALS_MTTKRP_WNMAX", 0);
  t.wm = env_int("CALS_MTTKRP_WM", 0);
  t.per_cu = env_int("CALS_MTTKRP_PERCU", 0);
  t.splits = env_int("CALS_MTTKRP_SPLITS", 0);
  t.contig_u = env_int("CALS_MTTKRP_CONTIGU", -1);
  t.no_contig = env_int("CALS_MTTKRP_NOCONTIG", 0) != 0;
  t.no_rowpair = env_int("CALS_MTTKRP_NOROWPAIR", 0) != 0;
  t.no_pair = env_int("CALS_MTTKRP_NOPAIR", 0) != 0;
  t.kernel = env_int("CALS_MTTKRP_KERNEL", 0);
  t.rows_wmb = env_int("CALS_MTTKRP_ROWS_WMB", 0);
  t.rows_wnb = env_int("CALS_MTTKRP_ROWS_WNB", 0);
  t.rows_nsb = env_int("CALS_MTTKRP_ROWS_NSB", 0);
  return t;
}

// How the kernel reads the tensor along the contraction (see the mode list in mttkrp_kernel.h), and the length of
// the fast contracted index as the kernel counts it: kContig4U pads every run of Ia contiguous elements to a
// multiple of 4 positions, so the contraction range it is launched on is Ia_pad * Ib.
static int tensor_read_mode(const MttkrpProblem& p, int wm, const MttkrpTuning& tune, int* ia_counted) {
  const int ka = 16;
  *ia_counted = p.Ia;
  int mode = (p.Ia < ka) ? kGeneral : ((p.sb == (int64_t)p.Ia * p.sa) ? kAffine : kWrap);
  if (mode != kGeneral && p.sa == 1 && !tune.no_contig) {
    // rows contiguous along the contraction: four consecutive indices per lane, 16-byte loads
    if (p.Ia % 4 == 0 && p.sm % 2 == 0 && p.sb % 2 == 0 && (reinterpret_cast<uintptr_t>(p.T) & 15) == 0) return kContig4;
    // not aligned: the same layout with padded runs and shifted loads.  It pays while the launch is bound by memory
    // (999 x 1001 x 997, modes 2 and 3: 5.9 / 4.9 -> 9.5 / 9.0 TFLOP/s at 8 columns, 32 / 27 -> 39 / 38 at 48) and,
    // on tensors too large for the last-level cache, at every width (62 / 50 -> 64 / 64 at 256); small tensors at
    // larger widths are as fast or faster read element by element
    const int force = tune.contig_u;
    const double tensor_bytes = 8.0 * (double)p.In * (double)p.Ia * (double)p.Ib;
    if (force == 1 || (force != 0 && (p.ncols <= 48 || tensor_bytes > 1073741824.0))) {
      *ia_counted = (p.Ia + 3) / 4 * 4;
      return kContig4U;
    }
  }
  // rows contiguous in memory (mode 1), even row count, 16-byte aligned columns: two rows per 16-byte load
  if (mode == kAffine && p.sm == 1 && wm % 2 == 0 && p.In % 2 == 0 && p.sa % 2 == 0 && p.sb % 2 == 0 &&
      (reinterpret_cast<uintptr_t>(p.T) & 15) == 0 && !tune.no_rowpair)
    return kRowPair;
  return mode;
}

static constexpr int kMaxWn = kMaxWnTiles;     // widest column block of a workgroup, in 16-column tiles

// The plan for column blocks of at most `wn_max` tiles of 16 columns, and its modelled time in microseconds.
static MttkrpPlan plan_for_width(const MttkrpProblem& p, int num_cus, int wn_max, const MttkrpTuning& tune, double* cost_us) {
  MttkrpPlan pl{};
  const int ntile16 = (p.ncols + 15) / 16;
  // Column blocks: as few as `wn_max` allows, widths as even as possible.  Blocks of the wider and of
  // the narrower kind run as separate launches, each with the kernel of its own width, so no MFMA works on
  // padding tile columns (the tensor is read once per column block either way).
  const int ny = (ntile16 + wn_max - 1) / wn_max;
  const int base = ntile16 / ny, rem = ntile16 % ny;
  if (rem == 0) {
    pl.nparts = 1;
    pl.part[0] = MttkrpPart{base, ny, 0};
  } else {
    pl.nparts = 2;
    pl.part[0] = MttkrpPart{base + 1, rem, 0};
    pl.part[1] = MttkrpPart{base, ny - rem, rem * (base + 1) * 16};
  }
  const int wn_top = pl.part[0].wn;
  // row tiles per wavefront: as many as the accumulator budget (WM*WN <= 28 tiles) and the row count allow
  // (more row tiles per wavefront = fewer instructions per MFMA, but rows are padded to 64*wm per workgroup:
  // the choice minimises padded rows x a measured relative cost per MFMA of 1.08 / 1.25 for wm = 2 / 1; wm = 4
  // is 1.0 with up to three column tiles (up to six when the rows are contiguous in memory, i.e. mode 1 with its
  // 16-byte row-pair loads) and 1.12 beyond -- with 16 or more accumulator tiles a wavefront has no co-resident
  // to hide its waits, and 64 rows per wavefront along a long-stride mode cost more than they save: 1000^3 at
  // width 96: mode 3 57 TFLOP/s with wm = 4, 63 with wm = 2; mode 1 64 and 62)
  // Three row tiles per wavefront (192-row workgroups) are a candidate for modes read along the contraction whose
  // rows lie at most 1 MiB apart -- measured on 180^4 against one row tile per wavefront (the same 192 padded rows):
  // inner modes +10-12 % at 64 columns, +7-10 % at 128 and 256, +2-4 % at 420 in blocks of 9 tiles; the first mode
  // (rows contiguous, no row-pair loads with an odd tile count) and the last (rows 46 MB apart) gain nothing or lose
  // 2 %: relative cost 1.14.
  const bool wm3_ok = p.sa == 1 && p.sm > 1 && (double)p.sm * 8.0 <= 1048576.0;
  int wm = 1;
  {
    double best = 1e300;
    for (int cand : {4, 3, 2, 1}) {
      if (cand * wn_top > 28) continue;
      if (cand == 3 && !wm3_ok) continue;
      const double padded = (double)((p.In + 64 * cand - 1) / (64 * cand)) * (64 * cand);
      const double cost = padded * (cand == 4 ? ((wn_top <= 3 || (p.sm == 1 && wn_top <= 6)) ? 1.0 : 1.12)
                                              : (cand == 3 ? 1.14 : (cand == 2 ? 1.08 : 1.25)));
      if (cost < best) { best = cost; wm = cand; }
    }
  }
  int ia_counted = p.Ia;
  (void)tensor_read_mode(p, 2, tune, &ia_counted);
  const int64_t K = (int64_t)ia_counted * p.Ib;
  // the tensor once per column block at the practical read rate (tensors of up to 1 GiB are largely served by the
  // last-level cache: about twice the rate)
  const double tensor_bytes = (double)p.In * (double)K * 8.0;
  const double tensor_us = tensor_bytes / (tensor_bytes > 1073741824.0 ? 5.5e6 : 11.0e6);
  // Bandwidth-bound launches (few columns): four row tiles per wavefront keep four times the tensor loads in flight
  // per wavefront and allow 16-byte loads along contiguous rows, which outweighs the padding of the row count to
  // 256 as long as the MFMA work on the padded rows stays well below the time the tensor takes to stream.
  if (wm != 4 && wn_top <= 7) {
    const double padded4 = (double)((p.In + 255) / 256) * 256.0;
    const double mfma4_us = 2.0 * padded4 * (double)K * 16.0 * ntile16 / (78.6e6 * 0.8);
    if (mfma4_us < 0.6 * tensor_us * ny) wm = 4;
  }
  if (tune.wm > 0) wm = tune.wm;
  if (wm < 1 || wm > 4) wm = 2;
  if (wm == 4 && wn_top > 7) wm = 2;
  if (wm == 3 && wn_top > 9) wm = 2;
  pl.wm = wm;
  pl.ka = 16;
  pl.mtiles = (p.In + 64 * wm - 1) / (64 * wm);
  // resident workgroups per CU: bounded by registers (accumulators) and LDS
  const int acc_tiles = wm * wn_top;
  int per_cu = (acc_tiles >= 17) ? 1 : (acc_tiles >= 10 ? 2 : (acc_tiles >= 8 ? 3 : 4));
  // one row tile per wavefront with 12 or more column tiles: the B fragments and the factor rows in flight take
  // so many registers next to the accumulators that only one workgroup fits (compiler's resource report)
  if (wm == 1 && wn_top >= 12) per_cu = 1;
  // three row tiles per wavefront: the tensor fragments of three tiles in flight leave room for two workgroups up to
  // five column tiles (compiler's resource report)
  if (wm == 3 && per_cu > 2) per_cu = (wn_top <= 1) ? 3 : 2;
  const int lds_fit = (int)(160 * 1024 / ((size_t)2 * pl.ka * 16 * wn_top * sizeof(double)));
  if (per_cu > lds_fit) per_cu = lds_fit;
  if (tune.per_cu > 0) per_cu = tune.per_cu;
  // Split of the contraction range, by a cost model in microseconds.  A stage of a workgroup with t accumulator
  // tiles per wavefront takes t x 4 MFMAs x 64 cycles at about 80 % MFMA utilisation, plus a fixed cost of about 6
  // stages per workgroup.  More than one split adds the partials' way through memory (below).  For a tensor that
  // streams from HBM the candidates are 1..7 and the multiples of 8, so that the XCD-pinned block order gives every
  // XCD the same number of splits and the column blocks of a split share the tensor tile in that XCD's L2.  A tensor
  // that the last-level cache holds does not need that, and what decides there is how evenly the workgroups fill
  // the compute units, so every split count is a candidate (300 x 300 x 40 at 630 columns, modes 1 and 2: 16 splits
  // = 400 workgroups 36-40 TFLOP/s, 20 splits = 500 workgroups 46-47; 300^3 at 420 columns 48 -> 51 splits +4 %;
  // 4000 x 200 x 50 at 640 columns, mode 2, 48 -> 51 splits +6 %); splits that are not a multiple of 8 are spread
  // over the XCDs.
  const int64_t max_splits = std::max<int64_t>(1, K / (4 * pl.ka));   // at least two stage pairs per split
  const int force_splits = tune.splits;
  const double us_per_tile_stage = 4.0 * 64.0 / 2400.0 / 0.8;          // one accumulator tile, one stage (KA = 16)
  // One In x ncols panel of partial sums: written by the contraction (mostly hidden behind its MFMAs: 4000 x 200 x 50
  // mode 1 at 640 columns, 20 MB panels, 24 -> 128 splits: 0.80 -> 0.98 ms), read once by the reduction kernel, which
  // measured takes about 5 us plus the bytes at 4-5 TB/s, or at 8 TB/s while all panels together stay in the caches.
  const double panel_bytes = (double)p.In * p.ncols * 8.0;
  // the practical read rate needs enough loads in flight: two workgroups per CU with four row tiles per wavefront,
  // three with two, four with one; and the workgroups share the bandwidth, so a launch lasts about as long as the
  // CU with the most of them
  const int64_t wgs_for_rate = (int64_t)num_cus * (wm == 4 ? 2 : (wm >= 2 ? 3 : 4));
  int64_t splits = 1;
  double best_cost = 1e300;
  const bool cache_resident = tensor_bytes <= 1073741824.0;
  auto next_candidate = [cache_resident](int64_t c) -> int64_t {
    if (!cache_resident) return c < 8 ? c + 1 : c + 8;
    return c < 64 ? c + 1 : (c < 128 ? c + 2 : c + 8);
  };
  for (int64_t cand = 1; cand <= std::min<int64_t>(max_splits, 4096); cand = next_candidate(cand)) {
    const int64_t pairs = (K + cand * 2 * pl.ka - 1) / (cand * 2 * pl.ka);
    double cost = 0.0;
    for (int q = 0; q < pl.nparts; ++q) {
      const int64_t wgs = (int64_t)pl.mtiles * pl.part[q].ny * cand;
      // The workgroups of a CU share its MFMA pipes whether they are resident together or one after the other, so
      // the busiest CU sets the time; co-residents hide each other's fixed cost and, for small tiles, each other's
      // non-MFMA instructions (measured: one / two / three resident workgroups of up to 9 accumulator tiles reach
      // 0.87 / 0.96 / 1 of the three-resident rate, of 10 to 16 tiles 0.92 / 1; 17 and more tiles leave room for one
      // workgroup only: 0.93 -- 1000^3 at width 512 runs at 62 TFLOP/s in blocks of 11 tiles, at 67 in blocks of 8).
      const int64_t on_cu = (wgs + num_cus - 1) / num_cus;
      const int resident = (int)std::min<int64_t>(per_cu, on_cu);
      const double overlap = (acc_tiles >= 17 || per_cu == 1) ? 0.93
                             : (acc_tiles >= 10 ? (resident >= 2 ? 1.0 : 0.92)
                                                : (resident >= 3 ? 1.0 : (resident == 2 ? 0.96 : 0.87)));
      const double mfma_us = (double)on_cu * (2.0 * pairs + 6.0 / resident) * us_per_tile_stage * wm * pl.part[q].wn / overlap;
      double fill = wgs >= wgs_for_rate ? 1.0 : (double)wgs_for_rate / (double)wgs;
      fill *= (double)((wgs + num_cus - 1) / num_cus * num_cus) / (double)wgs;
      const double hbm_us = tensor_us * pl.part[q].ny * fill;
      cost += mfma_us > hbm_us ? mfma_us : hbm_us;
    }
    if (cand > 1)
      cost += 5.0 + (double)(cand + 1) * panel_bytes / ((double)cand * panel_bytes <= 64.0e6 ? 8.0e6 : 4.5e6) + (double)cand * panel_bytes / 1.2e7;
    if (cost < best_cost) { best_cost = cost; splits = cand; }
  }
  if (force_splits > 0) splits = force_splits;
  int64_t chunk = (K + splits - 1) / splits;
  chunk = (chunk + 2 * pl.ka - 1) / (2 * pl.ka) * (2 * pl.ka);   // whole stage pairs
  splits = (K + chunk - 1) / chunk;
  pl.splits = (int)splits;
  pl.chunk = chunk;
  pl.workspace_bytes = (pl.splits > 1) ? (size_t)pl.splits * p.In * p.ld * sizeof(double) : 0;
  pl.read_mode = tensor_read_mode(p, pl.wm, tune, &pl.ia_counted);
  // factor rows 16-byte aligned: two columns per lane in the Khatri-Rao tile production
  pl.pair = (p.ld % 2 == 0 && ((reinterpret_cast<uintptr_t>(p.Ua) | reinterpret_cast<uintptr_t>(p.Ub)) & 15) == 0 && !tune.no_pair) ? 1 : 0;
  pl.kind = 0;
  pl.cost_us = best_cost;
  *cost_us = best_cost;
  return pl;
}

static MttkrpPlan tile_plan(const MttkrpProblem& p, int num_cus, const MttkrpTuning& tune) {
  // tuning knob (development aid): widest column block
  const int forced = tune.wn_max;
  double cost = 0.0;
  if (forced > 0) return plan_for_width(p, num_cus, forced > kMaxWn ? kMaxWn : forced, tune, &cost);
  // Column blocks of up to 14 tiles read the tensor the fewest times; blocks of up to 8 tiles leave room for a second
  // workgroup on the CU, which hides waits and barriers (worth it from about 12 tiles of width on: measured +2 % at
  // 192 columns, +4 % at 320-384, +6-8 % at 512-1024 on 1000^3; +13 % at 420 on 60^5, where the model sees a tie).
  // The modelled time decides -- it charges the extra passes over the tensor -- and near-ties go to the narrow blocks.
  MttkrpPlan wide = plan_for_width(p, num_cus, kMaxWn, tune, &cost);
  if ((p.ncols + 15) / 16 >= 12) {
    double cost8 = 0.0;
    MttkrpPlan narrow = plan_for_width(p, num_cus, 8, tune, &cost8);
    if (narrow.wm == 3) {
      // three row tiles per wavefront take blocks of up to 9 tiles (420 columns as 9+9+9 instead of 7+7+7+6: one
      // launch and one pass over the tensor fewer; 180^4 inner modes 59.2 / 58.2 -> 60.6 / 59.9 TFLOP/s)
      double cost9 = 0.0;
      const MttkrpPlan nine = plan_for_width(p, num_cus, 9, tune, &cost9);
      if (nine.wm == 3 && cost9 <= cost8) { narrow = nine; cost8 = cost9; }
    }
    if (cost8 <= 1.02 * cost) return narrow;
  }
  return wide;
}

// ---------------------------------------------------------------------------------------------------
// rows kernel: plan and launch
// ---------------------------------------------------------------------------------------------------

static const RowsVariant* find_rows_variant(int wmb, int wnb) {
  for (int grp = 0; grp < 2; ++grp) {
    int n = 0;
    const RowsVariant* t = grp == 0 ? mttkrp_rows_variants_a(&n) : mttkrp_rows_variants_b(&n);
    for (int i = 0; i < n; ++i)
      if (t[i].wmb == wmb && t[i].wnb == wnb) return &t[i];
  }
  return nullptr;
}

// Which way the rows kernel can read this problem's tensor, or -1 when it cannot take the problem at all: it needs a
// fast contracted index whose length is a multiple of 4 and at least a stage (a lane's 4 indices then share the slow
// index), 16-byte aligned factor rows, and one of its two aligned tensor layouts.
static int rows_read_mode(const MttkrpProblem& p, const MttkrpTuning& tune) {
  if (p.Ia < 16 || p.Ia % 4 != 0 || p.ld % 2 != 0 || tune.no_pair) return -1;
  if (((reinterpret_cast<uintptr_t>(p.Ua) | reinterpret_cast<uintptr_t>(p.Ub) | reinterpret_cast<uintptr_t>(p.T)) & 15) != 0) return -1;
  if (p.sa == 1 && p.sm % 2 == 0 && p.sb % 2 == 0 && !tune.no_contig) return kRowsContig;
  if (p.sm == 1 && p.sb == (int64_t)p.Ia * p.sa && p.In % 2 == 0 && p.sa % 2 == 0 && !tune.no_rowpair) return kRowsPair;
  return -1;
}

// The best launch of the rows kernel for the problem by modelled time, or false when no variant can take it.
static bool rows_plan(const MttkrpProblem& p, int num_cus, const MttkrpTuning& tune, MttkrpPlan* out) {
  const int amode = rows_read_mode(p, tune);
  if (amode < 0) return false;
  const int64_t K = (int64_t)p.Ia * p.Ib;
  const int tiles_m = (p.In + 15) / 16, tiles_n = (p.ncols + 15) / 16;
  const double tensor_bytes = (double)p.In * (double)K * 8.0;
  const double hbm_us = tensor_bytes / (tensor_bytes > 1073741824.0 ? 5.5e6 : 11.0e6);
  const double panel_us = (double)p.In * p.ncols * 8.0 / 3.0e6;
  bool found = false;
  MttkrpPlan best{};
  best.cost_us = 1e300;
  for (int grp = 0; grp < 2; ++grp) {
    int nv = 0;
    const RowsVariant* tab = grp == 0 ? mttkrp_rows_variants_a(&nv) : mttkrp_rows_variants_b(&nv);
    for (int i = 0; i < nv; ++i) {
      const int wmb = tab[i].wmb, wnb = tab[i].wnb;
      if ((tune.rows_wmb > 0 && wmb != tune.rows_wmb) || (tune.rows_wnb > 0 && wnb != tune.rows_wnb)) continue;
      // row blocks: as few as the variant allows, of equal size (an even number of tiles when rows are read in pairs
      // and there is more than one block)
      int nrb = (tiles_m + wmb - 1) / wmb, tpb = 0;
      for (;; ++nrb) {
        tpb = (tiles_m + nrb - 1) / nrb;
        if (amode == kRowsPair && nrb > 1 && tpb % 2 == 1) ++tpb;
        if (tpb <= wmb) break;
      }
      nrb = (tiles_m + tpb - 1) / tpb;
      // Measured against the tile kernel in steady state (thirteen shapes from 100^3 to 1000^3, widths 16 to 1024,
      // every mode).  Tensors the last-level cache holds (up to 256 MiB): the modelled times of the two kernels pick
      // the faster one, or one within a few per cent of it, in nearly every case (mean loss 0.8 %), so nothing else
      // is asked -- except of launches of a few microseconds (32^3), which stay with the tile kernel.  Larger tensors:
      // only a row block that holds the whole mode and leaves at most a sixth of the variant's row tiles empty
      // (4000 x 200 x 50, mode 2: 13 row tiles in one block 2-13 % faster than the tile kernel at 33 of 35 widths from
      // 96 to 640, two blocks of 7 up to 12 % slower); every column group reads the whole tensor, which the model
      // charges: 500^3, 180 x 180 x 2000 and 1000^3 are 5 to 40 % slower with this kernel at every width.
      const bool forced = tune.kernel == 2;
      const bool cache_resident = tensor_bytes <= 268435456.0;
      if (!forced && (double)p.In * (double)K * p.ncols < (cache_resident ? 1.0e7 : 1.0e8)) continue;
      if (!forced && !cache_resident && (nrb != 1 || 6 * tiles_m < 5 * wmb)) continue;
      // column groups of wnb tiles, some of wnb - 1
      const int ncg = (tiles_n + wnb - 1) / wnb;
      const int fewer = ncg * wnb - tiles_n;
      if (fewer > ncg || (wnb == 1 && fewer > 0)) continue;
      // Workgroup-level splits by modelled time.  A wavefront's stage is wmb x wnb accumulator tiles (all of the
      // variant's row tiles are computed, live or not) x 4 matrix instructions of 64 cycles, at the 72 % of the issue
      // rate these kernels reach; a workgroup pays a fixed 3 us (first loads, the exchange of the four accumulator
      // sets, stores); compute units take workgroups in rounds.  Every column group reads the whole tensor: measured,
      // the groups together draw about 6 TB/s from the caches behind L1 (200^3 at 7 groups: 81 us; 4000x200x50,
      // mode 2, at 4 / 11 / 20 groups: 195 / 709 / 1168 us), which bounds wide launches.
      const double stage_us = (double)wmb * wnb * 4.0 * 64.0 / 2400.0 / 0.72;
      const int64_t max_nsb = std::max<int64_t>(1, K / 128);     // at least two stages per wavefront
      for (int64_t nsb = 1; nsb <= std::min<int64_t>(max_nsb, 2048); nsb = nsb < 16 ? nsb + 1 : nsb + (nsb < 64 ? 2 : 8)) {
        if (tune.rows_nsb > 0 && nsb != tune.rows_nsb && nsb != 1) continue;
        if (tune.rows_nsb > 0 && nsb == 1 && tune.rows_nsb != 1) continue;
        int64_t chunk = (K + 4 * nsb - 1) / (4 * nsb);
        chunk = (chunk + 15) / 16 * 16;
        const int64_t nsb_eff = (K + 4 * chunk - 1) / (4 * chunk);
        // (row block, split) pairs go to the 8 XCDs in turn, each with all its column groups; a workgroup has a
        // compute unit to itself, so the busiest XCD sets the number of rounds (200^3 at 192 columns: 42 splits x 6
        // groups put 36 workgroups on two XCDs of 32 compute units and took 119 us; 40 splits take 77)
        const int64_t per_xcd = ((int64_t)nrb * nsb_eff + 7) / 8 * ncg;
        const int64_t cus_per_xcd = std::max<int64_t>(1, num_cus / 8);
        const int64_t rounds = (per_xcd + cus_per_xcd - 1) / cus_per_xcd;
        const double compute_us = (double)rounds * ((double)(chunk / 16) * stage_us + 3.0);
        const double mem_us = std::max(hbm_us, (double)ncg * tensor_bytes / 6.0e6);
        double cost = std::max(compute_us, mem_us);
        if (nsb_eff > 1) cost += (double)(nsb_eff + 1) * panel_us + 3.0;
        if (cost < best.cost_us) {
          found = true;
          best.cost_us = cost;
          best.kind = 1;
          best.rows_wmb = wmb; best.rows_wnb = wnb; best.rows_amode = amode; best.rows_tpb = tpb;
          best.rows_nrb = nrb; best.rows_ncg = ncg; best.rows_rem = ncg - fewer;
          best.splits = (int)nsb_eff;
          best.chunk = chunk;
          best.workspace_bytes = nsb_eff > 1 ? (size_t)nsb_eff * p.In * p.ld * sizeof(double) : 0;
        }
      }
    }
  }
  if (found) *out = best;
  return found;
}

MttkrpPlan mttkrp_plan(const MttkrpProblem& p, int num_cus, const MttkrpTuning& tune) {
  MttkrpPlan tiles = tile_plan(p, num_cus, tune);
  if (tune.kernel == 1) return tiles;
  MttkrpPlan rows{};
  if (!rows_plan(p, num_cus, tune, &rows)) return tiles;
  if (tune.kernel == 2) return rows;
  return rows.cost_us < tiles.cost_us ? rows : tiles;
}

// Records a timing event; a failed record only marks the launch as untimed (the error is cleared, the work goes on).
static inline void record_event(hipEvent_t* ev, int i, hipStream_t stream, bool* timed) {
  if (!ev) return;
  if (hipEventRecord(ev[i], stream) != hipSuccess) {
    (void)hipGetLastError();
    *timed = false;
  }
}

static hipError_t rows_launch(const MttkrpProblem& p, const MttkrpPlan& pl, double* workspace, hipStream_t stream,
                              hipEvent_t* ev, bool* timed) {
  const RowsVariant* v = find_rows_variant(pl.rows_wmb, pl.rows_wnb);
  if (!v || (pl.rows_amode != kRowsContig && pl.rows_amode != kRowsPair)) return hipErrorInvalidValue;
  // what the kernel assumes about its operands
  if (p.Ia < 16 || p.Ia % 4 != 0 || p.ld % 2 != 0) return hipErrorInvalidValue;
  if (((reinterpret_cast<uintptr_t>(p.Ua) | reinterpret_cast<uintptr_t>(p.Ub) | reinterpret_cast<uintptr_t>(p.T)) & 15) != 0) return hipErrorInvalidValue;
  if (pl.rows_amode == kRowsContig && (p.sa != 1 || p.sm % 2 != 0 || p.sb % 2 != 0)) return hipErrorInvalidValue;
  if (pl.rows_amode == kRowsPair && (p.sm != 1 || p.sb != (int64_t)p.Ia * p.sa || p.In % 2 != 0 || p.sa % 2 != 0)) return hipErrorInvalidValue;
  const int64_t K = (int64_t)p.Ia * p.Ib;
  if (pl.rows_tpb < 1 || pl.rows_tpb > pl.rows_wmb || (int64_t)pl.rows_nrb * pl.rows_tpb * 16 < p.In) return hipErrorInvalidValue;
  if (pl.rows_amode == kRowsPair && pl.rows_nrb > 1 && pl.rows_tpb % 2 != 0) return hipErrorInvalidValue;
  if (pl.rows_rem < 0 || pl.rows_rem > pl.rows_ncg || (pl.rows_wnb == 1 && pl.rows_rem != pl.rows_ncg)) return hipErrorInvalidValue;
  if (16 * (pl.rows_rem * pl.rows_wnb + (pl.rows_ncg - pl.rows_rem) * (pl.rows_wnb - 1)) < p.ncols) return hipErrorInvalidValue;
  if (pl.chunk < 16 || pl.chunk % 16 != 0 || pl.chunk >= (1LL << 31) || (int64_t)pl.splits * 4 * pl.chunk < K) return hipErrorInvalidValue;
  if (pl.splits > 1 && !workspace) return hipErrorInvalidValue;
  RowsKernelArgs a;
  a.T = p.T; a.Ua = p.Ua; a.Ub = p.Ub;
  a.P = pl.splits > 1 ? workspace : p.M;
  a.sm = p.sm; a.sa = p.sa; a.sb = p.sb;
  a.K = K; a.chunk = pl.chunk;
  a.pstride = (int64_t)p.In * p.ld;
  a.In = p.In; a.Ia = p.Ia; a.Ib = p.Ib; a.ncols = p.ncols; a.ld = p.ld;
  a.nrb = pl.rows_nrb; a.ncg = pl.rows_ncg; a.nsb = pl.splits; a.tpb = pl.rows_tpb;
  a.col0 = 0; a.rem = pl.rows_rem;
  const int64_t groups = ((int64_t)a.nrb * a.nsb + 7) / 8 * 8;
  const int64_t nblocks = groups * a.ncg;
  if (nblocks >= (1LL << 31)) return hipErrorInvalidValue;
  record_event(ev, 0, stream, timed);
  hipLaunchKernelGGL(v->fn[pl.rows_amode], dim3((unsigned)nblocks), dim3(256), rows_lds_bytes(v->wmb, v->wnb), stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  record_event(ev, 1, stream, timed);
  if (pl.splits > 1) {
    record_event(ev, 2, stream, timed);
    e = launch_splitk_reduce(workspace, p.M, a.pstride, p.ld, p.ncols, pl.splits, stream);
    record_event(ev, 3, stream, timed);
  }
  return e;
}

hipError_t mttkrp_launch(const MttkrpProblem& p, const MttkrpPlan& pl, double* workspace, hipStream_t stream,
                         hipEvent_t* ev, bool* timed_out) {
  bool timed_local = true;
  bool* timed = timed_out ? timed_out : &timed_local;
  *timed = (ev != nullptr);
  if (p.ncols < 1 || p.ncols > p.ld || p.In < 1 || p.Ia < 1 || p.Ib < 1) return hipErrorInvalidValue;
  if (pl.kind == 1) return rows_launch(p, pl, workspace, stream, ev, timed);
  if (pl.nparts < 1 || pl.nparts > 2) return hipErrorInvalidValue;
  if ((int64_t)pl.mtiles * 64 * pl.wm < p.In) return hipErrorInvalidValue;
  const int ia_counted = pl.ia_counted;
  const int mode = pl.read_mode;
  if (mode < kAffine || mode > kContig4U || ia_counted < p.Ia || ia_counted > p.Ia + 3) return hipErrorInvalidValue;
  if (pl.ka != 16) return hipErrorInvalidValue;
  if (pl.chunk % pl.ka != 0 || (int64_t)pl.splits * pl.chunk < (int64_t)ia_counted * p.Ib) return hipErrorInvalidValue;
  if (pl.splits > 1 && !workspace) return hipErrorInvalidValue;
  if (!p.zeros || (reinterpret_cast<uintptr_t>(p.zeros) & 15)) return hipErrorInvalidValue;
  // the parts tile the columns without gaps
  int covered = 0;
  for (int q = 0; q < pl.nparts; ++q) {
    if (pl.part[q].col0 != covered || pl.part[q].wn < 1 || pl.part[q].ny < 1) return hipErrorInvalidValue;
    covered += 16 * pl.part[q].wn * pl.part[q].ny;
  }
  if (covered < p.ncols) return hipErrorInvalidValue;
  MttkrpKernelArgs a;
  a.T = p.T; a.Ua = p.Ua; a.Ub = p.Ub; a.zeros = p.zeros;
  a.P = (pl.splits > 1) ? workspace : p.M;
  a.sm = p.sm; a.sa = p.sa; a.sb = p.sb;
  a.K = (int64_t)ia_counted * p.Ib; a.chunk = pl.chunk;
  a.pstride = (int64_t)p.In * p.ld;
  a.In = p.In; a.Ia = ia_counted; a.Iav = p.Ia; a.Ib = p.Ib;
  a.ncols = p.ncols; a.ld = p.ld;
  a.mtiles = pl.mtiles; a.splits = pl.splits;
  a.pinned = (pl.splits % 8 == 0) ? 1 : 0;
  const int pair = pl.pair ? 1 : 0;
  record_event(ev, 0, stream, timed);
  for (int q = 0; q < pl.nparts; ++q) {
    const Variant* v = find_variant(pl.wm, pl.part[q].wn);
    if (!v || v->ka != pl.ka) return hipErrorInvalidValue;
    a.ny = pl.part[q].ny;
    a.col0 = pl.part[q].col0;
    // 1-D grid, decoded in the kernel: 8 interleaved sequences (one per XCD) of whole splits
    const int64_t nblocks = (int64_t)pl.mtiles * a.ny * pl.splits;
    if (nblocks >= (1LL << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(v->fn[mode][pair], dim3((unsigned)nblocks), dim3(256), variant_lds_bytes(*v), stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  record_event(ev, 1, stream, timed);
  hipError_t e = hipSuccess;
  if (pl.splits > 1) {
    const int64_t n = a.pstride;
    record_event(ev, 2, stream, timed);
    e = launch_splitk_reduce(workspace, p.M, n, p.ld, p.ncols, pl.splits, stream);
    record_event(ev, 3, stream, timed);
  }
  return e;
}

}  // namespace cals
