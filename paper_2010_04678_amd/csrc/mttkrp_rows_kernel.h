// Second kernel of the fused multi-model MTTKRP (Eq. (2) of the paper) for gfx950, for output modes with few rows:
//   M[m, c] = sum_{ia, ib} T[m, ia, ib] * (Ua[ia, c] * Ub[ib, c])      for every fused column c.
//
// The tile kernel (mttkrp_kernel.h) gives each wavefront a band of 16*WM rows and pads the row count to 64*WM per
// workgroup; on modes of 40, 50, 180, 200 or 300 rows a large part of its matrix instructions works on padding, and
// with one row tile per wavefront every B fragment read from LDS feeds a single instruction.  Here the roles are
// turned round:
//   - a wavefront owns ALL row tiles of its row block (up to WMB tiles of 16 rows, the live ones only) and a narrow
//     group of WNB column tiles; one B value feeds up to WMB matrix instructions;
//   - the B operand of v_mfma_f64_16x16x4_f64 is one value per lane, Ua[ia(k), c] * Ub[ib(k), c] for the lane's own
//     (k, c): the lane loads its two factors itself (buffer loads, one stage ahead; the factor panels live in L2)
//     and multiplies -- the Khatri-Rao product never exists anywhere, not even as an LDS tile, and the main loop has
//     no barrier and no LDS access at all;
//   - the four wavefronts of a workgroup work on the SAME output tiles over four consecutive quarters of the
//     workgroup's share of the contraction range, and add their accumulators through LDS in wavefront order before
//     one partial panel is written: four times fewer split-K partials than one panel per wavefront;
//   - workgroups that differ only in their column group read the same tensor fragments; the block order keeps them
//     on one XCD, next to each other, so that they share its L2.
// Tensor fragments go from global memory straight into the MFMA register layout, a lane owning 4 consecutive
// contraction indices per stage of 16 (k-step s uses element s): two 16-byte loads per row tile and stage when the
// contraction is contiguous in memory, one 16-byte load per pair of row tiles and index when the rows are.  The
// fragments of a row tile for the next stage are requested right after the tile's matrix instructions of this stage
// have been issued, into the same registers.
#pragma once
#include "mttkrp_kernel.h"

namespace cals {

struct RowsKernelArgs {
  const double* T;
  const double* Ua;   // row-major Ia x ld
  const double* Ub;   // row-major Ib x ld
  double* P;          // output: partial panels [nsb][In][ld], or M itself when nsb == 1
  int64_t sm, sa, sb; // element strides of T: output row, fast contracted index, slow contracted index
  int64_t K, chunk;   // contraction length Ia*Ib; indices per wavefront (multiple of 16)
  int64_t pstride;    // In * ld
  int In, Ia, Ib;     // Ia is a multiple of 4 and at least 16
  int ncols, ld;      // ld even, Ua and Ub 16-byte aligned
  int nrb, ncg, nsb;  // row blocks, column groups, workgroup-level splits of the contraction range
  int tpb;            // row tiles per row block (<= WMB; even for kRowsPair unless there is one row block)
  int col0;           // first column of column group 0
  int rem;            // the first `rem` column groups have WNB column tiles, the others WNB-1
};

// How the tensor is read:
//   kRowsContig: sa == 1, 16-byte aligned rows (modes 2 .. N of aligned tensors): a lane's 4 indices are contiguous
//   kRowsPair  : sm == 1, even row count, offsets affine in k (sb == Ia*sa), 16-byte aligned columns (mode 1): a lane
//                reads two adjacent rows per load; row tile 2p holds the even and 2p+1 the odd rows of the p-th
//                group of 32 rows (an odd last row tile is read row by row)
enum { kRowsContig = 0, kRowsPair = 1 };

// LDS of the final in-workgroup reduction: rounds of TH accumulator tiles, 4 wavefronts x 2 KiB per tile.
constexpr int rows_reduce_tiles(int tot) { return tot <= 19 ? tot : (tot + 1) / 2; }
constexpr size_t rows_lds_bytes(int wmb, int wnb) { return (size_t)rows_reduce_tiles(wmb * wnb) * 4 * 2048; }

template <int WMB, int WNB, int LC, int AMODE>
__device__ __forceinline__ void rows_body(const RowsKernelArgs& a, double* smem, int g, int cg) {
  constexpr int NPC = LC / 2;                    // pairs of column tiles (16-byte factor loads, columns interleaved)
  constexpr int SGC = LC % 2;                    // a last single column tile (8-byte factor loads)
  constexpr bool RP = (AMODE == kRowsPair);
  constexpr int NPR = RP ? WMB / 2 : 0;          // pairs of row tiles
  constexpr bool SGR = RP && (WMB % 2 == 1);     // kRowsPair: a last single row tile

  const int rb = g % a.nrb, zb = g / a.nrb;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lq = lane >> 4;
  const int m0 = rb * (16 * a.tpb);
  const int n0 = a.col0 + 16 * (cg < a.rem ? cg * WNB : a.rem * WNB + (cg - a.rem) * (WNB - 1));
  const int rows_left = a.In - m0;               // >= 1
  const int lt = (rows_left + 15) / 16 < a.tpb ? (rows_left + 15) / 16 : a.tpb;  // live row tiles
  // kRowsPair: live pairs of row tiles (an odd tile count below WMB rounds up: the half-empty pair's rows are masked;
  // at tpb == WMB odd the last tile is the single one)
  const int pairs_max = (a.tpb + 1) / 2 < NPR ? (a.tpb + 1) / 2 : NPR;
  const int lp = (rows_left + 31) / 32 < pairs_max ? (rows_left + 31) / 32 : pairs_max;
  const bool single_live = SGR && a.tpb == WMB && rows_left > 32 * NPR;
  const int64_t kb = ((int64_t)zb * 4 + wave) * a.chunk;
  const int64_t ke = (kb + a.chunk < a.K) ? (kb + a.chunk) : a.K;
  const int nstage = (kb < ke) ? (int)((ke - kb + 15) / 16) : 0;
  const int Ia = a.Ia;

  double4_t acc[WMB][LC];
#pragma unroll
  for (int t = 0; t < WMB; ++t)
#pragma unroll
    for (int j = 0; j < LC; ++j) acc[t][j] = double4_t{0.0, 0.0, 0.0, 0.0};

  // (No branch around the main part for a wavefront without work: with nstage == 0 the prologue reads valid addresses
  // and the loop does not run.  A branch here makes the register allocator keep the accumulators in vector registers
  // and copy all of them in and out of the accumulation registers around every tile.)
  {
    // ---- this lane's first contraction index, and whether it has any (the last wavefront of the range may be short)
    const int64_t k0 = kb + 4 * lq;              // kb, ke and Ia are multiples of 4: the lane's 4 indices share ib
    const bool live0 = k0 < ke;
    const int64_t kk = live0 ? k0 : 0;           // a lane without work keeps reading valid addresses; its B is zero
    const int64_t ib0 = kk / Ia;
    const int ia0 = (int)(kk - ib0 * Ia);

    // ---- tensor fragments.  cursor: where the next loads read; advanced by 16 indices per stage while the lane has
    // work left, otherwise left where it is (every address stays inside the tensor).
    const int64_t a_wrap = a.sb - (int64_t)Ia * a.sa;    // added when ia wraps (zero for affine offsets)
    const double* Pt[RP ? (NPR + 1) : WMB];
    if constexpr (RP) {
#pragma unroll
      for (int p = 0; p < NPR; ++p) {
        const int r = m0 + 32 * p + 2 * li;
        Pt[p] = a.T + (int64_t)(r < a.In ? r : a.In - 2) + kk * a.sa;
      }
      const int r = m0 + 32 * NPR + li;
      Pt[NPR] = a.T + (int64_t)(r < a.In ? r : a.In - 1) + kk * a.sa;
    } else {
#pragma unroll
      for (int t = 0; t < WMB; ++t) {
        const int r = m0 + 16 * t + li;
        Pt[t] = a.T + (int64_t)(r < a.In ? r : a.In - 1) * a.sm + (int64_t)ia0 * a.sa + ib0 * a.sb;
      }
    }
    int a_ia = ia0;
    int a_left = live0 ? (int)(ke - k0) : 0;     // indices from the cursor to the end of the range (<= chunk < 2^31)
    int64_t a_inc = 0;                           // what the cursor moves by after the loads in progress

    double areg[WMB][4];
    auto plan_a_advance = [&]() {
      const int left = a_left - 16;
      const bool go = left > 0;
      int ia = a_ia + 16;
      const bool wrap = ia >= Ia;
      ia = wrap ? ia - Ia : ia;
      a_inc = go ? (16 * a.sa + (wrap ? a_wrap : 0)) : 0;
      a_ia = go ? ia : a_ia;
      a_left = left;
    };
    auto load_tile = [&](int t) {                // kRowsContig: tile t
      const double2 v01 = *reinterpret_cast<const double2*>(Pt[t]);
      const double2 v23 = *reinterpret_cast<const double2*>(Pt[t] + 2);
      areg[t][0] = v01.x; areg[t][1] = v01.y; areg[t][2] = v23.x; areg[t][3] = v23.y;
      Pt[t] += a_inc;
    };
    auto load_pair = [&](int p) {                // kRowsPair: tiles 2p (even rows) and 2p+1 (odd rows)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const double2 v = *reinterpret_cast<const double2*>(Pt[p] + s * a.sa);
        areg[2 * p][s] = v.x;
        areg[2 * p + (WMB > 1 ? 1 : 0)][s] = v.y;
      }
      Pt[p] += a_inc;
    };
    auto load_single = [&]() {                   // kRowsPair: the odd last tile, one row per lane
#pragma unroll
      for (int s = 0; s < 4; ++s) areg[WMB - 1][s] = *(Pt[NPR] + s * a.sa);
      Pt[NPR] += a_inc;
    };

    // ---- factors.  A lane's B value for tile j and k-step s is Ua[ia + s, c] * Ub[ib, c] with its own column c:
    // columns 2*li, 2*li+1 of a 32-column group feed a pair of column tiles (one 16-byte load per factor row), a last
    // single tile takes column li of its 16.  Lanes without work read "out of range" and receive zeros from Ub.
    const unsigned row_bytes = 8u * (unsigned)a.ld;
    const __amdgpu_buffer_rsrc_t rsrc_a = factor_rsrc(a.Ua, row_bytes * (unsigned)a.Ia);   // < 2^32 (checked on the host)
    const __amdgpu_buffer_rsrc_t rsrc_b = factor_rsrc(a.Ub, row_bytes * (unsigned)a.Ib);
    unsigned cbp[NPC > 0 ? NPC : 1], cbs = 0;
#pragma unroll
    for (int q = 0; q < NPC; ++q) {
      const int gc = n0 + 32 * q + 2 * li;
      cbp[q] = 8u * (unsigned)(gc <= a.ld - 2 ? gc : a.ld - 2);   // columns past the matrix: any valid pair (never stored)
    }
    if (SGC) {
      const int gc = n0 + 32 * NPC + li;
      cbs = 8u * (unsigned)(gc <= a.ld - 1 ? gc : a.ld - 1);
    }
    const unsigned wrap_a = row_bytes * (unsigned)Ia;
    unsigned u_oa = (unsigned)ia0 * row_bytes, u_ob = (unsigned)ib0 * row_bytes;
    int u_left = a_left;
    const int rb1 = __builtin_amdgcn_readfirstlane((int)row_bytes);
    double uar[4][LC], ubr[LC], breg[4][LC];
    auto load_factors = [&]() {
      const bool dead = u_left <= 0;
      constexpr unsigned kBeyond = 0xffffff00u;                   // beyond every descriptor's range: reads as zero
#pragma unroll
      for (int q = 0; q < NPC; ++q) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const double2 v = buffer_load_f64x2(rsrc_a, u_oa + cbp[q], (unsigned)(s * rb1));
          uar[s][2 * q] = v.x;
          uar[s][2 * q + (LC > 1 ? 1 : 0)] = v.y;
        }
        const double2 w = buffer_load_f64x2(rsrc_b, dead ? kBeyond : (u_ob + cbp[q]), 0u);
        ubr[2 * q] = w.x;
        ubr[2 * q + (LC > 1 ? 1 : 0)] = w.y;
      }
      if (SGC) {
#pragma unroll
        for (int s = 0; s < 4; ++s) uar[s][LC - 1] = buffer_load_f64(rsrc_a, u_oa + cbs, (unsigned)(s * rb1));
        ubr[LC - 1] = buffer_load_f64(rsrc_b, dead ? kBeyond : (u_ob + cbs), 0u);
      }
      // move the cursor
      const int left = u_left - 16;
      const bool go = left > 0;
      unsigned oa = u_oa + 16u * row_bytes, ob = u_ob;
      const bool wrap = oa >= wrap_a;
      oa = wrap ? oa - wrap_a : oa;
      ob = wrap ? ob + row_bytes : ob;
      u_oa = go ? oa : u_oa;
      u_ob = go ? ob : u_ob;
      u_left = left;
    };
    auto multiply_factors = [&]() {
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < LC; ++j) breg[s][j] = uar[s][j] * ubr[j];
    };
    auto mfma_tile = [&](int t) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < LC; ++j)
          acc[t][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(areg[t][s], breg[s][j], acc[t][j], 0, 0, 0);
    };

    // ---- prologue: fragments of stage 0, products of stage 0, factors of stage 1 on their way.
    // Every one of the WMB row tiles is loaded and multiplied, live or not (a tile past the end of the block's rows
    // reads clamped rows and its results are dropped): the main loop is straight-line code, so the accumulators stay
    // in place in the accumulation registers.  The host picks the variant whose WMB fits the row count.
    load_factors();
    plan_a_advance();
    if constexpr (RP) {
#pragma unroll
      for (int p = 0; p < NPR; ++p) load_pair(p);
      if constexpr (SGR) load_single();
    } else {
#pragma unroll
      for (int t = 0; t < WMB; ++t) load_tile(t);
    }
    multiply_factors();
    load_factors();

    for (int st = 0; st < nstage; ++st) {
      plan_a_advance();
      if constexpr (RP) {
#pragma unroll
        for (int p = 0; p < NPR; ++p) {
          mfma_tile(2 * p);
          mfma_tile(2 * p + (WMB > 1 ? 1 : 0));
          __builtin_amdgcn_sched_barrier(0);
          load_pair(p);
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (SGR) {
          mfma_tile(WMB - 1);
          __builtin_amdgcn_sched_barrier(0);
          load_single();
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int t = 0; t < WMB; ++t) {
          mfma_tile(t);
          __builtin_amdgcn_sched_barrier(0);
          load_tile(t);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      multiply_factors();                         // products of the next stage (factors requested a stage ago)
      load_factors();                             // factors of the stage after it
    }
  }

  // ---- the four wavefronts' accumulators are added in wavefront order through LDS, TH tiles per round; wavefront w
  // adds and stores the tiles whose index within the round is w modulo 4.  Row tiles beyond the block's live ones
  // hold nothing and are neither exchanged nor stored (their rows may belong to the next row block).
  constexpr int TOT = WMB * LC;
  constexpr int TH = rows_reduce_tiles(WMB * WNB);
  constexpr int ROUNDS = (TOT + TH - 1) / TH;
  double* P = a.P + (int64_t)zb * a.pstride;
#pragma unroll
  for (int rd = 0; rd < ROUNDS; ++rd) {
    if (rd > 0) __syncthreads();
#pragma unroll
    for (int t = 0; t < WMB; ++t) {
      const bool tile_live = RP ? (t < 2 * lp || (SGR && t == WMB - 1 && single_live)) : (t < lt);   // uniform
#pragma unroll
      for (int j = 0; j < LC; ++j) {
        const int f = t * LC + j;
        if (f / TH == rd && tile_live) {
          const int fl = f - rd * TH;
#pragma unroll
          for (int q = 0; q < 4; ++q) smem[((fl * 4 + wave) * 4 + q) * 64 + lane] = acc[t][j][q];
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < WMB; ++t) {
      const bool tile_live = RP ? (t < 2 * lp || (SGR && t == WMB - 1 && single_live)) : (t < lt);
#pragma unroll
      for (int j = 0; j < LC; ++j) {
        const int f = t * LC + j;
        if (f / TH == rd && tile_live) {
          const int fl = f - rd * TH;
          if (wave == (fl & 3)) {                 // uniform over the wavefront
            // rows and column of this lane's four results of tile (t, j)
            int col;
            if (j < 2 * NPC) col = n0 + 32 * (j / 2) + 2 * li + (j % 2);
            else col = n0 + 32 * NPC + li;
            const bool paired_rows = RP && t < 2 * NPR;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const double* src = smem + (fl * 4 * 4 + q) * 64 + lane;
              const double sum = ((src[0] + src[4 * 64]) + src[2 * 4 * 64]) + src[3 * 4 * 64];
              const int r = paired_rows ? m0 + 32 * (t / 2) + 2 * (4 * q + lq) + (t % 2) : m0 + 16 * t + 4 * q + lq;
              if (r < a.In && col < a.ncols) P[(int64_t)r * a.ld + col] = sum;
            }
          }
        }
      }
    }
  }
}

template <int WMB, int WNB, int AMODE>
__global__ void __launch_bounds__(256) mttkrp_rows_kernel(RowsKernelArgs a) {
  extern __shared__ double smem[];
  // Hardware hands consecutive workgroup ids to the 8 XCDs in turn.  Workgroups of one (row block, split) pair differ
  // only in their column group and read the same tensor fragments: they get ids that are congruent modulo 8 and
  // adjacent in that XCD's sequence.
  const int id = blockIdx.x;
  const int x = id & 7, tq = id >> 3;
  const int cg = tq % a.ncg;
  const int g = (tq / a.ncg) * 8 + x;
  if (g >= a.nrb * a.nsb) return;                 // the whole workgroup leaves: no barrier is skipped by part of it
  if (WNB == 1 || cg < a.rem) rows_body<WMB, WNB, WNB, AMODE>(a, smem, g, cg);
  else rows_body<WMB, WNB, (WNB > 1 ? WNB - 1 : 1), AMODE>(a, smem, g, cg);
}

typedef void (*mttkrp_rows_fn)(RowsKernelArgs);
struct RowsVariant {
  int wmb, wnb;
  mttkrp_rows_fn fn[2];   // indexed by kRowsContig / kRowsPair
};
#define CALS_ROWS_VARIANT(WMB_, WNB_) \
  { WMB_, WNB_, { mttkrp_rows_kernel<WMB_, WNB_, kRowsContig>, mttkrp_rows_kernel<WMB_, WNB_, kRowsPair> } }

// Variant tables, one translation unit per group (compiled in parallel).
const RowsVariant* mttkrp_rows_variants_a(int* n);
const RowsVariant* mttkrp_rows_variants_b(int* n);

}  // namespace cals
