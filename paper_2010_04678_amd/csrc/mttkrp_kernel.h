// Device code of the fused multi-model MTTKRP (Eq. (2) of the paper) for gfx950:
//   M[m, c] = sum_{ia, ib} T[m, ia, ib] * (Ua[ia, c] * Ub[ib, c])      for every fused column c.
//
// One workgroup = 4 wavefronts; wavefront w owns WM 16-row MFMA tiles (rows m0 .. m0+16*WM) and ALL
// 16*WN columns of the workgroup's column block; the WM*WN accumulator tiles (v_mfma_f64_16x16x4_f64,
// 4 doubles per lane each) stay in registers over the workgroup's whole share of the contraction range.
//
// Measured on MI355X: an fp64 MFMA occupies its SIMD's issue port for all of its 64 cycles -- no other
// instruction of any wavefront on that SIMD issues meanwhile.  Every non-MFMA instruction therefore costs
// MFMA time, and the kernel is organised to need as few of them per MFMA as possible:
//   - a wavefront holds WM row tiles, so one B fragment (one LDS read) feeds WM MFMAs;
//   - the Khatri-Rao tile (KA x 16*WN) is produced once per workgroup in LDS (one fp64 multiply per
//     element, a quarter of the rows per wavefront) and never exists in HBM; the row a wavefront produces
//     is the same for all its lanes, so its address arithmetic runs on the scalar unit;
//   - tensor fragments go from global memory straight into the MFMA register layout (lane l holds
//     A[l%16][l/16]); one 64-bit offset serves all WM fragments of a k-step;
//   - B fragments of k-step s+1 are read from LDS before the MFMAs of k-step s are issued; factor rows and
//     tensor fragments are requested a whole stage before they are used: no wait inside a k-step.
// The LDS tile is double-buffered with one barrier per stage of KA contraction indices.
#pragma once
#include "cals_internal.h"

namespace cals {

typedef double double4_t __attribute__((ext_vector_type(4)));
typedef unsigned uint2_t __attribute__((ext_vector_type(2)));

// Factor rows are read through buffer descriptors: scalar base (the matrix), scalar offset (the row, uniform
// over the wavefront) and a 32-bit per-lane offset (the column) -- no vector address arithmetic at all.
__device__ inline __amdgpu_buffer_rsrc_t factor_rsrc(const double* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(base), 0, (int)bytes, 0x00020000);
}
__device__ inline double buffer_load_f64(__amdgpu_buffer_rsrc_t rsrc, unsigned lane_byte, unsigned row_byte) {
  return __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_byte, (int)row_byte, 0));
}
__device__ inline double2 buffer_load_f64x2(__amdgpu_buffer_rsrc_t rsrc, unsigned lane_byte, unsigned row_byte) {
  return __builtin_bit_cast(double2, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_byte, (int)row_byte, 0));
}

struct MttkrpKernelArgs {
  const double* T;
  const double* Ua;
  const double* Ub;
  double* P;          // output: partials [split][In][ld], or M itself when there is one split
  const double* zeros; // >= 4 zero doubles, 16-byte aligned: what a lane past the end of its split loads
  int64_t sm, sa, sb; // element strides of T: output row, fast contracted index, slow contracted index
  int64_t K, chunk;   // contraction length Ia*Ib; indices per split (multiple of KA)
  int64_t pstride;    // In * ld
  int In, Ia, Ib;     // Ia: length of the fast contracted index as the kernel counts it (kContig4U: rounded up to 4)
  int Iav;            // its valid length (rows of Ua, elements per run in memory); equals Ia except for kContig4U
  int ncols, ld;
  int mtiles, ny, splits;   // logical grid: row blocks, column blocks, splits
  int col0;                 // first column of column block 0
  int pinned;               // splits is a multiple of 8: keep every split on one XCD
};

// How a contraction index k = ia + Ia*ib maps to a tensor offset ia*sa + ib*sb:
//   kAffine : sb == Ia*sa, offset = k*sa (modes 1 and 3: no wrap bookkeeping at all)
//   kWrap   : Ia >= KA, an index advanced by at most KA wraps at most once (mode 2)
//   kGeneral: any Ia >= 1 (wrap loop; tiny tensors)
//   kContig4: sa == 1, Ia % 4 == 0, Ia >= KA, 16-byte aligned rows (modes 2 and 3 of aligned tensors): a lane
//             owns 4 CONSECUTIVE contraction indices per stage (two 16-byte loads, fully coalesced rows); MFMA
//             k-step s then takes element s of every lane, i.e. tile row 4*lq + s instead of 4*s + lq.
//   kRowPair: kAffine with sm == 1 (mode 1), an even row count and 16-byte aligned columns: a lane reads TWO
//             adjacent rows with one 16-byte load and feeds them to two row tiles, so row tile 2p holds the even
//             and row tile 2p+1 the odd rows of the wavefront's p-th group of 32 rows (needs WM even; kernels
//             with odd WM treat it as kAffine and are never launched with it).
//   kContig4U: sa == 1, Ia >= KA, but Ia not a multiple of 4 or rows not 16-byte aligned (odd-sized tensors): the
//             same lane-owns-4-consecutive-indices layout on a contraction index PADDED to a multiple of 4 per run
//             (k = ia + Ia_pad*ib, positions ia >= Iav load zeros), with 16-byte loads at 8-byte alignment; a load
//             that would straddle the end of a run is moved back by one element and its values are shifted, so no
//             byte outside the run is ever read.  One load instruction then touches whole cache lines of 16 rows
//             instead of one 32-byte sector each.  The extra selects cost issue slots, so the host uses it for narrow,
//             memory-bound launches only.
enum { kAffine = 0, kWrap = 1, kGeneral = 2, kContig4 = 3, kRowPair = 4, kContig4U = 5 };

typedef double double2_u __attribute__((ext_vector_type(2), aligned(8)));   // 16-byte load at 8-byte alignment

template <int WM, int WN, int KA, int MODE, bool PAIR>
__global__ void __launch_bounds__(256) mttkrp_kernel(MttkrpKernelArgs a) {
  constexpr int NC = 16 * WN;                 // columns of the LDS tile
  constexpr int KS = KA / 4;                  // MFMA k-steps per stage = tile rows produced per wavefront
  constexpr int PW = PAIR ? 2 : 1;            // adjacent columns a lane produces (2: 16-byte loads and stores)
  constexpr int CU = (NC / PW + 63) / 64;     // chunks of 64*PW columns of a tile row
  constexpr int TILE = KA * NC;               // doubles per LDS buffer
  extern __shared__ double smem[];            // [2][KA][NC]

  // ---- logical block coordinates.  Hardware hands consecutive workgroup ids to the 8 XCDs in turn.  With 8k
  // splits all workgroups of one split (same factor rows, and for ny > 1 the same tensor tile) are kept on one
  // XCD so that they share its L2; with fewer splits the workgroups of a split are spread over the XCDs.
  int bx, by, bz;
  {
    const int id = blockIdx.x;
    const int per_split = a.mtiles * a.ny;
    int g;
    if (a.pinned) {
      const int xcd = id & 7, slot = id >> 3;
      bz = (slot / per_split) * 8 + xcd;
      g = slot % per_split;
    } else {
      bz = id / per_split;
      g = id % per_split;
    }
    by = g % a.ny;
    bx = g / a.ny;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15;                   // A: row within the tile / B,D: column within the tile
  const int lq = lane >> 4;                   // A,B: k within the k-step / D: row group
  const int m0 = bx * (64 * WM) + wave * (16 * WM);
  const int n0 = a.col0 + by * NC;
  const int64_t kb = (int64_t)bz * a.chunk;
  const int64_t ke = (kb + a.chunk < a.K) ? (kb + a.chunk) : a.K;
  const int nstage = (int)((ke - kb + KA - 1) / KA);
  const int Ia = a.Ia;
  constexpr bool RP = (MODE == kRowPair) && (WM % 2 == 0);     // rows interleaved over pairs of row tiles
  constexpr bool AFF = (MODE == kAffine) || (MODE == kRowPair);

  double4_t acc[WM][WN];
#pragma unroll
  for (int t = 0; t < WM; ++t)
#pragma unroll
    for (int j = 0; j < WN; ++j) acc[t][j] = double4_t{0.0, 0.0, 0.0, 0.0};

  // ---- tensor fragments: lane (li, lq) of row tile t reads T[Prow[t] + koff], koff = offset of its k.
  // Rows past the end of the matrix are clamped to the last row (their results are never stored).
  const double* Prow[WM];
#pragma unroll
  for (int t = 0; t < WM; ++t) {
    if (RP) {         // the even row of the lane's pair; only tiles 0, 2, ... load (In is even: the pair is in range)
      const int r = m0 + 32 * (t / 2) + 2 * li;
      Prow[t] = a.T + (int64_t)(r < a.In ? r : a.In - 2);
    } else {
      const int r = m0 + 16 * t + li;
      Prow[t] = a.T + (int64_t)(r < a.In ? r : a.In - 1) * a.sm;
    }
  }
  int64_t koff;                               // ia*sa + ib*sb of this lane's current k
  int a_ia = 0;                               // only tracked when the offset is not affine in k
  int a_left;                                 // contraction indices left before ke, from this lane's k
  {
    const int64_t k = kb + ((MODE == kContig4 || MODE == kContig4U) ? 4 * lq : lq);
    if (AFF) {
      koff = k * a.sa;
    } else {
      const int64_t ib = k / Ia;
      a_ia = (int)(k - ib * Ia);
      koff = (int64_t)a_ia * a.sa + ib * a.sb;
    }
    a_left = (int)(ke - k);                   // <= chunk < 2^31 (checked on the host)
  }
  const int64_t a_step = 4 * a.sa;
  const int64_t a_wrap = a.sb - (int64_t)Ia * a.sa;

  double areg0[KS][WM], areg1[KS][WM];

  // Loads are unconditional; a lane past the end of the split reads from a zero buffer instead (pointer
  // select: no divergent control flow, and nothing to patch once the value arrives, which would make the
  // wavefront wait for the load right away).
  const double* const zeros = a.zeros;
  auto load_a_stage = [&](double (&dst)[KS][WM]) {
    if (MODE == kContig4) {
      static_assert(MODE != kContig4 || KA == 16, "a lane's run of 4 indices times 4 lane groups is one stage");
      // all four indices of a lane are on the same side of ke (ke, kb and Ia are multiples of 4)
      const bool ok = a_left > 0;
#pragma unroll
      for (int t = 0; t < WM; ++t) {
        const double* p = ok ? Prow[t] + koff : zeros;
        const double2 v01 = *reinterpret_cast<const double2*>(p);
        const double2 v23 = *reinterpret_cast<const double2*>(p + 2);
        dst[0][t] = v01.x;
        dst[1][t] = v01.y;
        dst[2][t] = v23.x;
        dst[3][t] = v23.y;
      }
      a_left -= KA;
      koff += KA;
      a_ia += KA;
      if (a_ia >= Ia) { a_ia -= Ia; koff += a_wrap; }
      return;
    }
    if (MODE == kContig4U) {
      static_assert(MODE != kContig4U || KA == 16, "a lane's run of 4 indices times 4 lane groups is one stage");
      // valid elements among the lane's four: all (>= 4), the first 3, 2 or 1, or none (padding, or past the split)
      const int nvalid = (a_left > 0) ? (a.Iav - a_ia) : 0;
      // Wide column blocks (compute-bound): when no lane of the wavefront sits on the end of a run -- the usual case --
      // a branch skips the selects, which would cost MFMA issue time.  Narrow blocks (memory-bound) always take the
      // general form: there the branch costs more than the selects (it keeps the loads from being issued early).
      if (WN > 3 && __builtin_amdgcn_ballot_w64(nvalid > 0 && nvalid < 4) == 0) {
        const bool ok = nvalid > 0;
#pragma unroll
        for (int t = 0; t < WM; ++t) {
          const double* p = ok ? Prow[t] + koff : zeros;
          const double2_u v0 = *reinterpret_cast<const double2_u*>(p);
          const double2_u v1 = *reinterpret_cast<const double2_u*>(p + 2);
          dst[0][t] = v0.x;
          dst[1][t] = v0.y;
          dst[2][t] = v1.x;
          dst[3][t] = v1.y;
        }
      } else {
        const bool lo2 = nvalid >= 2, lo1 = nvalid == 1, hi2 = nvalid >= 4, hi1 = nvalid == 3;
#pragma unroll
        for (int t = 0; t < WM; ++t) {
          const double* p = Prow[t] + koff;
          // halves (elements 0,1) and (2,3); a half with only its first element valid reads one element earlier
          const double* p0 = lo2 ? p : (lo1 ? p - 1 : zeros);
          const double* p1 = hi2 ? p + 2 : (hi1 ? p + 1 : zeros);
          const double2_u v0 = *reinterpret_cast<const double2_u*>(p0);
          const double2_u v1 = *reinterpret_cast<const double2_u*>(p1);
          dst[0][t] = lo1 ? v0.y : v0.x;
          dst[1][t] = lo1 ? 0.0 : v0.y;
          dst[2][t] = hi1 ? v1.y : v1.x;
          dst[3][t] = hi1 ? 0.0 : v1.y;
        }
      }
      a_left -= KA;
      koff += KA;
      a_ia += KA;
      if (a_ia >= Ia) { a_ia -= Ia; koff += a_wrap; }
      return;
    }
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bool ok = a_left > 0;
#pragma unroll
      for (int t = 0; t < WM; ++t) {
        const double* p = ok ? Prow[t] + koff : zeros;
        if (RP) {
          if (t % 2 == 0) {
            const double2 v = *reinterpret_cast<const double2*>(p);
            dst[s][t] = v.x;
            dst[s][t + (WM > 1 ? 1 : 0)] = v.y;
          }
        } else {
          dst[s][t] = *p;
        }
      }
      a_left -= 4;
      koff += a_step;
      if (MODE == kWrap) {
        a_ia += 4;
        if (a_ia >= Ia) { a_ia -= Ia; koff += a_wrap; }
      } else if (MODE == kGeneral) {
        a_ia += 4;
        while (a_ia >= Ia) { a_ia -= Ia; koff += a_wrap; }
      }
    }
  };

  // ---- Khatri-Rao tile production.  Wavefront w produces rows w, w+4, ... of the next stage's tile
  // (one row per k-step): lane l covers columns l, l+64, ...  The row index is uniform over the
  // wavefront, so (ia, ib) and the two row base pointers live in scalar registers.  Rows and columns
  // outside the problem are clamped to valid ones rather than zeroed: such a row only meets zero tensor
  // fragments (a_left <= 0), such a column only feeds output columns that are never stored.
  int tcol[CU];
  unsigned gbyte[CU];                         // byte offset of the lane's column within a factor row
#pragma unroll
  for (int u = 0; u < CU; ++u) {
    const int tc = PW * (lane + 64 * u);
    tcol[u] = tc < NC ? tc : NC - PW;         // surplus lanes repeat the last columns (same value, same address)
    const int gc = n0 + tcol[u];
    gbyte[u] = 8u * (unsigned)(gc <= a.ld - PW ? gc : a.ld - PW);   // PAIR: ld is even (checked on the host)
  }
  // Factor rows are fetched a whole stage before they are multiplied (row x of the tile after next is requested
  // right after row x of the next tile has been written), so that a miss in L2 never stalls the wavefront.
  double pua[KS][CU][PW], pub[KS][CU][PW];
  const unsigned row_bytes = 8u * (unsigned)a.ld;
  const __amdgpu_buffer_rsrc_t rsrc_a = factor_rsrc(a.Ua, row_bytes * (unsigned)a.Iav);   // < 2^32 (checked on the host)
  const __amdgpu_buffer_rsrc_t rsrc_b = factor_rsrc(a.Ub, row_bytes * (unsigned)a.Ib);
  // Byte offsets of the factor rows (ia, ib) of this wavefront's row x of the tile to fetch next: uniform over
  // the wavefront, kept in scalar registers and advanced by KA rows per fetch (one compare for the wrap of ia).
  unsigned row_oa[KS], row_ob[KS];
  const unsigned wrap_a = row_bytes * (unsigned)Ia;
  const unsigned last_b = row_bytes * (unsigned)(a.Ib - 1);
  // kContig4U counts Ia rounded up to 4: the padding rows Iav .. Ia-1 do not exist in Ua.  They only ever meet zero
  // tensor fragments, so any valid row serves; the offset is clamped to the last one (a scalar row offset is not
  // covered by the descriptor's range check).
  const unsigned last_a = row_bytes * (unsigned)(a.Iav - 1);
#pragma unroll
  for (int x = 0; x < KS; ++x) {
    const int64_t k = kb + wave + 4 * x;
    const int64_t ib = k / Ia;
    row_oa[x] = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)(k - ib * Ia) * row_bytes));
    row_ob[x] = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)ib * row_bytes));   // < 2^32: ib <= Ib
  }

  auto fetch_row = [&](int x, double (&ua)[CU][PW], double (&ub)[CU][PW]) {
    const unsigned oa = (MODE == kContig4U && row_oa[x] > last_a) ? last_a : row_oa[x];
    const unsigned ob = row_ob[x] < last_b ? row_ob[x] : last_b;   // rows past the end of K: any valid row
#pragma unroll
    for (int u = 0; u < CU; ++u) {
      if (PAIR) {
        const double2 va = buffer_load_f64x2(rsrc_a, gbyte[u], oa);
        const double2 vb = buffer_load_f64x2(rsrc_b, gbyte[u], ob);
        ua[u][0] = va.x; ua[u][PW - 1] = va.y;
        ub[u][0] = vb.x; ub[u][PW - 1] = vb.y;
      } else {
        ua[u][0] = buffer_load_f64(rsrc_a, gbyte[u], oa);
        ub[u][0] = buffer_load_f64(rsrc_b, gbyte[u], ob);
      }
    }
    // the same row of the following tile
    row_oa[x] += (unsigned)KA * row_bytes;
    if (MODE == kGeneral) {
      while (row_oa[x] >= wrap_a) { row_oa[x] -= wrap_a; row_ob[x] += row_bytes; }
    } else {
      if (row_oa[x] >= wrap_a) { row_oa[x] -= wrap_a; row_ob[x] += row_bytes; }
    }
  };
  auto commit_row = [&](double* tile, int x, const double (&ua)[CU][PW], const double (&ub)[CU][PW]) {
#pragma unroll
    for (int u = 0; u < CU; ++u) {
      double* dst = tile + (wave + 4 * x) * NC + tcol[u];
      if (PAIR)
        *reinterpret_cast<double2*>(dst) = double2{ua[u][0] * ub[u][0], ua[u][PW - 1] * ub[u][PW - 1]};
      else
        *dst = ua[u][0] * ub[u][0];
    }
  };
  // Narrow tiles (at most 64 columns, low total rank): a 16-byte load per factor covers 64 / LPR tile rows -- lane
  // l takes row l / LPR and column pair l % LPR -- so the wavefront's four rows of a tile take one load per factor
  // (two for 64 columns), one multiply pair and one LDS store each, instead of one of each per row.  The row
  // offsets are then per lane (vector registers).
  constexpr bool PACK = PAIR && (NC <= 64) && (KS == 4);
  constexpr int LPR = NC / 2;                        // lanes per tile row: 8, 16, 24 or 32
  constexpr int RPI = (64 / (LPR > 0 ? LPR : 1)) >= 4 ? 4 : 2;   // whole rows of this wavefront per load instruction
  constexpr int NIW = PACK ? KS / RPI : 1;           // load instructions per factor for the wavefront's four rows
  unsigned pk_oa[NIW], pk_ob[NIW], pk_col = 0;
  int pk_dst[NIW];
  double pk_ua[NIW][2], pk_ub[NIW][2];
  if (PACK) {
    const int xl = (lane / LPR < RPI) ? lane / LPR : RPI - 1;   // surplus lanes repeat the last row (same address, same value)
    const int cp = lane % LPR;
    const int gc = n0 + 2 * cp;
    pk_col = 8u * (unsigned)(gc <= a.ld - 2 ? gc : a.ld - 2);
#pragma unroll
    for (int i = 0; i < NIW; ++i) {
      const int xr = i * RPI + xl;                   // which of the wavefront's rows: tile row wave + 4 * xr
      pk_dst[i] = (wave + 4 * xr) * NC + 2 * cp;
      const int64_t k = kb + wave + 4 * xr;
      const int64_t ib = k / Ia;
      pk_oa[i] = (unsigned)(k - ib * Ia) * row_bytes;
      pk_ob[i] = (unsigned)ib * row_bytes;
    }
  }
  auto fetch_packed = [&](int i) {
    const unsigned ob = pk_ob[i] < last_b ? pk_ob[i] : last_b;
    const unsigned oa = (MODE == kContig4U && pk_oa[i] > last_a) ? last_a : pk_oa[i];
    const double2 va = buffer_load_f64x2(rsrc_a, oa + pk_col, 0u);
    const double2 vb = buffer_load_f64x2(rsrc_b, ob + pk_col, 0u);
    pk_ua[i][0] = va.x; pk_ua[i][1] = va.y;
    pk_ub[i][0] = vb.x; pk_ub[i][1] = vb.y;
    pk_oa[i] += (unsigned)KA * row_bytes;
    if (MODE == kGeneral) {
      while (pk_oa[i] >= wrap_a) { pk_oa[i] -= wrap_a; pk_ob[i] += row_bytes; }
    } else {
      if (pk_oa[i] >= wrap_a) { pk_oa[i] -= wrap_a; pk_ob[i] += row_bytes; }
    }
  };
  auto commit_packed = [&](double* tile, int i) {
    *reinterpret_cast<double2*>(tile + pk_dst[i]) = double2{pk_ua[i][0] * pk_ub[i][0], pk_ua[i][1] * pk_ub[i][1]};
  };

  double breg[2][WN];
  auto load_b = [&](const double* tile, int s, double (&b)[WN]) {
    const double* brow = tile + ((MODE == kContig4 || MODE == kContig4U) ? 4 * lq + s : 4 * s + lq) * NC + li;
#pragma unroll
    for (int j = 0; j < WN; ++j) b[j] = brow[16 * j];
  };

  // One stage: MFMAs on (acur, tile `cur`); meanwhile the tensor fragments of the next stage are fetched, the
  // next tile is written into the other buffer and the factor rows of the tile after it are requested.
  auto run_stage = [&](const double (&acur)[KS][WM], double (&anext)[KS][WM], int cur) {
    const double* tile = smem + cur * TILE;
    double* next_tile = smem + (cur ^ 1) * TILE;
    load_b(tile, 0, breg[0]);
    load_a_stage(anext);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s + 1 < KS) load_b(tile, s + 1, breg[(s + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int t = 0; t < WM; ++t)
          acc[t][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(acur[s][t], breg[s & 1][j], acc[t][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (PACK) {
        if (s < NIW) {
          commit_packed(next_tile, s);
          fetch_packed(s);
        }
      } else {
        commit_row(next_tile, s, pua[s], pub[s]);
        fetch_row(s, pua[s], pub[s]);
      }
    }
    __syncthreads();
  };

  // ---- prologue: tile 0, the factor rows of tile 1 and fragment 0
  if (PACK) {
#pragma unroll
    for (int i = 0; i < NIW; ++i) {
      fetch_packed(i);
      commit_packed(smem, i);
    }
#pragma unroll
    for (int i = 0; i < NIW; ++i) fetch_packed(i);
  } else {
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      fetch_row(x, pua[x], pub[x]);
      commit_row(smem, x, pua[x], pub[x]);
    }
#pragma unroll
    for (int x = 0; x < KS; ++x) fetch_row(x, pua[x], pub[x]);
  }
  // A wavefront whose rows all lie past the end of the matrix (the tail of a short mode) only helps to produce
  // the tiles: it issues no tensor loads and no matrix instructions, which leaves its SIMD to the wavefronts of
  // the other workgroups on the compute unit.
  auto produce_stage = [&](int cur) {
    double* next_tile = smem + (cur ^ 1) * TILE;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (PACK) {
        if (s < NIW) {
          commit_packed(next_tile, s);
          fetch_packed(s);
        }
      } else {
        commit_row(next_tile, s, pua[s], pub[s]);
        fetch_row(s, pua[s], pub[s]);
      }
    }
    __syncthreads();
  };
  if (m0 >= a.In) {             // uniform over the wavefront
    __syncthreads();
    for (int st = 0; st < nstage; st += 2) {
      produce_stage(0);
      produce_stage(1);
    }
    return;
  }
  load_a_stage(areg0);
  __syncthreads();

  // Stages run in pairs (the two register sets and LDS buffers alternate) with no branch in between, so the
  // accumulators stay in place; a split with an odd stage count runs one extra stage on zero fragments.
  for (int st = 0; st < nstage; st += 2) {
    run_stage(areg0, areg1, 0);
    run_stage(areg1, areg0, 1);
  }

  // ---- epilogue: D[4*v + lq][li] of every tile -> P[split][row][col]
  double* P = a.P + (int64_t)bz * a.pstride;
#pragma unroll
  for (int t = 0; t < WM; ++t) {
    if ((RP ? m0 + 32 * (t / 2) : m0 + 16 * t) < a.In) {
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        const int col = n0 + 16 * j + li;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int r = RP ? m0 + 32 * (t / 2) + 2 * (4 * v + lq) + (t % 2) : m0 + 16 * t + 4 * v + lq;
          if (r < a.In && col < a.ncols) P[(int64_t)r * a.ld + col] = acc[t][j][v];
        }
      }
    }
  }
}

typedef void (*mttkrp_fn)(MttkrpKernelArgs);
struct Variant {
  int wm, wn, ka;
  mttkrp_fn fn[6][2]; // indexed by kAffine / kWrap / kGeneral / kContig4 / kRowPair / kContig4U, and by PAIR
};
#define CALS_VARIANT(WM_, WN_, KA_)                                                                       \
  {                                                                                                       \
    WM_, WN_, KA_, {                                                                                      \
      {mttkrp_kernel<WM_, WN_, KA_, kAffine, false>, mttkrp_kernel<WM_, WN_, KA_, kAffine, true>},        \
          {mttkrp_kernel<WM_, WN_, KA_, kWrap, false>, mttkrp_kernel<WM_, WN_, KA_, kWrap, true>},        \
          {mttkrp_kernel<WM_, WN_, KA_, kGeneral, false>, mttkrp_kernel<WM_, WN_, KA_, kGeneral, true>},  \
          {mttkrp_kernel<WM_, WN_, KA_, kContig4, false>, mttkrp_kernel<WM_, WN_, KA_, kContig4, true>},  \
          {mttkrp_kernel<WM_, WN_, KA_, kRowPair, false>, mttkrp_kernel<WM_, WN_, KA_, kRowPair, true>},  \
          {mttkrp_kernel<WM_, WN_, KA_, kContig4U, false>, mttkrp_kernel<WM_, WN_, KA_, kContig4U, true>} \
    }                                                                                                     \
  }

// An odd number of row tiles per wavefront cannot pair rows: the planner never asks for kRowPair there, and the slot
// holds the kAffine kernel (which is what a kRowPair kernel with odd WM would be) instead of a second copy of it.
#define CALS_VARIANT_ODD(WM_, WN_, KA_)                                                                     \
  {                                                                                                         \
    WM_, WN_, KA_, {                                                                                        \
      {mttkrp_kernel<WM_, WN_, KA_, kAffine, false>, mttkrp_kernel<WM_, WN_, KA_, kAffine, true>},          \
          {mttkrp_kernel<WM_, WN_, KA_, kWrap, false>, mttkrp_kernel<WM_, WN_, KA_, kWrap, true>},          \
          {mttkrp_kernel<WM_, WN_, KA_, kGeneral, false>, mttkrp_kernel<WM_, WN_, KA_, kGeneral, true>},    \
          {mttkrp_kernel<WM_, WN_, KA_, kContig4, false>, mttkrp_kernel<WM_, WN_, KA_, kContig4, true>},    \
          {mttkrp_kernel<WM_, WN_, KA_, kAffine, false>, mttkrp_kernel<WM_, WN_, KA_, kAffine, true>},      \
          {mttkrp_kernel<WM_, WN_, KA_, kContig4U, false>, mttkrp_kernel<WM_, WN_, KA_, kContig4U, true>}   \
    }                                                                                                       \
  }
#define CALS_VARIANT_WM1(WN_, KA_) CALS_VARIANT_ODD(1, WN_, KA_)

// Variant tables, one translation unit per WM (compiled in parallel).
const Variant* mttkrp_variants_wm1(int* n);
const Variant* mttkrp_variants_wm2(int* n);
const Variant* mttkrp_variants_wm3(int* n);
const Variant* mttkrp_variants_wm4(int* n);

}  // namespace cals
