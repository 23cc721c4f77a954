// Host-only check of the fused MTTKRP launch plan (tile shape, column blocks, split of the contraction range):
// for a sweep of shapes, the invariants that the launcher relies on must hold.  No GPU is touched.
// Usage: plan_check  (prints "ok <count>" or the first violated case and exits non-zero)
#include <cstdio>
#include <cstdlib>

#include "../../paper_2010_04678_amd/csrc/cals_internal.h"

using namespace cals;

// The rows kernel's launch (kind 1): what its launcher checks and its kernel assumes.
static const char* check_rows(const MttkrpProblem& p, const MttkrpPlan& pl) {
  const long long K = (long long)p.Ia * p.Ib;
  if (p.Ia < 16 || p.Ia % 4 != 0 || p.ld % 2 != 0) return "rows: operand shape";
  if (pl.rows_amode != 0 && pl.rows_amode != 1) return "rows: read mode";
  if (pl.rows_amode == 0 && (p.sa != 1 || p.sm % 2 != 0 || p.sb % 2 != 0)) return "rows: contiguous read mode on the wrong strides";
  if (pl.rows_amode == 1 && (p.sm != 1 || p.sb != (long long)p.Ia * p.sa || p.In % 2 != 0 || p.sa % 2 != 0)) return "rows: pair read mode on the wrong strides";
  if (pl.rows_wmb * pl.rows_wnb > 26 || pl.rows_wnb < 1) return "rows: variant";
  if (pl.rows_tpb < 1 || pl.rows_tpb > pl.rows_wmb) return "rows: tiles per block";
  if ((long long)pl.rows_nrb * pl.rows_tpb * 16 < p.In || (long long)(pl.rows_nrb - 1) * pl.rows_tpb * 16 >= p.In) return "rows: row blocks";
  if (pl.rows_amode == 1 && pl.rows_nrb > 1 && pl.rows_tpb % 2 != 0) return "rows: odd row block in pair mode";
  if (pl.rows_rem < 0 || pl.rows_rem > pl.rows_ncg || (pl.rows_wnb == 1 && pl.rows_rem != pl.rows_ncg)) return "rows: column groups";
  if (16 * (pl.rows_rem * pl.rows_wnb + (pl.rows_ncg - pl.rows_rem) * (pl.rows_wnb - 1)) != 16 * ((p.ncols + 15) / 16)) return "rows: column groups must cover exactly the tiles";
  if (pl.chunk < 16 || pl.chunk % 16 != 0 || pl.splits < 1) return "rows: chunk";
  if ((long long)pl.splits * 4 * pl.chunk < K || (long long)(pl.splits - 1) * 4 * pl.chunk >= K) return "rows: splits cover K exactly once";
  if (pl.workspace_bytes != (pl.splits > 1 ? (size_t)pl.splits * p.In * p.ld * sizeof(double) : 0)) return "rows: workspace";
  return nullptr;
}

static long g_rows_plans = 0;

// `layout`: 0 = no strides given (the tile kernel's plan only), 1 = output mode 1 of an In x Ia x Ib tensor (rows
// contiguous), 2 = an output mode whose fast contracted index is the tensor's first (contraction contiguous).
static int check(int In, int Ia, int Ib, int ncols, int cus, int layout = 0) {
  MttkrpProblem p{};
  p.In = In; p.Ia = Ia; p.Ib = Ib; p.ncols = ncols; p.ld = (ncols + 15) / 16 * 16;
  if (layout == 1) { p.sm = 1; p.sa = In; p.sb = (long long)In * Ia; }
  if (layout == 2) { p.sa = 1; p.sm = Ia; p.sb = (long long)Ia * In; }
  const MttkrpPlan pl = mttkrp_plan(p, cus);
  // the contraction range as the tile kernel counts it (padded runs for unaligned contiguous reads)
  const long long K = (long long)(pl.kind == 0 ? pl.ia_counted : Ia) * Ib;
  const char* why = nullptr;
  if (pl.kind == 0 && (pl.ia_counted < Ia || pl.ia_counted > Ia + 3)) why = "counted length of the fast index";
  if (pl.kind == 1) {
    ++g_rows_plans;
    why = check_rows(p, pl);
    if (why) {
      printf("FAIL %s: In=%d Ia=%d Ib=%d ncols=%d cus=%d layout=%d -> wmb=%d wnb=%d tpb=%d nrb=%d ncg=%d rem=%d splits=%d chunk=%lld\n", why, In, Ia, Ib,
             ncols, cus, layout, pl.rows_wmb, pl.rows_wnb, pl.rows_tpb, pl.rows_nrb, pl.rows_ncg, pl.rows_rem, pl.splits, (long long)pl.chunk);
      return 1;
    }
    return 0;
  }
  if (why) {}
  else if (pl.wm < 1 || pl.wm > 4) why = "wm";
  else if (pl.ka != 16) why = "ka";
  else if (pl.nparts < 1 || pl.nparts > 2) why = "nparts";
  else if ((long long)pl.mtiles * 64 * pl.wm < In || (long long)(pl.mtiles - 1) * 64 * pl.wm >= In) why = "mtiles";
  else if (pl.splits < 1 || pl.chunk < 1 || pl.chunk % (2 * pl.ka) != 0) why = "chunk";
  else if ((long long)pl.splits * pl.chunk < K || (long long)(pl.splits - 1) * pl.chunk >= K) why = "splits cover K exactly once";
  else if (pl.workspace_bytes != (pl.splits > 1 ? (size_t)pl.splits * In * p.ld * sizeof(double) : 0)) why = "workspace";
  int covered = 0;
  for (int q = 0; !why && q < pl.nparts; ++q) {
    const MttkrpPart& pt = pl.part[q];
    if (pt.col0 != covered) why = "parts leave a gap";
    else if (pt.wn < 1 || pt.wn > 14 || pt.ny < 1) why = "part shape";
    else if (pl.wm * pt.wn > 28) why = "accumulator budget";
    else if (pl.wm == 4 && pt.wn > 7) why = "wm 4 needs wn <= 7";
    else if (pl.wm == 3 && pt.wn > 9) why = "wm 3 needs wn <= 9";
    else if ((size_t)2 * pl.ka * 16 * pt.wn * sizeof(double) > 160 * 1024) why = "LDS";
    covered += 16 * pt.wn * pt.ny;
  }
  if (!why && covered != 16 * ((ncols + 15) / 16)) why = "column blocks must cover exactly the 16-column tiles of the width";
  if (why) {
    printf("FAIL %s: In=%d Ia=%d Ib=%d ncols=%d cus=%d -> wm=%d nparts=%d wn=%d ny=%d splits=%d chunk=%lld mtiles=%d\n", why, In, Ia, Ib,
           ncols, cus, pl.wm, pl.nparts, pl.part[0].wn, pl.part[0].ny, pl.splits, (long long)pl.chunk, pl.mtiles);
    return 1;
  }
  return 0;
}

int main() {
  const int dims[] = {1, 2, 3, 15, 16, 17, 40, 50, 63, 64, 65, 128, 180, 200, 255, 256, 257, 300, 1000, 4000, 32400};
  const int widths[] = {1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 110, 128, 208, 224, 225, 256, 420, 432, 433, 448, 449, 630, 640, 1024, 4096};
  const int nd = sizeof(dims) / sizeof(dims[0]), nw = sizeof(widths) / sizeof(widths[0]);
  long count = 0;
  for (int cus : {256, 304, 64})
    for (int a = 0; a < nd; ++a)
      for (int b = 0; b < nd; ++b)
        for (int c = 0; c < nd; ++c) {
          if ((long long)dims[a] * dims[b] * dims[c] > (1LL << 36)) continue;
          for (int w = 0; w < nw; ++w) {
            for (int layout = 0; layout < 3; ++layout) {
              if (check(dims[a], dims[b], dims[c], widths[w], cus, layout)) return 1;
              ++count;
            }
          }
        }
  // pseudo-random shapes
  unsigned long long s = 88172645463325252ull;
  auto next = [&]() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; };
  for (int i = 0; i < 20000; ++i) {
    const int In = 1 + (int)(next() % 5000), Ia = 1 + (int)(next() % 3000), Ib = 1 + (int)(next() % 3000);
    const int nc = 1 + (int)(next() % 1500);
    if (check(In, Ia, Ib, nc, 256, i % 3)) return 1;
    ++count;
  }
  if (g_rows_plans < 1000) { printf("FAIL: the sweep reached the rows kernel's planner only %ld times\n", g_rows_plans); return 1; }
  printf("ok %ld (%ld of them rows-kernel plans)\n", count, g_rows_plans);
  return 0;
}
