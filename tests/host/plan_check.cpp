// Host-only check of the fused MTTKRP launch plan (tile shape, column blocks, split of the contraction range):
// for a sweep of shapes, the invariants that the launcher relies on must hold.  No GPU is touched.
// Usage: plan_check  (prints "ok <count>" or the first violated case and exits non-zero)
#include <cstdio>
#include <cstdlib>

#include "../../paper_2010_04678_amd/csrc/cals_internal.h"

using namespace cals;

static int check(int In, int Ia, int Ib, int ncols, int cus) {
  MttkrpProblem p{};
  p.In = In; p.Ia = Ia; p.Ib = Ib; p.ncols = ncols; p.ld = (ncols + 15) / 16 * 16;
  const MttkrpPlan pl = mttkrp_plan(p, cus);
  const long long K = (long long)Ia * Ib;
  const char* why = nullptr;
  if (pl.wm != 1 && pl.wm != 2 && pl.wm != 4) why = "wm";
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
            if (check(dims[a], dims[b], dims[c], widths[w], cus)) return 1;
            ++count;
          }
        }
  // pseudo-random shapes
  unsigned long long s = 88172645463325252ull;
  auto next = [&]() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; };
  for (int i = 0; i < 20000; ++i) {
    const int In = 1 + (int)(next() % 5000), Ia = 1 + (int)(next() % 3000), Ib = 1 + (int)(next() % 3000);
    const int nc = 1 + (int)(next() % 1500);
    if (check(In, Ia, Ib, nc, 256)) return 1;
    ++count;
  }
  printf("ok %ld\n", count);
  return 0;
}
