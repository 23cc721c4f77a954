// Instantiations of the fused MTTKRP kernel with WM = 3 row tiles per wavefront (192-row workgroups: modes of
// 129 to 192 rows, and of 321 to 384, ..., fit them with less padding than 128- or 256-row workgroups and at a
// lower cost per MFMA than one row tile per wavefront).  Up to 9 column tiles (27 accumulator tiles).
#include "mttkrp_kernel.h"

namespace cals {

static const Variant kTable[] = {
    CALS_VARIANT_ODD(3, 1, 16),
    CALS_VARIANT_ODD(3, 2, 16),
    CALS_VARIANT_ODD(3, 3, 16),
    CALS_VARIANT_ODD(3, 4, 16),
    CALS_VARIANT_ODD(3, 5, 16),
    CALS_VARIANT_ODD(3, 6, 16),
    CALS_VARIANT_ODD(3, 7, 16),
    CALS_VARIANT_ODD(3, 8, 16),
    CALS_VARIANT_ODD(3, 9, 16),
};

const Variant* mttkrp_variants_wm3(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}

}  // namespace cals
