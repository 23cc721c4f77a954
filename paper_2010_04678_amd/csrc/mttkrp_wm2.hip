// Instantiations of the fused MTTKRP kernel with WM = 2 row tiles per wavefront.
#include "mttkrp_kernel.h"

namespace cals {

static const Variant kTable[] = {
    CALS_VARIANT(2, 1, 16),
    CALS_VARIANT(2, 2, 16),
    CALS_VARIANT(2, 3, 16),
    CALS_VARIANT(2, 4, 16),
    CALS_VARIANT(2, 5, 16),
    CALS_VARIANT(2, 6, 16),
    CALS_VARIANT(2, 7, 16),
    CALS_VARIANT(2, 8, 16),
    CALS_VARIANT(2, 9, 16),
    CALS_VARIANT(2, 10, 16),
    CALS_VARIANT(2, 11, 16),
    CALS_VARIANT(2, 12, 16),
    CALS_VARIANT(2, 13, 16),
    CALS_VARIANT(2, 14, 16),
};

const Variant* mttkrp_variants_wm2(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}

}  // namespace cals
