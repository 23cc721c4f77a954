// Instantiations of the fused MTTKRP kernel with WM = 1 row tiles per wavefront.
#include "mttkrp_kernel.h"

namespace cals {

static const Variant kTable[] = {
    CALS_VARIANT(1, 1, 16),
    CALS_VARIANT(1, 2, 16),
    CALS_VARIANT(1, 3, 16),
    CALS_VARIANT(1, 4, 16),
    CALS_VARIANT(1, 5, 16),
    CALS_VARIANT(1, 6, 16),
    CALS_VARIANT(1, 7, 16),
    CALS_VARIANT(1, 8, 16),
    CALS_VARIANT(1, 9, 16),
    CALS_VARIANT(1, 10, 16),
    CALS_VARIANT(1, 11, 16),
    CALS_VARIANT(1, 12, 16),
    CALS_VARIANT(1, 13, 16),
    CALS_VARIANT(1, 14, 16),
};

const Variant* mttkrp_variants_wm1(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}

}  // namespace cals
