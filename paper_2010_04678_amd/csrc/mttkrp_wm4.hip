// Instantiations of the fused MTTKRP kernel with WM = 4 row tiles per wavefront.
#include "mttkrp_kernel.h"

namespace cals {

static const Variant kTable[] = {
    CALS_VARIANT(4, 1, 16),
    CALS_VARIANT(4, 2, 16),
    CALS_VARIANT(4, 3, 16),
    CALS_VARIANT(4, 4, 16),
    CALS_VARIANT(4, 5, 16),
    CALS_VARIANT(4, 6, 16),
    CALS_VARIANT(4, 7, 16),
};

const Variant* mttkrp_variants_wm4(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}

}  // namespace cals
