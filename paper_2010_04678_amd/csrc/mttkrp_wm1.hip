// Instantiations of the fused MTTKRP kernel with WM = 1 row tiles per wavefront.
#include "mttkrp_kernel.h"

namespace cals {

static const Variant kTable[] = {
    CALS_VARIANT_WM1(1, 16),
    CALS_VARIANT_WM1(2, 16),
    CALS_VARIANT_WM1(3, 16),
    CALS_VARIANT_WM1(4, 16),
    CALS_VARIANT_WM1(5, 16),
    CALS_VARIANT_WM1(6, 16),
    CALS_VARIANT_WM1(7, 16),
    CALS_VARIANT_WM1(8, 16),
    CALS_VARIANT_WM1(9, 16),
    CALS_VARIANT_WM1(10, 16),
    CALS_VARIANT_WM1(11, 16),
    CALS_VARIANT_WM1(12, 16),
    CALS_VARIANT_WM1(13, 16),
    CALS_VARIANT_WM1(14, 16),
};

const Variant* mttkrp_variants_wm1(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}

}  // namespace cals
