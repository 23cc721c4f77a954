// Instantiations of the rows kernel of the fused MTTKRP: row blocks of up to 4 and up to 7 tiles of 16 rows.
#include "mttkrp_rows_kernel.h"

namespace cals {

static const RowsVariant kTable[] = {
    CALS_ROWS_VARIANT(4, 2),
    CALS_ROWS_VARIANT(4, 4),
    CALS_ROWS_VARIANT(7, 2),
};

const RowsVariant* mttkrp_rows_variants_a(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}

}  // namespace cals
