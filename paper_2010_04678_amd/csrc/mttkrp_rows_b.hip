// Instantiations of the rows kernel of the fused MTTKRP: row blocks of up to 13 tiles of 16 rows.
#include "mttkrp_rows_kernel.h"

namespace cals {

static const RowsVariant kTable[] = {
    CALS_ROWS_VARIANT(13, 2),
};

const RowsVariant* mttkrp_rows_variants_b(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}

}  // namespace cals
