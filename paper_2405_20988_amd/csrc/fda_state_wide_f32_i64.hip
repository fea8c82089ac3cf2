// Fallback state kernels: float slab, 64-bit integer cells.
#define FDA_TU_TYPE float
#define FDA_TU_CELL fda::kCellI64
#define FDA_TU_NAME launch_wide_f32_i64
#include "fda_state_wide.inc"
