// Fallback state kernels: fda::bf16_t slab, 64-bit integer cells.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_CELL fda::kCellI64
#define FDA_TU_NAME launch_wide_bf16_i64
#include "fda_state_wide.inc"
