// Fallback state kernels: fda::bf16_t slab, fp64 cells.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_CELL fda::kCellF64
#define FDA_TU_NAME launch_wide_bf16_f64
#include "fda_state_wide.inc"
