// 32-bit-cell state kernels: float slab, 1 worker slot.
#define FDA_TU_TYPE float
#define FDA_TU_KC 1
#define FDA_TU_NAME launch_narrow_f32_kc1
#include "fda_state_narrow.inc"
