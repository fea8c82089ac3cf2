// 32-bit-cell state kernels: float slab, 2 worker slots.
#define FDA_TU_TYPE float
#define FDA_TU_KC 2
#define FDA_TU_NAME launch_narrow_f32_kc2
#include "fda_state_narrow.inc"
