// 32-bit-cell state kernels: float slab, 5 worker slots.
#define FDA_TU_TYPE float
#define FDA_TU_KC 5
#define FDA_TU_NAME launch_narrow_f32_kc5
#include "fda_state_narrow.inc"
