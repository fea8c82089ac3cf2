// 32-bit-cell state kernels: float slab, 8 worker slots.
#define FDA_TU_TYPE float
#define FDA_TU_KC 8
#define FDA_TU_NAME launch_narrow_f32_kc8
#include "fda_state_narrow.inc"
