// 32-bit-cell state kernels: float slab, 3 worker slots.
#define FDA_TU_TYPE float
#define FDA_TU_KC 3
#define FDA_TU_NAME launch_narrow_f32_kc3
#include "fda_state_narrow.inc"
