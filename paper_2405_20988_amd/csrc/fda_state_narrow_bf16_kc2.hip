// 32-bit-cell state kernels: fda::bf16_t slab, 2 worker slots.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_KC 2
#define FDA_TU_NAME launch_narrow_bf16_kc2
#include "fda_state_narrow.inc"
