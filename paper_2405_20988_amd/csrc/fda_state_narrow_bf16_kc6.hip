// 32-bit-cell state kernels: fda::bf16_t slab, 6 worker slots.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_KC 6
#define FDA_TU_NAME launch_narrow_bf16_kc6
#include "fda_state_narrow.inc"
