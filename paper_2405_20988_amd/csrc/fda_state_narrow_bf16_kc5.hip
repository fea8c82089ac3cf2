// 32-bit-cell state kernels: fda::bf16_t slab, 5 worker slots.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_KC 5
#define FDA_TU_NAME launch_narrow_bf16_kc5
#include "fda_state_narrow.inc"
