// 32-bit-cell state kernels: fda::bf16_t slab, 1 worker slot.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_KC 1
#define FDA_TU_NAME launch_narrow_bf16_kc1
#include "fda_state_narrow.inc"
