// State kernels: fda::bf16_t slab, 64-bit integer sketch cells, worker slots 5, 6, 8.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_FX true
#define FDA_TU_HI 1
#define FDA_TU_NAME launch_state_bf16_fx_hi
#include "fda_state_tu.inc"
