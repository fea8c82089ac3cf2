// State kernels: fda::bf16_t slab, fp64 sketch cells, worker slots 5, 6, 8.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_FX false
#define FDA_TU_HI 1
#define FDA_TU_NAME launch_state_bf16_f64_hi
#include "fda_state_tu.inc"
