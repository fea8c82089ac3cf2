// State kernels: fda::bf16_t slab, fp64 sketch cells, worker slots 1..4.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_FX false
#define FDA_TU_HI 0
#define FDA_TU_NAME launch_state_bf16_f64_lo
#include "fda_state_tu.inc"
