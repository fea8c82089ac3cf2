// State kernels: float slab, fp64 sketch cells, worker slots 1..4.
#define FDA_TU_TYPE float
#define FDA_TU_FX false
#define FDA_TU_HI 0
#define FDA_TU_NAME launch_state_f32_f64_lo
#include "fda_state_tu.inc"
