// Mean-state kernels: float slab, fp64 cells.
#define FDA_TU_TYPE float
#define FDA_TU_BATCH fda::kMeanBatchF32
#define FDA_TU_CELL fda::kCellF64
#define FDA_TU_NAME launch_mean_f32_f64
#include "fda_mean.inc"
