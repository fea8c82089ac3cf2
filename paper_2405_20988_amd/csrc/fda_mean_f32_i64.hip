// Mean-state kernels: float slab, 64-bit integer cells.
#define FDA_TU_TYPE float
#define FDA_TU_BATCH fda::kMeanBatchF32
#define FDA_TU_CELL fda::kCellI64
#define FDA_TU_NAME launch_mean_f32_i64
#include "fda_mean.inc"
