// Mean-state kernels: bf16 slab, fp64 cells.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_BATCH fda::kMeanBatchBF16
#define FDA_TU_CELL fda::kCellF64
#define FDA_TU_NAME launch_mean_bf16_f64
#include "fda_mean.inc"
