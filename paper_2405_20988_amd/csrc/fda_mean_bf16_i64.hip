// Mean-state kernels: bf16 slab, 64-bit integer cells.
#define FDA_TU_TYPE fda::bf16_t
#define FDA_TU_BATCH fda::kMeanBatchBF16
#define FDA_TU_CELL fda::kCellI64
#define FDA_TU_NAME launch_mean_bf16_i64
#include "fda_mean.inc"
