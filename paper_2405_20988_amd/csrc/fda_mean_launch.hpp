// Launchers of the mean-state kernel, one translation unit per (slab type, cell kind).
// prm == nullptr: only raise the kernels' dynamic-LDS limit to `lds`.
// Returns hipErrorInvalidValue when no kernel is instantiated for the number of row slots.
#pragma once
#include <hip/hip_runtime.h>

#include "fda_mean_kernel.hpp"

namespace fda {
constexpr int kMeanMaxLR = 8;                // sketch-row slots of one workgroup: 1..8
constexpr int kMeanBatchF32 = 4;             // slab rows per batch: 4 x 16 bytes per lane ...
constexpr int kMeanBatchBF16 = 4;            // ... or 4 x 8 bytes

// FB: bits per field of the tabulated hash (field_bits_for(m)): 11 or 16
#define FDA_MEAN_LAUNCHER(t, c) \
  hipError_t launch_mean_##t##_##c(int LR, int FB, const MeanParams* prm, size_t lds, hipStream_t st)
FDA_MEAN_LAUNCHER(f32, i64); FDA_MEAN_LAUNCHER(f32, f64);
FDA_MEAN_LAUNCHER(bf16, i64); FDA_MEAN_LAUNCHER(bf16, f64);

template <typename T, int KB, int LR, int CELL, int FB>
hipError_t launch_mean_kernel(const MeanParams* prm, size_t lds, hipStream_t st) {
  auto kern = mean_state_kernel<T, KB, LR, CELL, FB>;
  if (prm == nullptr)
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(prm->R * prm->P), dim3(kStateThreads), lds, st, *prm);
  return hipGetLastError();
}
}  // namespace fda
