// Launchers of the state kernel.  The instantiations are spread over many translation units so
// that they compile in parallel: one per (slab type, worker-slot count) for the 32-bit-cell
// pass every call runs, one per (slab type, cell kind) for the two fallback passes, which only
// come in a few shapes.
// prm == nullptr: only raise the kernel's dynamic-LDS limit to `lds`.
// Returns hipErrorInvalidValue when no kernel is instantiated for the shape.
#pragma once
#include <hip/hip_runtime.h>

#include "fda_kernels.hpp"

namespace fda {
// 32-bit-cell pass: worker slots KC in kKCSet, row slots LR in 1..kMaxLR, KC * LR <= kMaxSlots
constexpr int kKCSet[] = {1, 2, 3, 4, 5, 6, 8};
constexpr int kMaxLR = 8;
constexpr int kMaxSlots = 32;
// fallback passes (8-byte cells)
constexpr int kWideKCSet[] = {1, 2, 4};
constexpr int kWideLRSet[] = {1, 2, 4, 8};

// FB: bits per field of the tabulated hash (field_bits_for(m)): 11 or 16
#define FDA_NARROW_LAUNCHER(t, kc) \
  hipError_t launch_narrow_##t##_kc##kc(int LR, int FB, const StateParams* prm, size_t lds, hipStream_t st)
#define FDA_WIDE_LAUNCHER(t, c) \
  hipError_t launch_wide_##t##_##c(int KC, int LR, const StateParams* prm, size_t lds, hipStream_t st)
FDA_NARROW_LAUNCHER(f32, 1); FDA_NARROW_LAUNCHER(f32, 2); FDA_NARROW_LAUNCHER(f32, 3);
FDA_NARROW_LAUNCHER(f32, 4); FDA_NARROW_LAUNCHER(f32, 5); FDA_NARROW_LAUNCHER(f32, 6);
FDA_NARROW_LAUNCHER(f32, 8);
FDA_NARROW_LAUNCHER(bf16, 1); FDA_NARROW_LAUNCHER(bf16, 2); FDA_NARROW_LAUNCHER(bf16, 3);
FDA_NARROW_LAUNCHER(bf16, 4); FDA_NARROW_LAUNCHER(bf16, 5); FDA_NARROW_LAUNCHER(bf16, 6);
FDA_NARROW_LAUNCHER(bf16, 8);
FDA_WIDE_LAUNCHER(f32, i64); FDA_WIDE_LAUNCHER(f32, f64);
FDA_WIDE_LAUNCHER(bf16, i64); FDA_WIDE_LAUNCHER(bf16, f64);

template <typename T, int KC, int LR, int CELL, int FB>
hipError_t launch_state_kernel(const StateParams* prm, size_t lds, hipStream_t st) {
  auto kern = state_kernel<T, KC, LR, CELL, FB>;
  if (prm == nullptr)
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(prm->G * prm->R * prm->P), dim3(kStateThreads), lds, st, *prm);
  return hipGetLastError();
}
}  // namespace fda
