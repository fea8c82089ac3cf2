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
// 32-bit-cell pass: worker slots KC in kKCSet, row slots LR in 1..kMaxLR, KC * LR <= kMaxSlots.
// Kernels with sign-split LDS rows exist for the even KC, kernels with plain rows for KC <= 2 (with
// more slots, half the slots per workgroup and split rows need the same LDS and less work).
constexpr int kKCSet[] = {1, 2, 4, 6, 8};
constexpr int kMaxLR = 8;
constexpr int kMaxSlots = 32;
constexpr bool narrow_kernel_exists(int KC, bool split) { return split ? KC % 2 == 0 : KC <= 2; }
// ... and kernels for a table with placed rows (fields of kPlacedFieldBits bits) for the even KC: there a
// field is a bucket number in a whole group of rows
constexpr bool placed_kernel_exists(int KC) { return KC % 2 == 0; }
// fallback passes (8-byte cells)
constexpr int kWideKCSet[] = {1, 2, 4};
constexpr int kWideLRSet[] = {1, 2, 4, 8};

// FB: bits per field of the tabulated hash (field_bits_for(m): 11 or 16; kPlacedFieldBits with placed rows); split: sign-split LDS rows
// (even worker-slot counts only)
#define FDA_NARROW_LAUNCHER(t, kc) \
  hipError_t launch_narrow_##t##_kc##kc(int LR, int FB, int split, const StateParams* prm, size_t lds, hipStream_t st)
#define FDA_WIDE_LAUNCHER(t, c) \
  hipError_t launch_wide_##t##_##c(int KC, int LR, const StateParams* prm, size_t lds, hipStream_t st)
FDA_NARROW_LAUNCHER(f32, 1); FDA_NARROW_LAUNCHER(f32, 2); FDA_NARROW_LAUNCHER(f32, 4);
FDA_NARROW_LAUNCHER(f32, 6); FDA_NARROW_LAUNCHER(f32, 8);
FDA_NARROW_LAUNCHER(bf16, 1); FDA_NARROW_LAUNCHER(bf16, 2); FDA_NARROW_LAUNCHER(bf16, 4);
FDA_NARROW_LAUNCHER(bf16, 6); FDA_NARROW_LAUNCHER(bf16, 8);
FDA_WIDE_LAUNCHER(f32, i64); FDA_WIDE_LAUNCHER(f32, f64);
FDA_WIDE_LAUNCHER(bf16, i64); FDA_WIDE_LAUNCHER(bf16, f64);

template <typename T, int KC, int LR, int CELL, int FB, bool SPLIT = false>
hipError_t launch_state_kernel(const StateParams* prm, size_t lds, hipStream_t st) {
  auto kern = state_kernel<T, KC, LR, CELL, FB, SPLIT>;
  if (prm == nullptr)
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(kern, dim3(prm->G * prm->R * prm->P), dim3(kStateThreads), lds, st, *prm);
  return hipGetLastError();
}
}  // namespace fda
