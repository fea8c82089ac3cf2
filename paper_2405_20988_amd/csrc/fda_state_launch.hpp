// Launchers of the state kernel; each lives in its own translation unit (one per slab type,
// cell type and half of the worker-slot counts) so that the instantiations compile in parallel.
// prm == nullptr: only raise the kernel's dynamic-LDS limit to `lds`.
// Returns hipErrorInvalidValue when no kernel is instantiated for (KC, LR).
#pragma once
#include <hip/hip_runtime.h>

#include "fda_kernels.hpp"

namespace fda {
// worker slots per workgroup that have a kernel; sketch-row slots are 1..kMaxLR
constexpr int kKCSet[] = {1, 2, 3, 4, 5, 6, 8};
constexpr int kMaxLR = 8;

#define FDA_DECLARE_LAUNCHER(name) \
  hipError_t name(int KC, int LR, const StateParams* prm, size_t lds, hipStream_t st)
FDA_DECLARE_LAUNCHER(launch_state_f32_fx_lo);
FDA_DECLARE_LAUNCHER(launch_state_f32_fx_hi);
FDA_DECLARE_LAUNCHER(launch_state_f32_f64_lo);
FDA_DECLARE_LAUNCHER(launch_state_f32_f64_hi);
FDA_DECLARE_LAUNCHER(launch_state_bf16_fx_lo);
FDA_DECLARE_LAUNCHER(launch_state_bf16_fx_hi);
FDA_DECLARE_LAUNCHER(launch_state_bf16_f64_lo);
FDA_DECLARE_LAUNCHER(launch_state_bf16_f64_hi);
}  // namespace fda
