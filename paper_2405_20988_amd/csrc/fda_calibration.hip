// Measurement aids of the FDA library (no part of the method): kernels of known traffic and known
// LDS work, so that the rates the FDA kernels are judged against -- what this chip streams from
// and to HBM with 16-byte accesses, what its LDS sustains in atomic additions -- are measured by the
// same library, in the same run, instead of being quoted.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "fda.h"

namespace {

constexpr int kThreads = 256;
constexpr int kLdsThreads = 512;
constexpr int kLdsWords = 36864;            // 144 KiB of cells, the size class of the sketch in LDS

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- streaming kernels: one 16-byte vector per lane and access; workgroup b owns the contiguous range
// [b * per, (b + 1) * per) of vectors and walks it 8 x 4 KiB per trip; NT: nontemporal hint ----
template <bool NT>
__device__ __forceinline__ u32x4 ld(const u32x4* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT>
__device__ __forceinline__ void st(u32x4* p, u32x4 v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}
constexpr int kUnroll = 8;

template <bool NT>
__global__ void __launch_bounds__(kThreads)
calib_read_kernel(const u32x4* __restrict__ src, long long nvec, uint32_t* __restrict__ sink) {
  const long long per = (nvec + gridDim.x - 1) / gridDim.x;
  const long long beg = (long long)blockIdx.x * per, end = beg + per < nvec ? beg + per : nvec;
  long long i = beg + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + (kUnroll - 1) * kThreads < end; i += kUnroll * kThreads) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int q = 0; q < kUnroll; ++q) v[q] = ld<NT>(src + i + q * kThreads);
#pragma unroll
    for (int q = 0; q < kUnroll; ++q) acc ^= v[q];
  }
  for (; i < end; i += kThreads) acc ^= ld<NT>(src + i);
  const uint32_t folded = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (folded == 0x9e3779b9u) *sink = folded;           // keeps the loads alive; practically never taken
}

template <bool NT>
__global__ void __launch_bounds__(kThreads)
calib_write_kernel(u32x4* __restrict__ dst, long long nvec, uint32_t value) {
  const long long per = (nvec + gridDim.x - 1) / gridDim.x;
  const long long beg = (long long)blockIdx.x * per, end = beg + per < nvec ? beg + per : nvec;
  const u32x4 v = {value, value, value, value};
  for (long long i = beg + threadIdx.x; i < end; i += kThreads) st<NT>(dst + i, v);
}

template <bool NT>
__global__ void __launch_bounds__(kThreads)
calib_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, long long nvec) {
  const long long per = (nvec + gridDim.x - 1) / gridDim.x;
  const long long beg = (long long)blockIdx.x * per, end = beg + per < nvec ? beg + per : nvec;
  long long i = beg + threadIdx.x;
  for (; i + (kUnroll - 1) * kThreads < end; i += kUnroll * kThreads) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int q = 0; q < kUnroll; ++q) v[q] = ld<NT>(src + i + q * kThreads);
#pragma unroll
    for (int q = 0; q < kUnroll; ++q) st<NT>(dst + i + q * kThreads, v[q]);
  }
  for (; i < end; i += kThreads) st<NT>(dst + i, ld<NT>(src + i));
}

// ---- LDS atomic additions --------------------------------------------------------------------
// Every lane holds eight cell indices, fixed for the whole launch, and re-issues one atomic addition to
// each of them per iteration: almost no vector-ALU work, so the rate is the LDS's own.
//   OP       0: 32-bit integer add that returns the old value   1: 32-bit integer add, no return
//            2: 64-bit integer add   3: fp64 add   4: fp32 add   5: 64-bit integer add that returns the old value
//            6 / 7: no addition at all, a plain read of 8 / 16 bytes (what a gather from LDS would cost; the
//               cell moves by a fixed step per iteration so that the reads stay in the loop)
//   PATTERN  0: every lane an independent random cell
//            1: lane t the cell t (no two lanes of an instruction on one bank)
//            2/3/4/5: groups of 4/8/16/32 lanes share a random group of consecutive cells, lane q of
//               the group on cell q -- the layout [bucket][worker] addressed by (coordinate, worker) lanes
template <int OP, int PATTERN>
__global__ void __launch_bounds__(kLdsThreads)
calib_lds_kernel(int iters, uint32_t* __restrict__ sink) {
  extern __shared__ __align__(16) unsigned char raw[];
  uint32_t* words = reinterpret_cast<uint32_t*>(raw);
  const int tid = threadIdx.x, lane = tid & 63;
  for (int t = tid; t < kLdsWords; t += kLdsThreads) words[t] = 0u;
  __syncthreads();
  constexpr int kWordsPerCell = OP == 7 ? 4 : (OP == 2 || OP == 3 || OP == 5 || OP == 6) ? 2 : 1;
  constexpr int kCells = kLdsWords / kWordsPerCell;
  uint32_t idx[8];
  uint32_t s = (uint32_t)tid * 2654435761u + blockIdx.x * 97u + 12345u;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    s = s * 1664525u + 1013904223u;
    const uint32_t r = s >> 8;
    if constexpr (PATTERN == 0) {
      idx[q] = r % kCells;
    } else if constexpr (PATTERN == 1) {
      idx[q] = (uint32_t)(tid + q * 1021) % kCells;
    } else {
      constexpr int G = PATTERN == 2 ? 4 : PATTERN == 3 ? 8 : PATTERN == 4 ? 16 : 32;
      const uint32_t rg = (uint32_t)__shfl((int)r, lane & ~(G - 1), 64);
      idx[q] = (rg % (kCells / (G + 1))) * (G + 1) + (uint32_t)(lane & (G - 1));   // odd group stride
    }
  }
  uint32_t seen = 0u;
  unsigned long long seen64 = 0ull;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if constexpr (OP == 0) seen |= atomicAdd(words + idx[q], 3u);
      if constexpr (OP == 1) atomicAdd(words + idx[q], 3u);
      if constexpr (OP == 2) atomicAdd(reinterpret_cast<unsigned long long*>(raw) + idx[q], 3ull);
      if constexpr (OP == 3) atomicAdd(reinterpret_cast<double*>(raw) + idx[q], 1.0);
      if constexpr (OP == 4) atomicAdd(reinterpret_cast<float*>(raw) + idx[q], 1.0f);
      if constexpr (OP == 5) seen64 |= atomicAdd(reinterpret_cast<unsigned long long*>(raw) + idx[q], 3ull);
      if constexpr (OP == 6 || OP == 7) {
        idx[q] += 1021u;                                   // below kCells: one conditional subtraction wraps
        idx[q] = idx[q] >= (uint32_t)kCells ? idx[q] - (uint32_t)kCells : idx[q];
        if constexpr (OP == 6) {
          seen64 += reinterpret_cast<const unsigned long long*>(raw)[idx[q]];
        } else {
          const u32x4 v = reinterpret_cast<const u32x4*>(raw)[idx[q]];
          seen += v.x ^ v.y;
          seen64 += v.z ^ v.w;
        }
      }
    }
  }
  __syncthreads();
  uint32_t acc = (seen & 1u) + (uint32_t)(seen64 >> 63);
  for (int t = tid; t < kLdsWords; t += kLdsThreads) acc += words[t];
  if (acc == 0x9e3779b9u) *sink = acc;                 // keeps the additions alive
}

thread_local char g_calib_err[256] = "";

template <int OP>
hipError_t launch_lds(int pattern, int blocks, int iters, uint32_t* sink, hipStream_t st, bool setup) {
  const size_t lds = (size_t)kLdsWords * 4;
#define FDA_PAT(p)                                                                                    \
  case p:                                                                                             \
    if (setup)                                                                                        \
      return hipFuncSetAttribute(reinterpret_cast<const void*>(calib_lds_kernel<OP, p>),              \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);               \
    hipLaunchKernelGGL((calib_lds_kernel<OP, p>), dim3(blocks), dim3(kLdsThreads), lds, st, iters, sink); \
    return hipGetLastError()
  switch (pattern) { FDA_PAT(0); FDA_PAT(1); FDA_PAT(2); FDA_PAT(3); FDA_PAT(4); FDA_PAT(5); }
#undef FDA_PAT
  return hipErrorInvalidValue;
}

hipError_t launch_lds_any(int op, int pattern, int blocks, int iters, uint32_t* sink, hipStream_t st, bool setup) {
  switch (op) {
    case 0: return launch_lds<0>(pattern, blocks, iters, sink, st, setup);
    case 1: return launch_lds<1>(pattern, blocks, iters, sink, st, setup);
    case 2: return launch_lds<2>(pattern, blocks, iters, sink, st, setup);
    case 3: return launch_lds<3>(pattern, blocks, iters, sink, st, setup);
    case 4: return launch_lds<4>(pattern, blocks, iters, sink, st, setup);
    case 5: return launch_lds<5>(pattern, blocks, iters, sink, st, setup);
    case 6: return launch_lds<6>(pattern, blocks, iters, sink, st, setup);
    case 7: return launch_lds<7>(pattern, blocks, iters, sink, st, setup);
  }
  return hipErrorInvalidValue;
}

}  // namespace

extern "C" {

int fda_calib_stream(int mode, const void* src, void* dst, size_t bytes, int reps, void* stream,
                     double* ms_per_rep) {
  if (ms_per_rep == nullptr || reps < 1 || bytes < 16 || mode < 0 || mode > 6 || mode == 3) return FDA_EINVAL;
  const bool nt = mode >= 4;
  mode &= 3;
  if ((mode != 1 && src == nullptr) || dst == nullptr) return FDA_EINVAL;
  if (reinterpret_cast<uintptr_t>(dst) % 16 != 0 || (src && reinterpret_cast<uintptr_t>(src) % 16 != 0))
    return FDA_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return FDA_EHIP;
  const long long nvec = (long long)(bytes / 16);
  long long blocks = (nvec + kThreads * kUnroll - 1) / (kThreads * kUnroll);
  if (blocks > (long long)cus * 64) blocks = (long long)cus * 64;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return FDA_EHIP;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return FDA_EHIP; }
  int rc = FDA_OK;
  for (int r = -1; r < reps && rc == FDA_OK; ++r) {       // one untimed launch first
    if (r == 0 && hipEventRecord(e0, st) != hipSuccess) rc = FDA_EHIP;
    const dim3 g((unsigned)blocks), b(kThreads);
    const u32x4* s4 = static_cast<const u32x4*>(src);
    u32x4* d4 = static_cast<u32x4*>(dst);
    if (mode == 0 && nt) hipLaunchKernelGGL(calib_read_kernel<true>, g, b, 0, st, s4, nvec, static_cast<uint32_t*>(dst));
    else if (mode == 0) hipLaunchKernelGGL(calib_read_kernel<false>, g, b, 0, st, s4, nvec, static_cast<uint32_t*>(dst));
    else if (mode == 1 && nt) hipLaunchKernelGGL(calib_write_kernel<true>, g, b, 0, st, d4, nvec, 0x3f800000u);
    else if (mode == 1) hipLaunchKernelGGL(calib_write_kernel<false>, g, b, 0, st, d4, nvec, 0x3f800000u);
    else if (nt) hipLaunchKernelGGL(calib_copy_kernel<true>, g, b, 0, st, s4, d4, nvec);
    else hipLaunchKernelGGL(calib_copy_kernel<false>, g, b, 0, st, s4, d4, nvec);
    if (hipGetLastError() != hipSuccess) rc = FDA_EHIP;
  }
  float ms = 0.0f;
  if (rc == FDA_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                       hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = FDA_EHIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == FDA_OK) *ms_per_rep = (double)ms / reps;
  return rc;
}

int fda_calib_lds_atomics(int op, int pattern, int iters, void* sink_dev, void* stream,
                          double* lane_ops_per_clock_per_cu, double* clock_ghz) {
  if (lane_ops_per_clock_per_cu == nullptr || sink_dev == nullptr || iters < 1 || op < 0 || op > 7 ||
      pattern < 0 || pattern > 5)
    return FDA_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int dev = 0, cus = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess || khz <= 0)
    return FDA_EHIP;
  uint32_t* sink = static_cast<uint32_t*>(sink_dev);
  if (launch_lds_any(op, pattern, cus, iters, sink, st, true) != hipSuccess) return FDA_EHIP;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return FDA_EHIP;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return FDA_EHIP; }
  int rc = FDA_OK;
  if (launch_lds_any(op, pattern, cus, 8, sink, st, false) != hipSuccess) rc = FDA_EHIP;      // untimed
  if (rc == FDA_OK && hipEventRecord(e0, st) != hipSuccess) rc = FDA_EHIP;
  if (rc == FDA_OK && launch_lds_any(op, pattern, cus, iters, sink, st, false) != hipSuccess) rc = FDA_EHIP;
  float ms = 0.0f;
  if (rc == FDA_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                       hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = FDA_EHIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == FDA_OK) {
    const double ghz = (double)khz * 1e-6;
    const double ops = (double)cus * kLdsThreads * 8.0 * (double)iters;
    *lane_ops_per_clock_per_cu = ops / ((double)ms * 1e-3) / cus / (ghz * 1e9);
    if (clock_ghz != nullptr) *clock_ghz = ghz;
  }
  return rc;
}

}  // extern "C"
