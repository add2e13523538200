// Device-side helpers shared by the kernel files of the stage-level partition search (value
// limits, address-space casts, the atomic fold, wave broadcasts, input limits).
#pragma once

#include "rannc_dp_internal.h"

#include "../../include/rannc_dp.h"

namespace rannc {

template <typename VT> struct Lim;
template <> struct Lim<uint32_t> { static constexpr uint32_t inf = 0xFFFFFFFFu; };
template <> struct Lim<uint64_t> { static constexpr uint64_t inf = 0x7FFFFFFFFFFFFFFFull; };

template <typename VT> __device__ __forceinline__ VT vmax(VT a, VT b) { return a > b ? a : b; }
template <typename VT> __device__ __forceinline__ VT vmin(VT a, VT b) { return a < b ? a : b; }

// Pointers that are read out of a descriptor in memory are generic to the compiler, and generic
// (FLAT) loads count against the 4-bit LDS/scalar counter: at most 15 of them can be in flight per
// wave.  Everything the library addresses is device memory, so the hot kernels say so and get
// GLOBAL loads, which have 63 in flight.
#define RANNC_GLOBAL __attribute__((address_space(1)))
template <typename T> __device__ __forceinline__ T RANNC_GLOBAL *gptr(T *p) { return (T RANNC_GLOBAL *)p; }

template <typename VT> __device__ __forceinline__ void global_min(VT RANNC_GLOBAL *p, VT v) {
  (void)__hip_atomic_fetch_min(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t lane_bcast(uint32_t v, int q) {
  return (uint32_t)__builtin_amdgcn_readlane((int)v, q);
}
__device__ __forceinline__ uint64_t lane_bcast(uint64_t v, int q) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, q);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), q);
  return ((uint64_t)hi << 32) | lo;
}

static constexpr uint64_t kSumLimit = 1ull << 62;
static constexpr uint64_t kCutLimit = (kSumLimit - 1) / 1000;  // largest bytes of a cut: 1000 * bytes < 2^62

// Time in ns to send `bytes` at `bw` bytes per microsecond from one replica (the communication term
// of a stage's execution time, Sec. III-C); flags as in the prefix sums.  With r replicas each
// sends 1/r of it: ceil(1000*bytes / (r*bw)) = ceil(ceil(1000*bytes / bw) / r), so the per-cut
// value is all the table builder needs.
__device__ __forceinline__ uint64_t cut_time(int64_t bytes, int64_t bw, int &flags) {
  if (bytes < 0) { flags |= 1; bytes = 0; }
  uint64_t u = (uint64_t)bytes;
  if (u > kCutLimit) { flags |= 2; u = kCutLimit; }
  return (u * 1000ull + (uint64_t)bw - 1) / (uint64_t)bw;
}
static constexpr int kNoRow = 0x7fffffff;

// Split-objective level kernel: waves per workgroup, and the smallest work item the adaptive work
// list makes for it (rows of one chunk); the work-list kernel needs both.
constexpr int kSplitWaves = 8;
constexpr int kSplitMinRows = 4;  // smallest work item the adaptive work list makes (rows of one chunk)

}  // namespace rannc
