// Device-side helpers shared by the kernel files of the stage-level partition search (value
// limits, address-space casts, the atomic fold, wave broadcasts, input limits).
#pragma once

#include "rannc_dp_internal.h"

#include "../../include/rannc_dp.h"

namespace rannc {

template <typename VT> struct Lim;
template <> struct Lim<uint32_t> { static constexpr uint32_t inf = 0xFFFFFFFFu; };
// 64-bit tables: "no plan" is the bit pattern of +infinity in double precision, above every value
// a search can form (they stay below 2^62).  Bit patterns below it, read as doubles, are
// non-negative finite numbers (normal or denormal, never NaN) whose order is the order of the
// integers, so the maximum and minimum of two 64-bit values are ONE double-precision instruction
// each instead of a 64-bit compare and four selects.  The boundary still reports INT64_MAX.
template <> struct Lim<uint64_t> { static constexpr uint64_t inf = 0x7FF0000000000000ull; };

template <typename VT> __device__ __forceinline__ VT vmax(VT a, VT b) { return a > b ? a : b; }
template <typename VT> __device__ __forceinline__ VT vmin(VT a, VT b) { return a < b ? a : b; }
// (inline assembly: the compiler's own double-precision maximum first rewrites each operand to
// quiet signalling NaNs, which cannot occur here, at three instructions instead of one; double
// precision denormals are always enabled on this target)
template <> __device__ __forceinline__ uint64_t vmax<uint64_t>(uint64_t a, uint64_t b) {
  uint64_t r;
  asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
template <> __device__ __forceinline__ uint64_t vmin<uint64_t>(uint64_t a, uint64_t b) {
  uint64_t r;
  asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// maximum with a wave-uniform first operand that lives in scalar registers
template <typename VT> __device__ __forceinline__ VT vmax_su(VT a_uniform, VT b) { return vmax(a_uniform, b); }
template <> __device__ __forceinline__ uint64_t vmax_su<uint64_t>(uint64_t a_uniform, uint64_t b) {
  uint64_t r;
  asm("v_max_f64 %0, %1, %2" : "=v"(r) : "s"(a_uniform), "v"(b));
  return r;
}

// Pointers that are read out of a descriptor in memory are generic to the compiler, and generic
// (FLAT) loads count against the 4-bit LDS/scalar counter: at most 15 of them can be in flight per
// wave.  Everything the library addresses is device memory, so the hot kernels say so and get
// GLOBAL loads, which have 63 in flight.
#define RANNC_GLOBAL __attribute__((address_space(1)))
template <typename T> __device__ __forceinline__ T RANNC_GLOBAL *gptr(T *p) { return (T RANNC_GLOBAL *)p; }

template <typename VT> __device__ __forceinline__ void global_min(VT RANNC_GLOBAL *p, VT v) {
  (void)__hip_atomic_fetch_min(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every global load
// and store the wave has in flight (its fence covers global memory); where the waves exchange data
// through LDS alone, that wait puts a memory round trip in front of every barrier.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

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
