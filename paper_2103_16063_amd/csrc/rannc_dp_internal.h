// Internal declarations shared by the host orchestration and the gfx950 kernels of the
// stage-level partition search.  Not part of the public ABI (see include/rannc_dp.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rannc {

// ---------------------------------------------------------------------------------------
// Table layout in HBM.
//
// Indices follow the recurrence of Sec. III-C: a stage holds blocks i+1..j (0 <= i < j <= N)
// and runs on r = d - d' replicas.  The level kernel keeps one output column j per lane, so
// every table that is indexed by j is stored with j fastest: a wavefront then reads 64
// consecutive columns of one (i, r) row with one coalesced 256-byte (32-bit values) or
// 512-byte (64-bit values) request.
//
// Columns are addressed by jj = j-1 and grouped in chunks of 64.  The row of predecessor i
// covers the chunks that can hold a j > i, i.e. chunks g(i) = i/64 .. nch-1, so each row
// starts on a chunk boundary (rows stay 256-byte aligned) and has
//     row_len(i) = 64 * (nch - i/64)         entries (nch = ceil(N/64)).
// Entries with jj < i or jj >= N are padding: never written, never read.
//
//   rmin[rows_before(i) + (jj - 64*(i/64))]                uint8: smallest r whose stage fits
//                                                          memory (the m <= M rule), 255 = none
//   cost[rows_before(i)*D + (r-1)*row_len(i) + (jj - 64*(i/64))]
//                                                          stage time h(i,j,r); INF if r < rmin
//   V[(s-1)*(N+1)*DP + j*DP + (d-1)]                       level s >= 1, DP = 8/16/32/64 >= D;
//                                                          entries with d > D hold 0
//
// The d-fastest layout of V makes the row V[s-1][i][.] one contiguous, wave-uniform read.
// ---------------------------------------------------------------------------------------

__host__ __device__ inline int64_t row_len(int nch, int i) { return 64LL * (nch - (i >> 6)); }

// sum of row_len(i') over i' < i
__host__ __device__ inline int64_t rows_before(int nch, int i) {
  const int64_t g = i >> 6;
  return 4096LL * (g * nch - g * (g - 1) / 2) + (int64_t)(i - 64 * g) * 64LL * (nch - g);
}

__host__ __device__ inline int dp_class(int D) { return D <= 8 ? 8 : D <= 16 ? 16 : D <= 32 ? 32 : 64; }

struct ProblemDev {
  int32_t N, D, S_eff, MB;
  int32_t DP;   // padded device dimension of a V row
  int32_t nch;  // 64-wide column chunks
  int32_t bits; // 32 or 64: width of the values in cost and V
  int32_t pad_;
  int64_t M;
  int64_t time_limit;          // limits.max_total_time_ns
  const int64_t *t, *p, *a;    // caller's inputs (DEVICE), N entries each
  int64_t *T, *P, *A;          // prefix sums, N+1 entries each
  uint8_t *rmin;
  void *cost;
  void *V;
  int32_t *ilo;                // [N+1], by j: smallest i whose stage (i,j) fits for some r <= D; j if none
  int32_t *status;             // RANNC_DP_PROBLEM_*
  int64_t *res;                // res[0] = opt (int64, INT64_MAX if none), res[1] = n_stages
};

struct LaunchShape {
  int nprob;     // problems in the launch (blockIdx.z runs over list[0..nprob))
  int max_N;     // largest N among them
  int max_nch;   // largest nch among them
  int max_D;
  int max_S_eff;
};

// Kernel launchers (rannc_dp_kernels.hip).  All enqueue on `st` and return the launch status.
hipError_t launch_prefix(const ProblemDev *d_probs, int Q, hipStream_t st);
hipError_t launch_fill(const ProblemDev *d_probs, int Q, hipStream_t st);
hipError_t launch_build(const ProblemDev *d_probs, const int32_t *d_list, const LaunchShape &sh,
                        int bits, int DP, hipStream_t st);
hipError_t launch_level_merge(const ProblemDev *d_probs, const int32_t *d_list,
                              const LaunchShape &sh, int bits, int DP, int s, int i_steps,
                              hipStream_t st);
hipError_t launch_level_scan(const ProblemDev *d_probs, const int32_t *d_list,
                             const LaunchShape &sh, int bits, int s, int write_v, int32_t *arg_i,
                             int32_t *arg_d, hipStream_t st);
hipError_t launch_select(const ProblemDev *d_probs, int Q, int64_t *d_opt, int32_t *d_n_stages,
                         int64_t *d_est, int32_t *d_status, hipStream_t st);
hipError_t launch_traceback(const ProblemDev *d_probs, int Q, int plan_stride, int32_t *d_stage_end,
                            int32_t *d_replicas, hipStream_t st);
hipError_t launch_export(const ProblemDev *d_probs, int q, int which, const ProblemDev &host_copy,
                         void *d_dst, hipStream_t st);

}  // namespace rannc
