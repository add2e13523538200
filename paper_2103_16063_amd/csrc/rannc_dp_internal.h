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
// the stage-time table is cut into UNITS: unit (i, c) holds predecessor row i for the 64
// columns jj = j-1 in [64c, 64c+63], all D replica counts, as a contiguous block
//
//     cost[(unit(i,c) * D + (r-1)) * 64 + (jj - 64c)]         stage time h(i,j,r), INF if r < rmin
//     rmin[ unit(i,c) * 64      + (jj - 64c)]                 uint8: smallest r whose stage fits
//                                                             memory (the m <= M rule), 255 = none
//
// so that one wavefront reads a unit with D coalesced 256-byte (32-bit values) or 512-byte
// (64-bit) requests out of one contiguous 16 KiB / 32 KiB region.  Row i has units for the
// chunks that can hold a j > i, c = i/64 .. nch-1 (nch = ceil(N/64)); units are numbered row by
// row.  Lanes with jj < i or jj >= N are padding: never written, never read.
//
//     V[(s-1)*(N+1)*DP + j*DP + (d-1)]     level s >= 1, DP = 8/16/32/64 >= D; entries d > D hold 0
//
// The d-fastest layout of V makes the row V[s-1][i][.] one contiguous, wave-uniform read.
// ---------------------------------------------------------------------------------------

// number of units in rows i' < i
__host__ __device__ inline int64_t units_before(int nch, int i) {
  const int64_t g = i >> 6;
  return 64LL * (g * nch - g * (g - 1) / 2) + (int64_t)(i - 64 * g) * (nch - g);
}
__host__ __device__ inline int64_t unit_index(int nch, int i, int c) {
  return units_before(nch, i) + (c - (i >> 6));
}

// upper bound on the number of work items ("runs") of one level: every chunk's rows cut into
// groups of at least 4 rows (chunk c has at most 64(c+1) rows), or, for a search of at most
// kSplitSmallRows rows, into items of one or two rows (split_rows_per_item)
constexpr int kSplitSmallRows = 1024;
__host__ __device__ inline int64_t max_runs(int nch) {
  const int64_t by4 = 8LL * nch * (nch + 1), rows = 32LL * nch * (nch + 1);
  const int64_t small = rows < kSplitSmallRows + nch ? rows : kSplitSmallRows + nch;
  return by4 > small ? by4 : small;
}

// Sorted-merge level kernel: waves per work item; a wave takes 1, 2, 4, ... of the item's rows.  The
// host sizes the grid for items of 16 rows when the searches of a launch together hold at least
// kMergeRows16From rows (unpruned), of 8 from kMergeRows8From, of 4 below.
constexpr int kMergeWaves = 4;
constexpr int kMergeMinRows = 4;
constexpr int kMergeRows8From = 6144;
constexpr int kMergeRows16From = 16384;
// From this many rows in a launch on, a 32-bit search without a communication term has its stage
// times recomputed in the level kernel (RANNC_DP_ALGO_AUTO): the launch then runs many rounds of
// workgroups and is bound by throughput, where recomputing beats reading the table; below, the
// level is a single round bound by latency, where the shorter table kernel wins.
constexpr int kRecomputeRowsFrom = 32768;
// A launch over SEVERAL searches recomputes from far fewer rows on: it needs no stage-time table
// built in front, and measured ahead of the table form from 2 700 rows (outer driver at 192 blocks)
// upwards at every memory tightness, by 1 to 14 %; below (two or three small searches) the table form
// keeps its edge.
constexpr int kRecomputeRowsFromMany = 2048;

__host__ __device__ inline int dp_class(int D) { return D <= 8 ? 8 : D <= 16 ? 16 : D <= 32 ? 32 : 64; }

struct ProblemDev {
  int32_t N, D, S_eff, MB;
  int32_t DP;   // padded device dimension of a V row
  int32_t nch;  // 64-wide column chunks
  int32_t bits; // 32 or 64: width of the values in cost and V
  int32_t q;    // index of the problem in the caller's batch (outputs go there)
  int64_t M;
  int64_t time_limit;          // limits.max_total_time_ns
  const int64_t *t, *p, *a;    // caller's inputs (DEVICE), N entries each
  const int64_t *tb;           // caller's backward block times (DEVICE), or null: one time per block (min-max search)
  int64_t *TB;                 // prefix sums of tb, N+1 entries; null when tb is null
  void *costb;                 // backward stage-time table, layout of cost; null when tb is null
  void *VF, *VB;               // largest forward / backward stage time of the plan behind each V entry
                               // (layout of V); null when tb is null
  void *keys;                  // [DP][N+1] uint64: packed (value, i, d') winners of the level in flight;
                               // only with tb and a time bound the packing can hold, else null
  const int64_t *o;            // caller's bytes per cut (DEVICE), N entries, or null: no communication term
  int64_t bw;                  // bandwidth in bytes per microsecond (>= 1 when o is given)
  int64_t *T, *P, *A;          // prefix sums, N+1 entries each
  int64_t *C;                  // C[j] = ns to send the bytes of the cut after block j at one replica
                               // (C[0] = C[N] = 0), N+1 entries; null when o is null
  uint8_t *rmin;
  void *cost;
  void *V;
  uint8_t *ufit;               // per unit: 1 if any of its stages fits for some r <= D
  int32_t *wlo;                // [nch] smallest row i with a stage (i, j in chunk) that fits for some
                               // r <= D; 0x7fffffff if none
  int32_t *runs;               // runs[0] = count, then ((rows - 1) << 26 | c << 16 | first row) per work item
  int32_t *status;             // RANNC_DP_PROBLEM_*
  int64_t *res;                // res[0] = opt (int64, INT64_MAX if none), res[1] = n_stages
};

struct LaunchShape {
  int nprob;     // problems in the launch (blockIdx.z runs over them)
  int max_N;     // largest N among them
  int max_nch;   // largest nch among them
  int max_D;
  int max_S_eff;
};

// Kernel launchers (rannc_dp_kernels.hip, rannc_dp_split.hip, rannc_dp_compact.hip).  All enqueue on `st` and return the launch status.
// `probs` points at the first ProblemDev of the launch; problems of one launch are contiguous.
hipError_t launch_prefix(const ProblemDev *probs, int Q, hipStream_t st);
hipError_t launch_fill(const ProblemDev *probs, int Q, hipStream_t st);
// parts: 1 = fits-in-memory tables (rmin, ufit) and level 1 of V, 2 = the stage-time table, 3 = both
hipError_t launch_build(const ProblemDev *probs, const LaunchShape &sh, int bits, int DP, int parts, hipStream_t st);
hipError_t launch_windows(const ProblemDev *probs, const LaunchShape &sh, hipStream_t st);
// rows_per_item: > 0 fixed, 0 chosen on the device for the split-objective kernel, -1 for the
// sorted-merge kernel (then the smallest item size whose item count fits max_items)
// slots: workgroups of the level kernel that the device holds at a time
// paired: the list for the level kernel that recomputes the stage times (diagonal blocks as row pairs)
hipError_t launch_runs(const ProblemDev *probs, int Q, int rows_per_item, int max_items, int slots, bool paired,
                       hipStream_t st);
int merge_workgroups_per_cu(int bits, int DP, bool recompute);
int merge_rows_per_item(int rows_per_wave);
// rows_for_list: what launch_runs is to be given as rows_per_item (the size the host fixed, or -1)
int merge_grid_items(const LaunchShape &sh, int rows_per_item, int slots, bool paired, int *rows_for_list);
// rows of the searches of a launch if nothing is pruned (every chunk c holds rows 0 .. 64c+63)
int64_t merge_launch_rows(const LaunchShape &sh);
// recompute: the level kernel computes the stage times from the prefix sums instead of reading
// their table (32-bit values only)
// items: merge_grid_items of the launch, the value launch_runs was given
// host_one: for a launch over one search, a host copy of its descriptor (passed by value), or null
hipError_t launch_level_merge(const ProblemDev *probs, const LaunchShape &sh, int bits, int DP, int s,
                              bool recompute, int items, const ProblemDev *host_one, hipStream_t st);
// whole search of problems with N <= small_max_blocks() in one launch, one workgroup each
int small_max_blocks();
// direct: the stage times are recomputed from the prefix sums and no table is written (only where
// small_can_recompute says so, and only for searches without a communication term);
// max_total_time: the largest total time a search of the launch can have without being flagged
bool small_can_recompute(int bits, int DP, int64_t max_total_time);
hipError_t launch_solve_small(const ProblemDev *probs, int Q, int bits, int DP, bool direct, int64_t *d_opt,
                              int32_t *d_n_stages, int64_t *d_est, int32_t *d_status, hipStream_t st);
hipError_t launch_level_scan(const ProblemDev *probs, const LaunchShape &sh, int bits, int s,
                             int write_v, int32_t *arg_i, int32_t *arg_d, hipStream_t st);
// Algorithm 1 with forward and backward maxima carried separately (problems with tb != null):
// level 1 from the two tables, then one launch per level s >= 2.  write_v = 0: only the argmin
// arrays (canonical layout of ONE problem) are written.
hipError_t launch_split_level1(const ProblemDev *probs, const LaunchShape &sh, int bits, hipStream_t st);
hipError_t launch_level_split(const ProblemDev *probs, const LaunchShape &sh, int bits, int s, int write_v,
                              int32_t *arg_i, int32_t *arg_d, hipStream_t st);
// needs the key table and the work list made by launch_runs(..., split_rows_per_item(), ...); with
// 64-bit tables only for time bounds up to kSplitPackedMax (the packed winner holds 42 value bits)
constexpr int64_t kSplitPackedMax = (1LL << 42) - 2;
// rows per work item: 1 or 2 for a launch whose rows (unpruned) then still fit one round of workgroups
// (a short chain of rows per workgroup: the launch is bound by latency), else 0 = chosen on the
// device from the size of the windows (4, 8 or 16); the level launcher is given the same value
int split_rows_per_item(const LaunchShape &sh, int n_cus);
hipError_t launch_level_split_fast(const ProblemDev *probs, const LaunchShape &sh, int bits, int DP, int s,
                                   int rows_per_item, hipStream_t st);
hipError_t launch_select(const ProblemDev *probs, int Q, int64_t *d_opt, int32_t *d_n_stages,
                         int64_t *d_est, int32_t *d_status, hipStream_t st);
// d_levels: per problem (caller's order) the exact stage count to recover, 0 = the best one; or null
// lds_bytes > 0: the kernel that first copies what the walk reads into LDS; every problem of the
// launch must be a min-max search with traceback_lds_bytes(...) <= lds_bytes <= kTracebackLdsMax
constexpr int kTracebackLdsMax = 150 * 1024;
int64_t traceback_lds_bytes(int N, int DP, int S_eff, int bits);
// rec != null: the plan of the search that rec[0] names is also written behind the six words of rec
hipError_t launch_traceback(const ProblemDev *probs, int Q, int plan_stride, int32_t *d_stage_end,
                            int32_t *d_replicas, const int32_t *d_levels, int64_t lds_bytes, int64_t *rec,
                            hipStream_t st);
hipError_t launch_level_values(const ProblemDev *probs, int Q, int stride, int64_t *d_out, hipStream_t st);
// compaction step of the block-level phase on a chain of G groups (one workgroup).  Chains whose
// state fits LDS (kCompactLds groups) need only the listing in the workspace, longer ones keep
// their whole state there.
constexpr int kCompactLds = 1600;
// bytes of one index list: room for the next power of two above G (the bitonic listing pads to it)
constexpr size_t compact_order_bytes(int G) {
  size_t P = 1;
  while (P < (size_t)G) P <<= 1;
  return (P * 4 + 255) / 256 * 256;
}
constexpr size_t compact_workspace_bytes(int G) {
  const size_t a8 = (((size_t)G * 8 + 255) / 256) * 256, a4 = (((size_t)G * 4 + 255) / 256) * 256;
  return 2 * compact_order_bytes(G) + (G > kCompactLds ? 3 * a8 + 4 * a4 : 0);
}
hipError_t launch_compact(int G, int k, int64_t M, int max_walks, const int64_t *t, const int64_t *p,
                          const int64_t *a, void *ws, int32_t *n_out, int32_t *block_end, int64_t *t_out,
                          int64_t *p_out, int64_t *a_out, int32_t *status, hipStream_t st);
// outer driver: Algorithm 2's loops over the values of a solved batch, and the chosen plan packed
// behind the result record (rec: 6 int64 {q, S, bad status, 0, V, estimate}, then 2*stride int32)
hipError_t launch_form_stage_select(const ProblemDev *probs, int Q, int stride, int N, int n_nodes,
                                    int devices_per_node, const int32_t *pair_n, const int32_t *pair_mb,
                                    int32_t *levels, int64_t *rec, hipStream_t st);
hipError_t launch_export(const ProblemDev *prob, int which, int bits, void *d_dst, hipStream_t st);


}  // namespace rannc
