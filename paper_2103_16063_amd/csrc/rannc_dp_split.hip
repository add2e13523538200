// gfx950 kernels of Algorithm 1 as printed (RaNNC Sec. III-C): forward and backward maxima carried
// separately, candidates valued by their sum.  Level 1, the literal level kernel, the packed-key
// level kernel with its finalize step, and their launchers.  Plan recovery for this objective is
// part of the traceback kernel (rannc_dp_kernels.hip).
#include "rannc_dp_device.h"

namespace rannc {

// ---------------------------------------------------------------------------------------
// Algorithm 1 as printed: forward and backward maxima carried separately (problems with backward
// times).  A cell keeps V = f + b together with the pair (f, b) of the first candidate, in the
// scan order (i ascending, then d' ascending), that attains the smallest sum; only that pair is
// seen by the next level.  The sum of two maxima does not separate over the two sequences, so the
// sorted-merge form does not apply: every candidate is evaluated, one wave per (64 columns, d),
// a lane per column j, as in the literal scan kernel.
// ---------------------------------------------------------------------------------------
// Level 1: the single stage 1..j on d replicas.
template <typename VT>
__global__ __launch_bounds__(64) void split_level1_kernel(const ProblemDev *__restrict__ probs) {
  const ProblemDev &pr = probs[blockIdx.z];
  const int c = blockIdx.x, d = blockIdx.y + 1;
  if (c >= pr.nch || d > pr.D) return;
  const int lane = threadIdx.x, jj = 64 * c + lane;
  if (jj >= pr.N) return;
  const int D = pr.D, DP = pr.DP;
  const int64_t u = unit_index(pr.nch, 0, c);
  const int64_t e = (int64_t)(jj + 1) * DP + d - 1;
  if (d < (int)pr.rmin[u * 64 + lane]) return;  // stays "no plan"
  const VT f = ((const VT *)pr.cost)[(u * D + (d - 1)) * 64 + lane];
  const VT b = ((const VT *)pr.costb)[(u * D + (d - 1)) * 64 + lane];
  ((VT *)pr.V)[e] = f + b;
  ((VT *)pr.VF)[e] = f;
  ((VT *)pr.VB)[e] = b;
}

template <typename VT>
__global__ __launch_bounds__(64) void level_split_kernel(const ProblemDev *__restrict__ probs, const int s,
                                                         const int write_v, int32_t *__restrict__ arg_i,
                                                         int32_t *__restrict__ arg_d) {
  const ProblemDev &pr = probs[blockIdx.z];
  const int N = pr.N, D = pr.D, DP = pr.DP, nch = pr.nch;
  if (s > pr.S_eff) return;
  const int c = blockIdx.x, d = blockIdx.y + 1;
  if (c >= nch || d > D || d < s) return;
  const int lane = threadIdx.x;
  const int jj = 64 * c + lane;
  const int j = jj + 1;
  constexpr VT INF = Lim<VT>::inf;
  const int64_t lvl = (int64_t)(N + 1) * DP;
  const VT RANNC_GLOBAL *Vprev = gptr((const VT *)pr.V) + (int64_t)(s - 2) * lvl;
  const VT RANNC_GLOBAL *Fprev = gptr((const VT *)pr.VF) + (int64_t)(s - 2) * lvl;
  const VT RANNC_GLOBAL *Bprev = gptr((const VT *)pr.VB) + (int64_t)(s - 2) * lvl;
  const VT RANNC_GLOBAL *costf = gptr((const VT *)pr.cost);
  const VT RANNC_GLOBAL *costb = gptr((const VT *)pr.costb);
  const uint8_t RANNC_GLOBAL *rmin = gptr((const uint8_t *)pr.rmin);
  const uint8_t RANNC_GLOBAL *ufit = gptr((const uint8_t *)pr.ufit);
  VT best = INF, bf = INF, bb = INF;
  int bi = -1, bd = -1;
  const int i_end = min(64 * c + 63, N - 1);
  for (int i = s - 1; i <= i_end; ++i) {
    // a plan of s-1 stages over blocks 1..i exists on d-1 devices iff it exists on any fewer
    if (Vprev[(int64_t)i * DP + d - 2] == INF) continue;
    const int64_t u = unit_index(nch, i, c);
    if (!ufit[u]) continue;  // no stage of this unit fits: its table rows were never written
    const bool act = (jj >= i) && (jj < N);
    const VT RANNC_GLOBAL *uf = costf + u * 64 * D + lane;
    const VT RANNC_GLOBAL *ub = costb + u * 64 * D + lane;
    const int rmn = act ? (int)rmin[u * 64 + lane] : 255;
    for (int dp = s - 1; dp <= d - 1; ++dp) {
      const VT a = Vprev[(int64_t)i * DP + dp - 1];
      if (a == INF) continue;      // earlier stages infeasible
      if (d - dp < rmn) continue;  // does not fit device memory
      const VT f = vmax(Fprev[(int64_t)i * DP + dp - 1], uf[(d - dp - 1) * 64]);
      const VT b = vmax(Bprev[(int64_t)i * DP + dp - 1], ub[(d - dp - 1) * 64]);
      const VT v = f + b;
      if (v < best) { best = v; bf = f; bb = b; bi = i; bd = dp; }
    }
  }
  if (jj >= N || j < s) return;
  if (write_v) {
    const int64_t e = (int64_t)(s - 1) * lvl + (int64_t)j * DP + d - 1;
    ((VT *)pr.V)[e] = best;
    ((VT *)pr.VF)[e] = bf;
    ((VT *)pr.VB)[e] = bb;
  }
  const int64_t e = ((int64_t)s * (N + 1) + j) * (D + 1) + d;
  if (arg_i) arg_i[e] = bi;
  if (arg_d) arg_d[e] = bd;
}

// Fast form of the same level for 32-bit tables.  The kept candidate of a cell is the smallest
// (sum, i, d') in lexicographic order, so partial results over disjoint sets of rows combine
// with a 64-bit atomicMin on the packed triple.  Work item (one workgroup of eight waves) = 16
// consecutive rows of one chunk's window, from the same work list as the merge kernel.  Per row the
// two stage-time units are staged in LDS once ([r][lane], conflict-free), the eight waves share
// them and split the device totals d between them (d = s + wave, s + wave + 8, ...): a lane keeps
// the running best of its column for each of its wave's d in registers.  The row of the previous
// level (values, carried maxima) is wave-uniform: scalar loads, one per d', shared by all d.
// split_finalize_kernel then turns the packed winners of the level into V and the two carried
// maxima, and clears the key table for the next level.

// Candidates d' = lo..hi of one staged row against the device totals d_k, k >= K0, of this wave
// (all of them lie above hi, so every (d', k) pair is a candidate).  lim[k] = d_k - rmin of the
// lane's stage (below 0 if d_k > D or nothing fits): the stage fits iff d' <= lim[k].
// Packed winner of a cell: (sum, i, d') in one 64-bit word whose unsigned order is the lexicographic
// order of the triple.  32-bit tables: 32 + 24 + 8 bits.  64-bit tables: 42 + 16 + 6 bits, which is
// why the packed kernel serves 64-bit handles only up to a time bound of 2^42 - 2 ns (73 minutes);
// the 32-bit key of the running best is always (i << 8) | d'.
template <typename VT> __device__ __forceinline__ unsigned long long split_pack(VT v, uint32_t key);
template <> __device__ __forceinline__ unsigned long long split_pack<uint32_t>(uint32_t v, uint32_t key) {
  return ((unsigned long long)v << 32) | key;
}
template <> __device__ __forceinline__ unsigned long long split_pack<uint64_t>(uint64_t v, uint32_t key) {
  return (v << 22) | ((unsigned long long)(key >> 8) << 6) | (key & 63u);
}
template <typename VT> __device__ __forceinline__ int split_key_i(unsigned long long k) {
  return sizeof(VT) == 4 ? (int)((k >> 8) & 0xFFFFFFull) : (int)((k >> 6) & 0xFFFFull);
}
template <typename VT> __device__ __forceinline__ int split_key_d(unsigned long long k) {
  return sizeof(VT) == 4 ? (int)(k & 0xFFull) : (int)(k & 63ull);
}
template <typename VT> __device__ __forceinline__ VT split_key_v(unsigned long long k) {
  return sizeof(VT) == 4 ? (VT)(k >> 32) : (VT)(k >> 22);
}

template <typename VT, int DP, int K0>
__device__ __forceinline__ void split_segment(int lo, int hi, int d0, int i, int lane,
                                              const VT RANNC_GLOBAL *__restrict__ Frow,
                                              const VT RANNC_GLOBAL *__restrict__ Brow,
                                              const VT *sf, const VT *sb,
                                              const int (&lim)[DP / kSplitWaves],
                                              VT (&best_v)[DP / kSplitWaves],
                                              uint32_t (&best_key)[DP / kSplitWaves]) {
  constexpr int KP = DP / kSplitWaves;
  for (int dp = lo; dp <= hi; ++dp) {
    const VT af = Frow[dp - 1], ab = Brow[dp - 1];  // wave-uniform
    const uint32_t key = ((uint32_t)i << 8) | (uint32_t)dp;
#pragma unroll
    for (int k = K0; k < KP; ++k) {
      const int r = d0 + kSplitWaves * k - dp;  // >= 1; at most DP (rows beyond the staged ones hold
                                                // stale values, masked by lim)
      const VT f = vmax(af, sf[(r - 1) * 64 + lane]);
      const VT b = vmax(ab, sb[(r - 1) * 64 + lane]);
      const VT v = f + b;
      const bool ok = (dp <= lim[k]) & (v < best_v[k]);
      best_v[k] = ok ? v : best_v[k];
      best_key[k] = ok ? key : best_key[k];
    }
  }
}

template <typename VT, int DP, int K0>
__device__ __forceinline__ void split_row(int dlo, int D, int d0, int i, int lane,
                                          const VT RANNC_GLOBAL *__restrict__ Frow,
                                          const VT RANNC_GLOBAL *__restrict__ Brow,
                                          const VT *sf, const VT *sb,
                                          const int (&lim)[DP / kSplitWaves],
                                          VT (&best_v)[DP / kSplitWaves],
                                          uint32_t (&best_key)[DP / kSplitWaves]) {
  if constexpr (K0 < DP / kSplitWaves) {
    // d' in [d_{K0-1}, d_{K0} - 1]: exactly the totals d_k with k >= K0 lie above it
    const int lo = K0 == 0 ? dlo : max(dlo, d0 + kSplitWaves * (K0 - 1));
    const int hi = min(d0 + kSplitWaves * K0 - 1, D - 1);
    split_segment<VT, DP, K0>(lo, hi, d0, i, lane, Frow, Brow, sf, sb, lim, best_v, best_key);
    split_row<VT, DP, K0 + 1>(dlo, D, d0, i, lane, Frow, Brow, sf, sb, lim, best_v, best_key);
  }
}

template <typename VT, int DP>
__global__ __launch_bounds__(64 * kSplitWaves) void level_split_fast_kernel(
    const ProblemDev *__restrict__ probs, const int s) {
  constexpr VT INF = Lim<VT>::inf;
  constexpr int KP = DP / kSplitWaves;  // device totals per wave
  const ProblemDev &pr = probs[blockIdx.z];
  if (s > pr.S_eff) return;
  const int N = pr.N, D = pr.D, nch = pr.nch;
  const int32_t RANNC_GLOBAL *__restrict__ runs = gptr((const int32_t *)pr.runs);
  if ((int)blockIdx.x >= runs[0]) return;
  const unsigned desc = (unsigned)runs[1 + blockIdx.x];
  const int c = (int)((desc >> 16) & 0x3ffu), i0 = (int)(desc & 0xffffu), rows = (int)(desc >> 26) + 1;
  if (64 * c + 64 < s) return;  // no column j >= s in this chunk
  const int i_hi = min(min(i0 + rows - 1, 64 * c + 63), N - 1);
  const int i_lo = max(i0, s - 1);
  if (i_hi < i_lo) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int jj = 64 * c + lane;
  const int64_t lvl = (int64_t)(N + 1) * DP;
  const VT RANNC_GLOBAL *__restrict__ Vprev = gptr((const VT *)pr.V) + (int64_t)(s - 2) * lvl;
  const VT RANNC_GLOBAL *__restrict__ Fprev = gptr((const VT *)pr.VF) + (int64_t)(s - 2) * lvl;
  const VT RANNC_GLOBAL *__restrict__ Bprev = gptr((const VT *)pr.VB) + (int64_t)(s - 2) * lvl;
  const VT RANNC_GLOBAL *__restrict__ costf = gptr((const VT *)pr.cost);
  const VT RANNC_GLOBAL *__restrict__ costb = gptr((const VT *)pr.costb);
  const uint8_t RANNC_GLOBAL *__restrict__ rmin = gptr((const uint8_t *)pr.rmin);
  const uint8_t RANNC_GLOBAL *__restrict__ ufit = gptr((const uint8_t *)pr.ufit);
  const int rl = D - s + 1;  // replicas left for stage s when s-1 devices are spent earlier
  const int d0 = s + wave;   // this wave's device totals: d0, d0 + 8, ...
  __shared__ VT sf[DP * 64], sb[DP * 64];

  VT best_v[KP];
  uint32_t best_key[KP];
#pragma unroll
  for (int k = 0; k < KP; ++k) { best_v[k] = INF; best_key[k] = 0xFFFFFFFFu; }

  for (int i = i_lo; i <= i_hi; ++i) {  // every condition below is uniform over the workgroup
    if (Vprev[(int64_t)i * DP + D - 2] == INF) continue;  // no (s-1)-stage plan over blocks 1..i
    const int64_t u = unit_index(nch, i, c);
    if (!ufit[u]) continue;  // no stage of this unit fits: its rows were never written
    __syncthreads();  // the previous row's reads of the staged units are done
    for (int e = tid; e < rl * 64; e += 64 * kSplitWaves) {
      sf[e] = costf[u * 64 * D + e];
      sb[e] = costb[u * 64 * D + e];
    }
    const int rmn = (jj >= i && jj < N) ? (int)rmin[u * 64 + lane] : 255;
    // first d' with a plan (finite values are a suffix of the row)
    const VT av = (lane < D) ? Vprev[(int64_t)i * DP + lane] : INF;
    const unsigned long long fin = __ballot(av != INF);
    const int dlo = max(s - 1, __ffsll((long long)fin));  // lane q holds d' = q + 1
    int lim[KP];
#pragma unroll
    for (int k = 0; k < KP; ++k) lim[k] = (d0 + kSplitWaves * k <= D) ? d0 + kSplitWaves * k - rmn : -1;
    __syncthreads();
    split_row<VT, DP, 0>(dlo, D, d0, i, lane, Fprev + (int64_t)i * DP, Bprev + (int64_t)i * DP, sf, sb, lim,
                     best_v, best_key);
  }
  if (jj >= N || jj + 1 < s) return;
  unsigned long long RANNC_GLOBAL *K = gptr((unsigned long long *)pr.keys);
#pragma unroll
  for (int k = 0; k < KP; ++k) {
    const int dk = d0 + kSplitWaves * k;
    if (dk <= D && best_v[k] != INF)
      (void)__hip_atomic_fetch_min(&K[(int64_t)(dk - 1) * (N + 1) + jj + 1], split_pack<VT>(best_v[k], best_key[k]),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <typename VT>
__global__ __launch_bounds__(256) void split_finalize_kernel(const ProblemDev *__restrict__ probs, const int s) {
  const ProblemDev &pr = probs[blockIdx.z];
  if (s > pr.S_eff) return;
  const int N = pr.N, D = pr.D, DP = pr.DP, nch = pr.nch;
  const int j = blockIdx.x * 256 + threadIdx.x, d = blockIdx.y + 1;
  if (j > N || d > D) return;
  unsigned long long *K = (unsigned long long *)pr.keys + (int64_t)(d - 1) * (N + 1) + j;
  const unsigned long long key = *K;
  if (key == ~0ull) return;  // no candidate: the cell keeps "no plan"
  *K = ~0ull;                // ready for the next level
  const int i = split_key_i<VT>(key), dp = split_key_d<VT>(key);
  const int jj = j - 1;
  const int64_t lvl = (int64_t)(N + 1) * DP;
  const int64_t pc = (int64_t)(s - 2) * lvl + (int64_t)i * DP + dp - 1;
  const int64_t te = (unit_index(nch, i, jj >> 6) * D + (d - dp - 1)) * 64 + (jj & 63);
  const int64_t e = (int64_t)(s - 1) * lvl + (int64_t)j * DP + d - 1;
  ((VT *)pr.V)[e] = split_key_v<VT>(key);
  ((VT *)pr.VF)[e] = vmax(((const VT *)pr.VF)[pc], ((const VT *)pr.cost)[te]);
  ((VT *)pr.VB)[e] = vmax(((const VT *)pr.VB)[pc], ((const VT *)pr.costb)[te]);
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
hipError_t launch_split_level1(const ProblemDev *p, const LaunchShape &sh, int bits, hipStream_t st) {
  for (int q0 = 0; q0 < sh.nprob; q0 += 65535) {
    const int nq = min(65535, sh.nprob - q0);
    const dim3 grid(sh.max_nch, sh.max_D, nq);
    if (bits == 32) hipLaunchKernelGGL((split_level1_kernel<uint32_t>), grid, dim3(64), 0, st, p + q0);
    else hipLaunchKernelGGL((split_level1_kernel<uint64_t>), grid, dim3(64), 0, st, p + q0);
  }
  return hipGetLastError();
}

hipError_t launch_level_split(const ProblemDev *p, const LaunchShape &sh, int bits, int s, int write_v,
                              int32_t *arg_i, int32_t *arg_d, hipStream_t st) {
  for (int q0 = 0; q0 < sh.nprob; q0 += 65535) {
    const int nq = min(65535, sh.nprob - q0);
    const dim3 grid(sh.max_nch, sh.max_D, nq);
    if (bits == 32)
      hipLaunchKernelGGL((level_split_kernel<uint32_t>), grid, dim3(64), 0, st, p + q0, s, write_v, arg_i,
                         arg_d);
    else
      hipLaunchKernelGGL((level_split_kernel<uint64_t>), grid, dim3(64), 0, st, p + q0, s, write_v, arg_i,
                         arg_d);
  }
  return hipGetLastError();
}

int split_rows_per_item(const LaunchShape &sh, int n_cus) {
  // two workgroups of eight waves per compute unit; the work list has room for kSplitSmallRows such items
  const int64_t rows = merge_launch_rows(sh), slots = std::min<int64_t>(2ll * n_cus, kSplitSmallRows / 2);
  return rows <= slots ? 1 : rows <= 2 * slots ? 2 : 0;
}

template <typename VT>
static void split_fast_go(const ProblemDev *p, const LaunchShape &sh, int DP, int s, int64_t items, hipStream_t st) {
  for (int q0 = 0; q0 < sh.nprob; q0 += 65535) {
    const int nq = min(65535, sh.nprob - q0);
    const dim3 grid((unsigned)items, 1, nq), block(64 * kSplitWaves);
    if (DP == 8) hipLaunchKernelGGL((level_split_fast_kernel<VT, 8>), grid, block, 0, st, p + q0, s);
    else if (DP == 16) hipLaunchKernelGGL((level_split_fast_kernel<VT, 16>), grid, block, 0, st, p + q0, s);
    else if (DP == 32) hipLaunchKernelGGL((level_split_fast_kernel<VT, 32>), grid, block, 0, st, p + q0, s);
    else hipLaunchKernelGGL((level_split_fast_kernel<VT, 64>), grid, block, 0, st, p + q0, s);
    hipLaunchKernelGGL((split_finalize_kernel<VT>), dim3((sh.max_N + 256) / 256, sh.max_D, nq), dim3(256), 0, st,
                       p + q0, s);
  }
}

hipError_t launch_level_split_fast(const ProblemDev *p, const LaunchShape &sh, int bits, int DP, int s,
                                   int rows_per_item, hipStream_t st) {
  const int per = rows_per_item > 0 ? rows_per_item : kSplitMinRows;
  int64_t items = 0;  // upper bound on the items of any problem of the launch
  for (int c = 0; c < sh.max_nch; ++c) items += (min(64 * c + 64, sh.max_N) + per - 1) / per;
  if (bits == 32) split_fast_go<uint32_t>(p, sh, DP, s, items, st);
  else split_fast_go<uint64_t>(p, sh, DP, s, items, st);
  return hipGetLastError();
}

}  // namespace rannc
