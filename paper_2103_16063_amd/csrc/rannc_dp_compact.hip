// gfx950 kernel of the compaction step of RaNNC's block-level phase (Sec. III-B) on a chain, and
// its launcher.
#include "rannc_dp_device.h"

namespace rannc {

// ---------------------------------------------------------------------------------------
// Compaction step of the block-level phase (Sec. III-B, last step before the stage-level search),
// on a chain of G groups.  A walk: the groups as they stand are listed by ascending computation
// time (equal times by position); a listed group that is still as listed merges with the
// neighbour whose current time is smaller if the union fits the device memory; the procedure ends
// as soon as k groups are left.  When a walk ends above k groups the groups are listed again by
// their current times and walked again, until k is reached, a walk merges nothing, or the caller's
// limit on the number of walks is met.  Every merge changes what the following groups see, so a
// walk itself is sequential (one lane follows the list; the state lives in LDS for chains of up to
// kCompactLds groups, in the workspace beyond that); the listing (a rank sort for up to 2048
// groups, a bitonic sort of the group indices beyond), the validation and the packing of the
// result into the block arrays of the search are parallel.  The kernel exists so that the chain
// stays on the device between the two phases.  One workgroup.
// ---------------------------------------------------------------------------------------
constexpr int kCompactThreads = 1024;
constexpr int kCompactRankSort = 2048;  // up to this many groups the listing is a rank sort

// (time, position) order of two listed groups; index -1 (padding) ranks behind everything
__device__ __forceinline__ bool compact_after(const int64_t *ct, int x, int y) {
  if (x < 0 || y < 0) return x < 0 && y >= 0;
  const int64_t tx = ct[x], ty = ct[y];
  return tx > ty || (tx == ty && x > y);
}

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(
    int G, int k, int64_t M, int max_walks, const int64_t *__restrict__ t, const int64_t *__restrict__ p,
    const int64_t *__restrict__ a, char *__restrict__ ws, int32_t *n_out, int32_t *block_end,
    int64_t *t_out, int64_t *p_out, int64_t *a_out, int32_t *status) {
  __shared__ int64_t l_ct[kCompactLds], l_cp[kCompactLds], l_ca[kCompactLds];
  __shared__ int32_t l_prev[kCompactLds], l_next[kCompactLds];
  __shared__ uint8_t l_listed[kCompactLds], l_alive[kCompactLds];
  __shared__ unsigned long long sum_t, sum_m;
  __shared__ int flags, scan[kCompactThreads], s_count, s_merged;
  const int tid = threadIdx.x;
  // state arrays: LDS for short chains, the workspace otherwise (same code through generic pointers)
  int64_t *ct = l_ct, *cp = l_cp, *ca = l_ca;
  int32_t *prev = l_prev, *next = l_next, *order = (int32_t *)ws;
  int32_t *heads = (int32_t *)(ws + compact_order_bytes(G));
  uint8_t *listed = l_listed, *alive = l_alive;
  if (G > kCompactLds) {
    char *w = ws + 2 * compact_order_bytes(G);
    const size_t a8 = (((size_t)G * 8 + 255) / 256) * 256, a4 = (((size_t)G * 4 + 255) / 256) * 256;
    ct = (int64_t *)w; w += a8;
    cp = (int64_t *)w; w += a8;
    ca = (int64_t *)w; w += a8;
    prev = (int32_t *)w; w += a4;
    next = (int32_t *)w; w += a4;
    listed = (uint8_t *)w; w += a4;
    alive = (uint8_t *)w;
  }
  if (tid == 0) { sum_t = 0ull; sum_m = 0ull; flags = 0; s_count = G; }
  __syncthreads();
  // ---- validation and initial state ----
  {
    unsigned long long st = 0ull, sm = 0ull;
    int myflags = 0;
    for (int g = tid; g < G; g += kCompactThreads) {
      int64_t tv = t[g], pv = p[g], av = a[g];
      if (tv < 0 || pv < 0 || av < 0) { myflags |= 1; tv = pv = av = 0; }
      if ((uint64_t)tv >= kSumLimit || (uint64_t)pv >= kSumLimit || (uint64_t)av >= kSumLimit) {
        myflags |= 2; tv = pv = av = 0;
      }
      st += (uint64_t)tv; if (st > kSumLimit) st = kSumLimit;
      sm += (uint64_t)pv; if (sm > kSumLimit) sm = kSumLimit;
      sm += (uint64_t)av; if (sm > kSumLimit) sm = kSumLimit;
      ct[g] = tv; cp[g] = pv; ca[g] = av;
      prev[g] = g - 1;
      next[g] = g + 1 < G ? g + 1 : -1;
      alive[g] = 1;
    }
    // totals, saturating (a few hundred adds on two LDS words)
    unsigned long long old = atomicAdd(&sum_t, st);
    if (old + st >= kSumLimit) myflags |= 2;
    old = atomicAdd(&sum_m, sm);
    if (old + sm >= kSumLimit) myflags |= 2;
    if (myflags) atomicOr(&flags, myflags);
  }
  __syncthreads();
  if (flags) {
    if (tid == 0) {
      *status = (flags & 1) ? RANNC_DP_PROBLEM_NEGATIVE_INPUT : RANNC_DP_PROBLEM_SUM_OVERFLOW;
      *n_out = 0;
    }
    return;
  }
  const int per = (G + kCompactThreads - 1) / kCompactThreads;
  const int lo = min(tid * per, G), hi = min(lo + per, G);
  for (int walk = 1; max_walks <= 0 || walk <= max_walks; ++walk) {
    const int n = s_count;  // groups as they stand; every thread reads it before thread 0 walks again
    if (n <= k) break;
    // ---- the group heads in chain order: heads[0..n) ----
    int mine = 0;
    for (int g = lo; g < hi; ++g) mine += alive[g];
    scan[tid] = mine;
    __syncthreads();
    for (int off = 1; off < kCompactThreads; off <<= 1) {
      const int add = tid >= off ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += add;
      __syncthreads();
    }
    {
      int u = scan[tid] - mine;
      for (int g = lo; g < hi; ++g) {
        listed[g] = alive[g];
        if (alive[g]) heads[u++] = g;
      }
    }
    __syncthreads();
    // ---- listing: the heads in the order (current time, position) ----
    if (n <= kCompactRankSort) {
      for (int x = tid; x < n; x += kCompactThreads) {
        const int g = heads[x];
        const int64_t tg = ct[g];
        int rank = 0;
        for (int y = 0; y < n; ++y) {
          const int64_t th = ct[heads[y]];
          rank += (th < tg) || (th == tg && y < x);  // heads ascend with their position in the list
        }
        order[rank] = g;
      }
      __syncthreads();
    } else {
      int P = 1;
      while (P < n) P <<= 1;
      for (int x = tid; x < P; x += kCompactThreads) order[x] = x < n ? heads[x] : -1;
      __syncthreads();
      for (int size = 2; size <= P; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
          for (int e = tid; e < (P >> 1); e += kCompactThreads) {
            const int x = 2 * e - (e & (stride - 1)), y = x + stride;
            const bool ascending = (x & size) == 0;
            const int gx = order[x], gy = order[y];
            if (compact_after(ct, gx, gy) == ascending) { order[x] = gy; order[y] = gx; }
          }
          __syncthreads();
        }
      }
    }
    // ---- the walk ----
    if (tid == 0) {
      int count = n, merged = 0;
      for (int x = 0; x < n && count > k; ++x) {
        const int v = order[x];
        if (!listed[v]) continue;
        const int l = prev[v], r = next[v];
        if (l < 0 && r < 0) break;
        int w;
        if (l < 0) w = r;
        else if (r < 0) w = l;
        else w = ct[r] < ct[l] ? r : l;
        if (cp[v] + ca[v] + cp[w] + ca[w] > M) continue;  // totals stay below 2^62: no overflow
        const int first = (w == l) ? l : v, second = (w == l) ? v : r;
        ct[first] += ct[second]; cp[first] += cp[second]; ca[first] += ca[second];
        const int nx = next[second];
        next[first] = nx;
        if (nx >= 0) prev[nx] = first;
        listed[first] = 0; listed[second] = 0;
        alive[second] = 0;
        --count;
        ++merged;
      }
      s_count = count;
      s_merged = merged;
    }
    __syncthreads();
    const int merged = s_merged;
    __syncthreads();  // everyone has read the walk's outcome before the next walk overwrites it
    if (merged == 0) break;
  }
  // ---- result: the surviving group heads in chain order ----
  __syncthreads();
  int mine = 0;
  for (int g = lo; g < hi; ++g) mine += alive[g];
  scan[tid] = mine;
  __syncthreads();
  for (int off = 1; off < kCompactThreads; off <<= 1) {
    const int add = tid >= off ? scan[tid - off] : 0;
    __syncthreads();
    scan[tid] += add;
    __syncthreads();
  }
  int u = scan[tid] - mine;
  for (int g = lo; g < hi; ++g) {
    if (!alive[g]) continue;
    block_end[u] = next[g] >= 0 ? next[g] : G;
    t_out[u] = ct[g]; p_out[u] = cp[g]; a_out[u] = ca[g];
    ++u;
  }
  if (tid == kCompactThreads - 1) { *n_out = scan[tid]; *status = RANNC_DP_PROBLEM_OK; }
}

hipError_t launch_compact(int G, int k, int64_t M, int max_walks, const int64_t *t, const int64_t *p,
                          const int64_t *a, void *ws, int32_t *n_out, int32_t *block_end, int64_t *t_out,
                          int64_t *p_out, int64_t *a_out, int32_t *status, hipStream_t st) {
  hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(kCompactThreads), 0, st, G, k, M, max_walks, t, p, a, (char *)ws,
                     n_out, block_end, t_out, p_out, a_out, status);
  return hipGetLastError();
}

}  // namespace rannc
