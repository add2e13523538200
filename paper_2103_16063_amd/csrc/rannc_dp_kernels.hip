// gfx950 kernels of the stage-level partition search (RaNNC Sec. III-C, Algorithm 1).
//
// One wavefront is 64 lanes; in every kernel that touches the stage-time table a lane owns one
// output column j (blocks 1..j covered), so table rows are read with coalesced requests and no
// value ever has to cross lanes.  All arithmetic is exact unsigned integer arithmetic.
//
// A problem whose inputs failed validation (status word != 0) still runs through the table and
// level kernels: every access stays inside the problem's own regions, and its values are never
// reported (the final selection, the plan recovery and the exports check the status word).
#include "rannc_dp_device.h"

#include <type_traits>

namespace rannc {

// ---------------------------------------------------------------------------------------
// Prefix sums T, P, A of the block inputs (the sums over a stage's members that stand in
// for profile(), Sec. IV-D) and input validation.  One workgroup per problem.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefix_kernel(const ProblemDev *__restrict__ probs) {
  const ProblemDev pr = probs[blockIdx.x];
  __shared__ uint64_t part[4][256];
  __shared__ int flags;
  __shared__ unsigned long long max_cut;
  const int N = pr.N, tid = threadIdx.x;
  const int seg = (N + 255) / 256;
  const int lo = min(tid * seg, N), hi = min(lo + seg, N);
  if (tid == 0) { flags = 0; max_cut = 0ull; }
  __syncthreads();
  const int64_t *in[4] = {pr.t, pr.p, pr.a, pr.tb};
  int64_t *out[4] = {pr.T, pr.P, pr.A, pr.TB};
  const int nw = pr.tb ? 4 : 3;  // backward times only with the split objective
  int myflags = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (w >= nw) break;
    uint64_t s = 0;
    for (int k = lo; k < hi; ++k) {
      int64_t v = in[w][k];
      if (v < 0) { myflags |= 1; v = 0; }
      uint64_t u = (uint64_t)v;
      if (u >= kSumLimit) { myflags |= 2; u = kSumLimit; }
      s = s + u; if (s > kSumLimit) s = kSumLimit;
    }
    part[w][tid] = s;
  }
  __syncthreads();
  // inclusive scan of the 256 segment sums (saturating add is associative on [0, limit])
  for (int off = 1; off < 256; off <<= 1) {
    uint64_t add[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) add[w] = (w < nw && tid >= off) ? part[w][tid - off] : 0;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (w >= nw) break;
      uint64_t v = part[w][tid] + add[w];
      part[w][tid] = v > kSumLimit ? kSumLimit : v;
    }
    __syncthreads();
  }
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (w >= nw) break;
    uint64_t run = tid ? part[w][tid - 1] : 0;  // sum of the segments before this thread's
    if (tid == 0) out[w][0] = 0;
    for (int k = lo; k < hi; ++k) {
      int64_t v = in[w][k];
      uint64_t u = v < 0 ? 0 : (uint64_t)v;
      if (u > kSumLimit) u = kSumLimit;
      run += u; if (run > kSumLimit) run = kSumLimit;
      if (run >= kSumLimit) myflags |= 2;
      out[w][k + 1] = (int64_t)run;
    }
  }
  if (pr.o) {  // per-cut send time; the last block has no follower
    unsigned long long mc = 0ull;
    if (tid == 0) pr.C[0] = 0;
    for (int k = lo; k < hi; ++k) {
      const uint64_t c = cut_time(pr.o[k], pr.bw, myflags);
      pr.C[k + 1] = (k + 1 < N) ? (int64_t)c : 0;
      if (k + 1 < N && c > mc) mc = c;
    }
    if (mc) atomicMax(&max_cut, mc);
  }
  if (myflags) atomicOr(&flags, myflags);
  __syncthreads();
  if (tid == 0) {
    int st = RANNC_DP_PROBLEM_OK;
    if (flags & 1) st = RANNC_DP_PROBLEM_NEGATIVE_INPUT;
    else if (flags & 2) st = RANNC_DP_PROBLEM_SUM_OVERFLOW;
    else if ((uint64_t)pr.T[N] + (pr.tb ? (uint64_t)pr.TB[N] : 0ull) + max_cut > (uint64_t)pr.time_limit)
      st = RANNC_DP_PROBLEM_TIME_TOO_LARGE;  // a value is at most forward + send + backward time of all blocks
    *pr.status = st;
  }
}

// ---------------------------------------------------------------------------------------
// Initial state: every V entry "no plan" (padding columns d > D hold 0 so that padded rows stay
// sorted).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_kernel(const ProblemDev *__restrict__ probs) {
  const ProblemDev pr = probs[blockIdx.y];
  const int64_t total = (int64_t)pr.S_eff * (pr.N + 1) * pr.DP;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (pr.keys) {  // packed winners of the split level kernel: "none"
    const int64_t nk = (int64_t)(pr.N + 1) * pr.DP;
    for (int64_t e = t0; e < nk; e += stride) ((unsigned long long *)pr.keys)[e] = ~0ull;
  }
  void *tabs[3] = {pr.V, pr.VF, pr.VB};
  for (int w = 0; w < (pr.VF ? 3 : 1); ++w) {
    if (pr.bits == 32) {
      uint32_t *V = (uint32_t *)tabs[w];
      for (int64_t e = t0; e < total; e += stride)
        V[e] = ((int)(e & (pr.DP - 1)) < pr.D) ? Lim<uint32_t>::inf : 0u;
    } else {
      uint64_t *V = (uint64_t *)tabs[w];
      for (int64_t e = t0; e < total; e += stride)
        V[e] = ((int)(e & (pr.DP - 1)) < pr.D) ? Lim<uint64_t>::inf : 0ull;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Stage-time and fits-in-memory tables: h(i,j,r) and the m(i,j,r) <= M rule of Sec. III-C for
// every stage (i,j) and replica count r.  One wave per unit (row i, 64-column chunk c), four
// rows per workgroup; a lane
// owns one j and writes its D entries, each store instruction covering 64 consecutive columns
// of one contiguous unit.  Memory is non-increasing in r, so the fit rule is stored as the
// smallest fitting r and folded into the time table as INF below it (within units that hold at
// least one fitting stage; the others keep only their rmin bytes).  Row i = 0 is also level 1
// of the DP (one stage on d devices), written here.
// ---------------------------------------------------------------------------------------
constexpr int kBuildWaves = 4;

// ceil(x / r) for every r = 1..DP of a 32-bit x, without integer division: for odd r one
// double-precision add and one fused multiply-add whose low word is the quotient (the derivation
// stands at DirectConsts below), for even r an add and a shift from ceil(x / (r/2)).
template <int DP>
__device__ __forceinline__ void ceil_div_all(uint32_t x, uint32_t (&q)[DP + 1]) {
  const double xf = (double)x;
  double magic = 0x1.8p52;
  asm("" : "+v"(magic));  // one register for all entries instead of a literal per instruction
#pragma unroll
  for (int r = 1; r <= DP; ++r) {
    if (r & 1) {
      const double add = (double)r / 2.0 - 1.0 + (double)r * 0x1p-18;
      const double y = __builtin_fma(xf + add, 1.0 / (double)r, magic);
      q[r] = (uint32_t)__double_as_longlong(y);
    } else {
      q[r] = (q[r / 2] + 1u) >> 1;
    }
  }
}

// The D entries of one stage (i,j): ceil(tij / r) (+ ceil(cj / r) with the communication term), INF
// below rmin.  NODIV: 32-bit values take the division-free form above (the table builder was bound
// by the quarter-rate integer multiplies of 64 divisions by constants per stage, not by its stores;
// the one-launch kernel, which has 128 registers per lane, keeps the integer form).  Otherwise r is
// a compile-time constant after unrolling, so the divisions are multiplications.
template <typename VT, int DP, bool COMM, bool NODIV>
__device__ __forceinline__ void build_rows(VT tij, VT cj, int rmin, int D, VT RANNC_GLOBAL *crow, VT *lds1) {
  constexpr bool FAST = NODIV && sizeof(VT) == 4;
  [[maybe_unused]] uint32_t qt[DP + 1], qc[DP + 1];
  if constexpr (FAST) {
    ceil_div_all<DP>((uint32_t)tij, qt);
    if (COMM) ceil_div_all<DP>((uint32_t)cj, qc);
  }
  auto entry = [&](const int r) -> VT {  // r is a compile-time number wherever this is called
    VT h;
    if constexpr (FAST) {
      h = qt[r];
      if (COMM) h += qc[r];
    } else {
      const VT q = tij / (VT)r;
      h = q + (VT)(q * (VT)r != tij);  // ceil
      if (COMM) {
        const VT qq = cj / (VT)r;
        h += qq + (VT)(qq * (VT)r != cj);
      }
    }
    return (r >= rmin) ? h : Lim<VT>::inf;
  };
  // one straight run of stores per destination; r <= D is a scalar test (every r keeps its own
  // code: the quotient arrays stay in registers only with compile-time indices)
  if (crow) {
#pragma unroll
    for (int r = 1; r <= DP; ++r)
      if (r <= D) crow[(r - 1) * 64] = entry(r);
  }
  if (lds1) {
#pragma unroll
    for (int r = 1; r <= DP; ++r)
      if (r <= D) lds1[r - 1] = entry(r);
  }
}

// One unit (row i, chunk c) of the tables, by one wave.  T, P, A, Cc may live in global memory or in
// LDS; Cc (per-cut send time at one replica, Cc[N] = 0) is null when there is no communication
// term.  Returns whether any stage of the unit fits.  Row 0's entries are level 1 of V: with
// lds_level1 given they go to LDS, row (j - row0) with row stride ls, and the caller copies them to
// the value table (a lane's D values are a row of V, so writing them from here would scatter every
// store instruction over 64 cache lines).  with_times = false: only the fits-in-memory part (rmin,
// ufit) and level 1 are produced, for searches whose level kernel recomputes the stage times.
// lds_rmin: the unit's 64 rmin bytes also go there (255 for a lane without a stage).
template <typename VT, int DP, bool NODIV = false>
__device__ __forceinline__ bool build_unit(const ProblemDev &pr, const int64_t *T, const int64_t *P,
                                           const int64_t *A, const int64_t *Cc, int i, int c, int lane,
                                           VT *lds_level1, int ls, int row0, const int64_t *TBp = nullptr,
                                           const bool with_times = true, uint8_t *lds_rmin = nullptr) {
  const int N = pr.N, D = pr.D, nch = pr.nch;
  const int jj = 64 * c + lane;
  const bool valid = (jj >= i) && (jj < N);
  const int j = valid ? jj + 1 : i + 1;  // padding lanes compute a harmless in-range stage
  const int64_t Tij = T[j] - T[i];
  const int64_t Pij = P[j] - P[i];
  const int64_t Aij = A[j] - A[i];
  // smallest r with Pij + ceil(Aij / r) <= M, using ceil(a/r) <= k  <=>  a <= k*r
  int rmin = 255;
  if (Pij <= pr.M) {
    const int64_t slack = pr.M - Pij;
    if (Aij <= slack) rmin = 1;
    else if (slack > 0) {
      const uint64_t need = ((uint64_t)Aij + (uint64_t)slack - 1) / (uint64_t)slack;
      if (need <= (uint64_t)D) rmin = (int)need;
    }
  }
  const bool fits = valid && rmin <= D;
  const bool unit_fits = __ballot(fits) != 0ull;
  const int64_t u = unit_index(nch, i, c);
  if (lane == 0) pr.ufit[u] = (uint8_t)unit_fits;
  if (lds_rmin) lds_rmin[lane] = (uint8_t)(valid ? rmin : 255);  // the caller's copy: every lane, 255 = no stage
  if (!valid) return unit_fits;
  pr.rmin[u * 64 + lane] = (uint8_t)rmin;
  // A unit in which no stage fits for any r is never read (every reader consults ufit or rmin
  // first): only those are written.  Row 0 also carries level 1 and is always written.
  if (!unit_fits && i != 0) return unit_fits;
  if (!with_times && !(i == 0 && lds_level1)) return unit_fits;
  VT RANNC_GLOBAL *crow = with_times ? gptr((VT *)pr.cost) + u * 64 * D + lane : nullptr;
  VT *lds1 = (i == 0 && lds_level1) ? lds_level1 + (j - row0) * ls : nullptr;
  const VT tij = (VT)Tij;
  if (Cc)  // wave-uniform: with the stage's own send time at one replica (0 for j = N)
    build_rows<VT, DP, true, NODIV>(tij, (VT)Cc[j], rmin, D, crow, lds1);
  else
    build_rows<VT, DP, false, NODIV>(tij, (VT)0, rmin, D, crow, lds1);
  if (TBp && with_times)  // split objective: the backward times get a table of their own (never a send time)
    build_rows<VT, DP, false, NODIV>((VT)(TBp[j] - TBp[i]), (VT)0, rmin, D,
                              gptr((VT *)pr.costb) + u * 64 * D + lane, nullptr);
  return unit_fits;
}

// parts: 1 = fits-in-memory tables and level 1 of V only, 3 = those and the stage-time table,
// 2 = the stage-time table alone (added later to a search that was solved without it)
// A wave takes `rows` consecutive rows of one chunk, one after the other: one row when the
// stage-time table is written (64 row stores per unit keep it busy), several when only the
// fits-in-memory part is (a unit is then 65 bytes of output, and a launch of one wave per unit is
// bound by the rate at which waves can be started).
// (The several-rows variant is held to the registers of four waves per SIMD: its time goes into the
// latency of many short units, and the 64 quotients of row 0, the only row that needs them there,
// would otherwise halve the waves in flight at 64 devices.)
template <typename VT, int DP, int ROWS>
__global__ __launch_bounds__(64 * kBuildWaves) __attribute__((amdgpu_waves_per_eu(ROWS > 1 ? 4 : 1)))
void build_kernel(const ProblemDev *__restrict__ probs, const int parts, const int pr_many) {
  // Workgroups go to the eight XCDs round-robin in the order of their linear index.  A launch over
  // several searches has grid = (searches, row groups, chunks): the search runs fastest and every
  // XCD gets rows of every chunk (with the chunk fastest and two chunks per search, the XCDs with
  // even numbers would get the triangle of chunk 0 and the others the three times larger chunk 1:
  // config 5, fits-in-memory part, 59 -> 39 us).  One search: grid = (chunks, row groups, 1).
  const bool many = pr_many != 0;
  const ProblemDev &pr = probs[many ? blockIdx.x : 0];
  const int lane = threadIdx.x & 63;
  const int i0 = (blockIdx.y * kBuildWaves + (int)(threadIdx.x >> 6)) * ROWS, c = many ? blockIdx.z : blockIdx.x;
  __shared__ VT tile[64 * (DP + 1)];  // level 1 of this chunk (only the wave that holds row 0 uses it)
  if (c >= pr.nch) return;
  auto one_row = [&](const int i) {
    const bool level1 = i == 0 && (parts & 1);
    (void)build_unit<VT, DP, true>(pr, pr.T, pr.P, pr.A, pr.C, i, c, lane, level1 ? tile : nullptr, DP + 1, 64 * c + 1,
                                   pr.TB, (parts & 2) != 0);
    if (level1) {
      // rows j = 64c+1 .. of level 1 are contiguous in V: written with consecutive lanes on
      // consecutive words (columns d > D keep the zeros of the fill)
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      const int D = pr.D, nrow = min(64, pr.N - 64 * c);
      VT RANNC_GLOBAL *v1 = gptr((VT *)pr.V) + (int64_t)(64 * c + 1) * DP;
      for (int e = lane; e < nrow * DP; e += 64) {
        const int row = e / DP, col = e % DP;
        if (col < D) v1[e] = tile[row * (DP + 1) + col];
      }
    }
  };
  if constexpr (ROWS == 1) {
    // straight-line: the wave ends behind its last store without waiting for it
    if (i0 < pr.N && c >= (i0 >> 6)) one_row(i0);
  } else {
#pragma unroll 1
    for (int i = i0; i < min(i0 + ROWS, pr.N); ++i) {
      if (c < (i >> 6)) break;  // the rows from here on have no column in this chunk
      one_row(i);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Window of the level kernels: wlo[c] = first row i that holds a stage into chunk c that fits for
// some r <= D (0x7fffffff if none).  Rows below it are never visited.  One workgroup per
// (chunk, problem); no global atomics (same-address atomics serialise badly).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void windows_kernel(const ProblemDev *__restrict__ probs) {
  const ProblemDev &pr = probs[blockIdx.y];
  const int c = blockIdx.x, nch = pr.nch;
  if (c >= nch) return;
  __shared__ int first;
  if (threadIdx.x == 0) first = kNoRow;
  __syncthreads();
  const int hi = min(64 * c + 63, pr.N - 1);
  int mine = kNoRow;
  for (int i = threadIdx.x; i <= hi; i += 256)
    if (pr.ufit[unit_index(nch, i, c)]) { mine = i; break; }  // rows ascend
  if (mine != kNoRow) atomicMin(&first, mine);
  __syncthreads();
  if (threadIdx.x == 0) pr.wlo[c] = first;
}

// ---------------------------------------------------------------------------------------
// Work list of the level kernels: the rows wlo[c] .. min(64c+63, N-1) of every chunk, cut into
// items of consecutive rows, listed chunk by chunk.  A compact list keeps the workgroups that have
// work at the front of the grid.  The number of rows of an item travels in the top bits of its
// descriptor: (rows - 1) << 26 | c << 16 | first row.  rows > 0: items of that many rows.
// rows = 0 (split-objective level kernel): 16, 8 or 4 rows, from the size of all windows together.
// rows = -1 (sorted-merge level kernel): the smallest multiple of 4 (up to 64) whose item count
// fits max_items, the grid the host launches (sized for the rows of an unpruned search: small
// items, i.e. many workgroups and a short critical path, when pruning leaves few rows; large ones,
// i.e. fewer folds and atomics per row, when the launch is full anyway; and never a workgroup
// without an item in a launch over many searches).  If that launch needs more than one round of
// workgroups (`slots` run at a time, `batch` searches in the launch), the smallest item size that
// brings it down to one round is taken instead, provided the round still fills half the device:
// the round is then as full as it can be, and no compute unit is left with one workgroup more
// than its neighbours.  (For a launch of many rounds, hundreds of searches, the host fixes the item
// size for all of them: merge_grid_items.)  One workgroup per problem.
// ---------------------------------------------------------------------------------------
// paired (the level kernel that recomputes the stage times): inside the diagonal block of a chunk
// (rows 64c .. 64c+63, where row 64c+p has work only in the lanes from p on) the list holds the
// rows p = 0 .. 32 only; the kernel treats row 64c+p as the PAIR of rows 64c+p and 64c+64-p, whose
// lanes with work add up to exactly one wave.  The rows in front of the block and the listed rows
// of the block form two segments, and no item crosses from one into the other; the last item of a
// segment carries the number of rows that are left.
struct RunSegments { int lo0, n0, lo1, n1; };
__device__ __forceinline__ RunSegments run_segments(const ProblemDev &pr, int c, int paired) {
  RunSegments g;
  const int lo = pr.wlo[c], hi = min(64 * c + 63, pr.N - 1);
  g.lo0 = lo; g.n0 = lo <= hi ? hi - lo + 1 : 0; g.lo1 = 0; g.n1 = 0;
  if (paired && lo <= hi && hi >= 64 * c) {
    const int w = max(lo, 64 * c) - 64 * c, hmax = hi - 64 * c;  // window start and last row inside the block
    g.n0 = max(64 * c - lo, 0);
    // pairs p_lo .. p_top: every pair that holds a row of the window (a few more when the window
    // starts inside the block; their rows have no stage that fits and cost a skipped pass)
    const int p_lo = w == 0 ? 0 : 1, p_top = w <= 32 ? min(32, hmax) : min(31, 64 - w);
    g.lo1 = 64 * c + p_lo;
    g.n1 = max(p_top - p_lo + 1, 0);
  }
  return g;
}

__global__ __launch_bounds__(256) void runs_kernel(const ProblemDev *__restrict__ probs, int rows, int max_items,
                                                    int batch, int slots, int paired) {
  const ProblemDev &pr = probs[blockIdx.x];
  __shared__ int start[1025];  // nch <= 1024 (N <= 65535)
  __shared__ RunSegments seg[1024];  // every chunk's segments, computed once (one read of wlo per chunk)
  constexpr int NC = 16;  // candidate item sizes 4, 8, ..., 64 rows
  __shared__ int total_rows, count[NC];
  const int nch = pr.nch, tid = threadIdx.x;
  int32_t *const runs = pr.runs;  // (read once: the stores below would make the compiler fetch it again)
  for (int c = tid; c < nch; c += 256) seg[c] = run_segments(pr, c, paired);
  __syncthreads();
  if (rows <= 0) {
    if (tid < NC) count[tid] = 0;
    if (tid == 0) total_rows = 0;
    __syncthreads();
    // thread t counts the items of candidate size 4 (t % 16 + 1) over the chunks t / 16, t / 16 + 16, ...
    {
      const int k = tid % NC, r = 4 * (k + 1);
      int mine = 0, cnt = 0;
      for (int c = tid / NC; c < nch; c += 256 / NC) {
        const RunSegments g = seg[c];
        mine += g.n0 + g.n1;
        cnt += (g.n0 + r - 1) / r + (g.n1 + r - 1) / r;
      }
      if (k == 0 && mine) atomicAdd(&total_rows, mine);
      if (cnt) atomicAdd(&count[k], cnt);
    }
    __syncthreads();
    if (rows == 0) {
      rows = total_rows >= 16 * 1024 ? 16 : total_rows >= 8 * 1024 ? 8 : kSplitMinRows;
    } else {
      int pick = NC - 1;
      for (int k = NC - 1; k >= 0; --k)
        if (count[k] <= max_items) pick = k;
      if ((long long)count[pick] * batch > slots) {
        bool one_round = false;
        for (int k = pick + 1; k < NC; ++k) {
          const long long then = (long long)count[k] * batch;
          if (then <= slots) {
            if (2 * then >= slots) { pick = k; one_round = true; }
            break;
          }
        }
        // one large search of the recomputing form with many rounds: the largest items that still
        // leave three rounds, by the rows that are really there (the host, which fixes the size for
        // a launch over many searches, cannot see the pruning of a single one)
        if (!one_round && paired && batch == 1)
          for (int k = NC - 1; k > pick; --k)
            if (count[k] >= 3 * slots) { pick = k; break; }
      }
      rows = 4 * (pick + 1);
    }
  }
  // per chunk: items of the two segments, and their rows dealt evenly over them (33 rows in items
  // of up to 16: three items of 11, not 16 + 16 + 1); seg[c] is reused for {items0, per0, lo1, per1}
  __shared__ int n0_of[1024], n1_of[1024];
  for (int c = tid; c < nch; c += 256) {
    const RunSegments g = seg[c];
    const int items0 = (g.n0 + rows - 1) / rows, items1 = (g.n1 + rows - 1) / rows;
    start[c + 1] = items0 + items1;  // items of chunk c
    n0_of[c] = g.n0;
    n1_of[c] = g.n1;
    RunSegments h;
    h.lo0 = g.lo0; h.n0 = items0; h.lo1 = g.lo1;
    h.n1 = ((items0 ? (g.n0 + items0 - 1) / items0 : 0) << 8) | (items1 ? (g.n1 + items1 - 1) / items1 : 0);  // per0, per1 <= 64
    seg[c] = h;
  }
  __syncthreads();
  if (tid == 0) {
    start[0] = 0;
    for (int c = 0; c < nch; ++c) start[c + 1] += start[c];
    runs[0] = start[nch];
  }
  __syncthreads();
  const int total = start[nch];
  for (int e = tid; e < total; e += 256) {
    int lo = 0, hi = nch - 1;  // the chunk whose items contain e: start[c] <= e < start[c + 1]
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (start[mid + 1] <= e) lo = mid + 1;
      else hi = mid;
    }
    const int c = lo, k = e - start[c];
    const RunSegments h = seg[c];
    const int items0 = h.n0, per0 = h.n1 >> 8, per1 = h.n1 & 255;
    const int first = k < items0 ? h.lo0 + k * per0 : h.lo1 + (k - items0) * per1;
    const int left = k < items0 ? n0_of[c] - k * per0 : n1_of[c] - (k - items0) * per1;
    const int take = max(min(k < items0 ? per0 : per1, left), 1);  // (never below one row: the word stays well-formed)
    runs[1 + e] = ((take - 1) << 26) | (c << 16) | first;
  }
}

// ---------------------------------------------------------------------------------------
// DP level s >= 2, sorted-merge form.
//
// For a fixed stage (i,j) the recurrence of Sec. III-C needs, for every device total d,
//     W[d] = min over d' + r = d of max(a[d'], c[r]),   a[d'] = V[s-1][i][d'], c[r] = h(i,j,r)
// (INF where r does not fit).  Both sequences are non-increasing: giving one more device to
// the last stage of a plan can only lower its time and its memory, and h, m are non-increasing
// in r.  For such sequences, W[d] <= x  <=>  (number of a's > x) + (number of c's > x) <= d-2,
// i.e. W[d] is the (d-1)-th largest element of the merged multiset {a[1..]} U {c[1..]}.  A wave
// therefore merges the two sorted D-vectors with a bitonic network held in registers
// (DP*(log2 DP + 1) max/min operations instead of D^2/2 max-min pairs) and folds the result into
// a per-lane running minimum over i.  V[s][j][d] = min over i of W[d] is then the value the
// five nested loops of Algorithm 1 produce; which (i,d') attains it is recovered where it is
// needed (traceback, table export) by the first-match scan, not carried here.
//
// Only replica counts r <= D-s+1 can occur at level s (s-1 devices are spent on the earlier
// stages); the larger ones rank below position D-1 of the merge, so they are not read.
//
// Work item (one workgroup of four waves) = 4 to 64 consecutive rows of one chunk's window,
// taken from the work list; wave w takes rows i0+w, i0+w+4, ... one after the other and keeps the
// running minimum over them in registers (one value array for the row in flight, one for the
// minimum: three waves per SIMD, i.e. three workgroups per compute unit, whose memory, merge and
// fold phases overlap).  A lane owns column jj = 64c + lane.  a[] is wave-uniform (one row of
// V[s-1], scalar loads), c[] comes from coalesced reads of one contiguous unit; the flags of the
// next row are fetched while the current one is merged.  The four waves then fold their minima
// together in LDS, and one transposed pass of device-scope atomicMin into V[s] (pre-filled with
// INF) combines the items of a chunk: min is order-independent, so the result is deterministic.
// ---------------------------------------------------------------------------------------
// One row's sorted merge: x := the DP largest elements of merge(a, c), sorted descending, for the
// lane's stage; all INF for a lane without work (`off` = INF there, 0 elsewhere).
//
// x[DP-1-m] = c[m+1]: reversed, so that max(a, x) is a bitonic sequence; then log2(DP) compare-
// exchange stages.  Replica counts beyond rl cannot occur at this level and rank below everything
// that matters in the merge.  NG = ceil(rl / 8) is a compile-time number, so that the reads of a
// row are one straight run of independent loads: the groups of eight rows beyond it are taken as
// 0, and inside the last group the row index is clamped to rl-1 (the repeated value keeps the
// sequence sorted, stays below rank D-1, and costs no memory traffic).  `unit` points at the
// lane's column, or for a lane without work at the column of a lane that has some (every load
// instruction then touches only lines that are needed); such a lane is switched off by folding
// `off` into the first maximum, which makes its whole result INF.
template <typename VT, int DP, int NG, typename AP>
__device__ __forceinline__ void row_merge(VT (&x)[DP], const VT RANNC_GLOBAL *__restrict__ unit, AP arow,
                                          VT off, int rl) {
#pragma unroll
  for (int m = 0; m < DP; ++m) {
    if (m < 8 * (NG - 1)) x[DP - 1 - m] = unit[m * 64];
    else if (m == 8 * (NG - 1)) x[DP - 1 - m] = unit[m * 64];       // 8(NG-1) <= rl-1: never clamped
    else if (m < 8 * NG) x[DP - 1 - m] = unit[min(m, rl - 1) * 64];  // wave-uniform clamp
    else x[DP - 1 - m] = (VT)0;
  }
#pragma unroll
  for (int q = 0; q < DP; ++q) {
    if constexpr (std::is_same<AP, const VT RANNC_GLOBAL *>::value) x[q] = vmax(vmax_su(arow[q], x[q]), off);
    else x[q] = vmax(vmax(arow[q], x[q]), off);
  }
#pragma unroll
  for (int h = DP / 2; h >= 1; h >>= 1) {
#pragma unroll
    for (int q = 0; q < DP; ++q) {
      if ((q & h) == 0) {
        const VT hi = vmax(x[q], x[q + h]);
        const VT lo = vmin(x[q], x[q + h]);
        x[q] = hi;
        x[q + h] = lo;
      }
    }
  }
}

// The same for a level kernel that recomputes the stage times instead of reading their table (32-bit
// values, no communication term): the lane's stage has total time tij, fits from rmn replicas on
// (255: never, or a lane without work), and c[r] = ceil(tij / r), INF for r < rmn.
//
// ceil(x / r) for 0 <= x < 2^32 and odd r <= 63 without an integer division, in double precision:
//     t = x + (r/2 - 1 + r * 2^-18)            exact (a multiple of 2^-18 below 2^33)
//     y = t * (1/r) + 1.5 * 2^52               one fused multiply-add
// t / r = (x + r - 1)/r - 1/2 + 2^-18; the fraction of (x + r - 1)/r is a multiple of 1/r, at most
// 62/63, and the rounded 1/r puts the product off by less than 2^-21, so t * (1/r) lies strictly
// between k - 1/2 and k + 1/2 for k = floor((x + r - 1) / r): the addition of 1.5 * 2^52 rounds it to
// that integer and leaves k in the low word of the sum.  Even replica counts follow from
// ceil(x / 2r) = ceil(ceil(x / r) / 2): an add and a shift.  Two full-rate instructions per entry.
// The 32 reciprocals and 1.5 * 2^52 live in vector registers for the whole kernel (as immediate
// operands they would need one scalar register pair each, which do not exist in that number).
// The INF below rmn comes from a per-lane bit mask (bit r-1 set for r < rmn), one bit-field extract
// per entry, folded into the first maximum of the merge together with a[].
struct DirectConsts {
  double inv[32];  // 1 / (2k + 1)
  double magic;    // 1.5 * 2^52
};
__device__ __forceinline__ void direct_consts_init(DirectConsts &k) {
#pragma unroll
  for (int q = 0; q < 32; ++q) {
    k.inv[q] = 1.0 / (double)(2 * q + 1);
    asm("" : "+v"(k.inv[q]));  // a register, not an immediate (not volatile: no memory effects)
  }
  k.magic = 0x1.8p52;
  asm("" : "+v"(k.magic));
}

// The same with 64-bit values, for stage times below 2^40 (the caller's bound on a search's total
// time guarantees it): the offset is 2^-8 instead of 2^-18, so that t stays exact (a multiple of 2^-8
// below 2^41: 49 bits) while the rounded reciprocal moves the product by less than 2^41 * 2^-53 =
// 2^-12, far inside both margins (2^-8 below, 1/63 - 2^-8 above).  The quotient, below 2^40, sits in
// the low 51 bits of the sum; the even counts are a 64-bit add and shift.
template <typename VT> struct DirectArith;
template <> struct DirectArith<uint32_t> {
  static constexpr double kOffset = 0x1p-18;
  static __device__ __forceinline__ uint32_t quotient(double y) { return (uint32_t)__double_as_longlong(y); }
  // 0 or INF from bit (m & 31) of the mask word
  static __device__ __forceinline__ uint32_t inf_if(int word, int m) {
    return (uint32_t)__builtin_amdgcn_sbfe(word, m & 31, 1);
  }
};
template <> struct DirectArith<uint64_t> {
  static constexpr double kOffset = 0x1p-8;
  static __device__ __forceinline__ uint64_t quotient(double y) {
    return (uint64_t)__double_as_longlong(y) & ((1ull << 51) - 1ull);
  }
  static __device__ __forceinline__ uint64_t inf_if(int word, int m) {
    return (uint64_t)((uint32_t)__builtin_amdgcn_sbfe(word, m & 31, 1) & (uint32_t)(Lim<uint64_t>::inf >> 32)) << 32;
  }
};
// largest stage time the 64-bit form is exact for
constexpr int64_t kDirectWideMaxTime = (int64_t)1 << 40;

// AP of the helpers below: x[] already holds the lane's own a[] row (read per lane, not wave-uniform)
struct InPlaceRow {};

// entry r = ODD << SH and the ones it is the parent of
template <typename VT, int DP, int NG, int ODD, int SH, typename AP>
__device__ __forceinline__ void direct_chain(VT (&x)[DP], AP arow, VT q_odd, int mlo, int mhi) {
  constexpr int R = ODD << SH, M = R - 1;
  if constexpr (R <= 8 * NG && R <= DP) {
    const VT h = SH == 0 ? q_odd : (q_odd + (VT)((1u << SH) - 1u)) >> SH;
    const VT inf = DirectArith<VT>::inf_if(M < 32 ? mlo : mhi, M);
    if constexpr (std::is_same<AP, InPlaceRow>::value) x[DP - 1 - M] = vmax(vmax(x[DP - 1 - M], h), inf);
    else x[DP - 1 - M] = vmax(vmax((VT)arow[DP - 1 - M], h), inf);
    direct_chain<VT, DP, NG, ODD, SH + 1, AP>(x, arow, q_odd, mlo, mhi);
  }
}

// t = x + (r/2 - 1 + r * offset) for the odd r = 2K + 1; the next odd r adds 1 + 2 * offset (exact:
// every t is a multiple of the offset inside the 53 bits), so one constant serves all entries
template <typename VT, int DP, int NG, typename AP, int K = 0>
__device__ __forceinline__ void direct_entries(VT (&x)[DP], AP arow, double t, const DirectConsts &k, int mlo,
                                               int mhi) {
  constexpr int ODD = 2 * K + 1;
  if constexpr (ODD <= 8 * NG && ODD <= DP) {
    const double y = __builtin_fma(t, k.inv[K], k.magic);
    direct_chain<VT, DP, NG, ODD, 0, AP>(x, arow, DirectArith<VT>::quotient(y), mlo, mhi);
    direct_entries<VT, DP, NG, AP, K + 1>(x, arow, t + (1.0 + 2.0 * DirectArith<VT>::kOffset), k, mlo, mhi);
  }
}

template <typename VT, int DP, int NG, typename AP>
__device__ __forceinline__ void row_merge_direct(VT (&x)[DP], AP arow, VT tij, int rmn, const DirectConsts &k) {
  // bit r-1 set for r < rmn: these replica counts do not fit (all of them for rmn = 255)
  const unsigned long long below = rmn > 64 ? ~0ull : ((1ull << (rmn - 1)) - 1ull);
  if constexpr (!std::is_same<AP, InPlaceRow>::value) {
#pragma unroll
    for (int m = 8 * NG; m < DP; ++m) x[DP - 1 - m] = arow[DP - 1 - m];  // max(a, 0): replica counts not needed
  }
  direct_entries<VT, DP, NG, AP>(x, arow, (double)tij + (DirectArith<VT>::kOffset - 0.5), k, (int)(uint32_t)below,
                                 (int)(uint32_t)(below >> 32));
#pragma unroll
  for (int h = DP / 2; h >= 1; h >>= 1) {
#pragma unroll
    for (int q = 0; q < DP; ++q) {
      if ((q & h) == 0) {
        const VT hi = vmax(x[q], x[q + h]);
        const VT lo = vmin(x[q], x[q + h]);
        x[q] = hi;
        x[q + h] = lo;
      }
    }
  }
}

// merge_rows for the recomputing level kernel: no table reads; per row one scalar read of T[i], the
// lane's rmin byte and the a[] row.
template <int DP, int NG>
__device__ __forceinline__ bool merge_rows_direct(uint32_t (&acc)[DP], uint32_t *tile, const ProblemDev &pr, const int s,
                                                  const int c, const int i0, const int i_hi, const int lane,
                                                  const int wave, const DirectConsts &k) {
  using VT = uint32_t;
  constexpr VT INF = Lim<VT>::inf;
  const int N = pr.N, D = pr.D, nch = pr.nch;
  const int jj = 64 * c + lane;
  const int64_t lvl = (int64_t)(N + 1) * DP;
  const VT RANNC_GLOBAL *__restrict__ Vprev = gptr((const VT *)pr.V) + (int64_t)(s - 2) * lvl;
  const uint8_t RANNC_GLOBAL *__restrict__ rmin = gptr((const uint8_t *)pr.rmin);
  const int64_t RANNC_GLOBAL *__restrict__ T = gptr((const int64_t *)pr.T);
  const int rl = D - s + 1;
  const int64_t Tj = T[min(jj + 1, N)];  // the lane's column (clamped: lanes beyond N have no work)
  // only the loads happen here, unconditionally; the values are looked at one iteration later (see
  // merge_rows)
  struct Row { VT alast; int rmn; int64_t Ti; };
  auto load_flags = [&](int i) -> Row {
    const int ic = min(max(i, s - 1), i_hi);
    Row r;
    r.alast = Vprev[(int64_t)ic * DP + D - 1];
    r.Ti = T[ic];
    r.rmn = rmin[unit_index(nch, ic, c) * 64 + lane];
    return r;
  };
  bool any = false;
  if (i0 >= 64 * c) {
    // Diagonal block: the listed row 64c+p stands for the pair of rows 64c+p (lanes p.. with their
    // own columns) and 64c+64-p (the p columns from 64-p on, on the lanes below p): one pass of a
    // full wave instead of two half-empty ones.  Every lane reads its own row of V[s-1] (straight
    // into the registers it is merged in), prefix sum and rmin byte.  The lanes of the second row
    // do not own their column, so their merge goes straight into the workgroup's tile.
    typedef uint32_t Quad __attribute__((ext_vector_type(4)));
    struct Pair { VT alast; int rmn; int64_t Ti, Tc; int row, col; };
    auto load_pair = [&](int p) -> Pair {
      const int pc = min(max(p, 0), 32);
      const bool second = lane < pc && pc < 32;  // rows 64c and 64c+32 have no partner
      Pair r;
      r.col = second ? lane + 64 - pc : lane;
      r.row = lane >= pc ? 64 * c + pc : second ? 64 * c + 64 - pc : -1;
      const int rc = min(max(r.row, s - 1), N - 1);  // in range for the reads; the row itself decides below
      r.alast = Vprev[(int64_t)rc * DP + D - 1];
      r.Ti = T[rc];
      r.Tc = T[min(64 * c + r.col + 1, N)];
      r.rmn = rmin[unit_index(nch, rc, c) * 64 + r.col];
      return r;
    };
    int p = i0 - 64 * c + wave;
    const int p_hi = i_hi - 64 * c;
    Pair cur = load_pair(p);
    while (p <= p_hi) {  // wave-uniform
      const int row = cur.row, col = cur.col;
      const bool act = row >= s - 1 && row < N && 64 * c + col < N && cur.alast != INF && cur.rmn <= rl;
      const uint32_t tij = (uint32_t)(cur.Tc - cur.Ti);
      const int rmn = act ? cur.rmn : 255;
      const int rc = min(max(row, s - 1), N - 1);
      cur = load_pair(p + kMergeWaves);
      if (__ballot(act) != 0ull) {
        any = true;
        VT x[DP];
        const Quad RANNC_GLOBAL *ap = (const Quad RANNC_GLOBAL *)(Vprev + (int64_t)rc * DP);
#pragma unroll
        for (int g = 0; g < DP / 4; ++g) {
          const Quad v = ap[g];
          x[4 * g] = v.x; x[4 * g + 1] = v.y; x[4 * g + 2] = v.z; x[4 * g + 3] = v.w;
        }
        row_merge_direct<uint32_t, DP, NG, InPlaceRow>(x, InPlaceRow(), tij, rmn, k);
        if (col == lane) {
#pragma unroll
          for (int t = 0; t < DP; ++t) acc[t] = vmin(acc[t], x[t]);
        } else if (act) {
#pragma unroll
          for (int t = 0; t < DP; ++t) atomicMin(&tile[col * (DP + 1) + t], x[t]);
        }
      }
      p += kMergeWaves;
    }
    return any;
  }
  int i = i0 + wave;
  Row cur = load_flags(i);
  while (i <= i_hi) {  // wave-uniform
    const bool act = i >= s - 1 && cur.alast != INF && jj >= i && jj < N && cur.rmn <= rl;
    const uint32_t tij = (uint32_t)(Tj - cur.Ti);
    const int rmn = act ? cur.rmn : 255;
    cur = load_flags(i + kMergeWaves);  // the next row's
    if (__ballot(act) != 0ull) {
      any = true;
      VT x[DP];
      row_merge_direct<uint32_t, DP, NG, const uint32_t RANNC_GLOBAL *>(x, Vprev + (int64_t)i * DP, tij, rmn, k);
#pragma unroll
      for (int t = 0; t < DP; ++t) acc[t] = vmin(acc[t], x[t]);
    }
    i += kMergeWaves;
  }
  return any;
}

// Waves per SIMD the level kernel is compiled for: the two value arrays of the widest 32-bit case
// fit the 168 registers of three waves per SIMD (the compiler left alone takes one more); the
// recomputing kernel also keeps 32 reciprocals in registers and runs two waves per SIMD.
template <typename VT, int DP, bool DIRECT> constexpr int merge_waves_per_simd() {
  return DP == 64 ? (sizeof(VT) == 4 ? (DIRECT ? 2 : 3) : 2) : (DP == 32 && DIRECT) ? 4 : 1;
}

// The rows i0+wave, i0+wave+4, ... <= i_hi of one work item, folded into acc (running minimum of the
// sorted merges).  Returns whether any row had work.
// ROWFOLD: the sorted merge of every row goes straight into the lane's row of the workgroup's LDS
// tile instead of a running minimum in registers (64-bit values at DP = 64: two value arrays would
// take all 256 registers of a wave and leave one wave per SIMD).
template <typename VT, int DP, int NG, bool ROWFOLD>
__device__ __forceinline__ bool merge_rows(VT (&acc)[DP], VT *tile_lane, const ProblemDev &pr, const int s,
                                           const int c, const int i0, const int i_hi, const int lane,
                                           const int wave) {
  constexpr VT INF = Lim<VT>::inf;
  const int N = pr.N, D = pr.D, nch = pr.nch;
  const int jj = 64 * c + lane;
  const int64_t lvl = (int64_t)(N + 1) * DP;
  const VT RANNC_GLOBAL *__restrict__ Vprev = gptr((const VT *)pr.V) + (int64_t)(s - 2) * lvl;
  const VT RANNC_GLOBAL *__restrict__ cost = gptr((const VT *)pr.cost);
  const uint8_t RANNC_GLOBAL *__restrict__ rmin = gptr((const uint8_t *)pr.rmin);
  const int rl = D - s + 1;  // replicas left for stage s when s-1 devices are spent earlier
  // Flags of a row: it can contribute if its row of V[s-1] holds a finite plan and the lane's
  // stage fits with at most rl replicas.  Only the loads happen here; the values are looked at one
  // iteration later, so that the wait for them never stands between a row and its own unit reads.
  // The loads are unconditional (rows outside the item are clamped to a row inside it, every column
  // of a unit has its rmin byte in memory): a load inside a branch would be waited for where the
  // branch ends.
  struct Flags { VT alast; int rmn; int64_t ubase; };
  auto load_flags = [&](int i) -> Flags {
    const int ic = min(max(i, s - 1), i_hi);
    Flags f;
    f.ubase = unit_index(nch, ic, c);
    f.alast = Vprev[(int64_t)ic * DP + D - 1];
    f.rmn = rmin[f.ubase * 64 + lane];
    return f;
  };
  bool any = false;
  int i = i0 + wave;
  Flags cur = load_flags(i);
  while (i <= i_hi) {  // wave-uniform
    const bool act = i >= s - 1 && cur.alast != INF && jj >= i && jj < N && cur.rmn <= rl;
    const int64_t ubase = cur.ubase;
    cur = load_flags(i + kMergeWaves);  // the next row's
    const unsigned long long work = __ballot(act);
    if (work != 0ull) {
      any = true;
      VT x[DP];
      const int col = act ? lane : __ffsll((long long)work) - 1;  // a lane without work reads a needed column
      row_merge<VT, DP, NG, const VT RANNC_GLOBAL *>(x, cost + ubase * 64 * D + col, Vprev + (int64_t)i * DP,
                                                     act ? (VT)0 : INF, rl);
      if constexpr (ROWFOLD) {
        if (act) {
#pragma unroll
          for (int t = 0; t < DP; ++t) atomicMin(&tile_lane[t], x[t]);
        }
      } else {
#pragma unroll
        for (int t = 0; t < DP; ++t) acc[t] = vmin(acc[t], x[t]);
      }
    }
    i += kMergeWaves;
  }
  return any;
}

template <typename VT, int DP, bool DIRECT>
__device__ __forceinline__ void level_merge_body(const ProblemDev &pr, const int s, const int item) {
  if (s > pr.S_eff) return;
  const int N = pr.N, D = pr.D;
  const int32_t RANNC_GLOBAL *__restrict__ runs = gptr((const int32_t *)pr.runs);
  if (item >= runs[0]) return;
  const unsigned desc = (unsigned)runs[1 + item];
  const int c = (int)((desc >> 16) & 0x3ffu), i0 = (int)(desc & 0xffffu), rows = (int)(desc >> 26) + 1;
  if (64 * c + 64 < s) return;  // no column j >= s in this chunk
  const int i_hi = min(min(i0 + rows - 1, 64 * c + 63), N - 1);
  // (an item of the diagonal block of the recomputing kernel also stands for the partner rows
  // 64c+64-p of its rows 64c+p, which lie above them)
  if (i_hi < s - 1 && !(DIRECT && i0 >= 64 * c)) return;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  constexpr VT INF = Lim<VT>::inf;
  VT RANNC_GLOBAL *Vcur = gptr((VT *)pr.V) + (int64_t)(s - 1) * (int64_t)(N + 1) * DP;

  // acc[t] = running minimum over this wave's rows of the sorted merge
  constexpr bool ROWFOLD = sizeof(VT) == 8 && DP == 64;
  constexpr bool EARLY_TILE = ROWFOLD || DIRECT;  // rows fold into the tile while the row loop runs
  __shared__ VT tile[64 * (DP + 1)];
  [[maybe_unused]] VT acc[DP];
  if constexpr (EARLY_TILE) {
    for (int e = threadIdx.x; e < 64 * (DP + 1); e += 64 * kMergeWaves) tile[e] = INF;
    __syncthreads();
  }
  if constexpr (!ROWFOLD) {
#pragma unroll
    for (int t = 0; t < DP; ++t) acc[t] = INF;
  }
  bool any = false;
  const int ng = (D - s + 1 + 7) >> 3;  // eight-row groups of a unit that this level needs
  if constexpr (DIRECT) {
    // stage times recomputed: groups in pairs (fewer variants; a group more costs a few instructions)
    DirectConsts k;
    direct_consts_init(k);
#define RANNC_ROWS(K)                                                                              \
  case K:                                                                                          \
    if constexpr (8 * K <= DP || (K == 1 && DP == 8))                                              \
      any = merge_rows_direct<DP, (8 * K <= DP ? K : 1)>(acc, tile, pr, s, c, i0, i_hi, lane, wave, k);  \
    break;
    switch (DP == 8 ? 1 : ((ng + 1) & ~1)) {
      RANNC_ROWS(1) RANNC_ROWS(2) RANNC_ROWS(4) RANNC_ROWS(6) RANNC_ROWS(8)
      default: break;
    }
#undef RANNC_ROWS
  } else {
#define RANNC_ROWS(K)                                                                     \
  case K:                                                                                 \
    if constexpr (8 * K <= DP)                                                            \
      any = merge_rows<VT, DP, K, ROWFOLD>(acc, tile + lane * (DP + 1), pr, s, c, i0, i_hi, lane, wave); \
    break;
    switch (ng) {
      RANNC_ROWS(1) RANNC_ROWS(2) RANNC_ROWS(3) RANNC_ROWS(4)
      RANNC_ROWS(5) RANNC_ROWS(6) RANNC_ROWS(7) RANNC_ROWS(8)
      default: break;
    }
#undef RANNC_ROWS
  }

  // acc[t] is W[d = t+2]; V rows are indexed by d-1 = t+1.  Fold the waves in LDS, then
  // write transposed so that one atomic instruction covers consecutive d of one column.
  if constexpr (ROWFOLD) {
    if (__syncthreads_or(any) == 0) return;
  } else {
    if constexpr (!EARLY_TILE)
      for (int e = threadIdx.x; e < 64 * (DP + 1); e += 64 * kMergeWaves) tile[e] = INF;
    if (__syncthreads_or(any) == 0) return;
    if (any) {
#pragma unroll
      for (int t = 0; t < DP; ++t) atomicMin(&tile[lane * (DP + 1) + t], acc[t]);  // folding INF in is a no-op
    }
    __syncthreads();
  }
  constexpr int RPP = 64 * kMergeWaves / DP;  // rows per pass
  const int t = threadIdx.x & (DP - 1);
  for (int row = threadIdx.x / DP; row < 64; row += RPP) {
    const VT v = tile[row * (DP + 1) + t];
    const int j = 64 * c + row + 1;
    if (t + 1 <= D - 1 && j <= N && j >= s && v != INF) global_min(&Vcur[(int64_t)j * DP + t + 1], v);
  }
}

template <typename VT, int DP, bool DIRECT>
__global__ __launch_bounds__(64 * kMergeWaves) __attribute__((amdgpu_waves_per_eu(merge_waves_per_simd<VT, DP, DIRECT>())))
void level_merge_kernel(const ProblemDev *__restrict__ probs, const int s, const int search_major) {
  // Workgroups go to the eight XCDs round-robin in the order of their linear index.  With the items
  // of a search next to each other (search_major) and, say, four items per search, item k of every
  // search lands on XCDs k and k + 4: the XCDs with the long items finish last and those with the
  // empty ones idle (config 5: 176 against 121 us per level).  In a launch of the recomputing form
  // over several searches the search index therefore runs fastest: every XCD gets every kind of item.
  if (search_major) level_merge_body<VT, DP, DIRECT>(probs[blockIdx.z], s, (int)blockIdx.x);
  else level_merge_body<VT, DP, DIRECT>(probs[blockIdx.x], s, (int)blockIdx.z);
}

// The same for a launch over ONE search, with the descriptor as a kernel argument: a workgroup then
// starts with its fields in scalar registers instead of fetching them through the descriptor
// array's pointer, one memory round trip less in a launch that consists of a few of them.
template <typename VT, int DP, bool DIRECT>
__global__ __launch_bounds__(64 * kMergeWaves) __attribute__((amdgpu_waves_per_eu(merge_waves_per_simd<VT, DP, DIRECT>())))
void level_merge_one_kernel(const ProblemDev pr, const int s) {
  level_merge_body<VT, DP, DIRECT>(pr, s, (int)blockIdx.x);
}

// ---------------------------------------------------------------------------------------
// Whole search of a SMALL problem (N <= 128, i.e. at most two column chunks) in one workgroup and
// one launch: prefix sums, tables, every level, choice of the stage count.  Same arithmetic as the
// kernels above (the same build_unit / row_merge), but two consecutive levels of V
// live in LDS, so the waves of the workgroup fold their merges with LDS atomics and meet at
// workgroup barriers: no launch per level, no global atomics.  Every level is also copied to the
// V table in memory (plan recovery and export read it there).  Meant for searches at the
// paper's own scale (k = 32 blocks, D <= 32, Sec. IV-A) and for batches of them (the many
// form_stage_dp calls of Algorithm 2): one workgroup per search.
// ---------------------------------------------------------------------------------------
constexpr int kSmallMaxN = 128;
// Sixteen waves per search, eight where a lane's value array alone takes 64 registers or more (64
// devices, or 64-bit values from 32 devices on): with the 128 registers of sixteen waves those
// kernels spilled up to 1 600 registers per lane.
constexpr int kSmallWavesMax = 16;
template <typename VT, int DP> constexpr int small_waves() { return sizeof(VT) * DP >= 256 ? 8 : kSmallWavesMax; }

__device__ __forceinline__ void select_finish(const ProblemDev &pr, int64_t v, int st, int64_t *d_opt,
                                              int32_t *d_n_stages, int64_t *d_est, int32_t *d_status);

// Waves per SIMD the one-launch kernel is compiled for.  The recomputing form on 32-bit values at 16
// devices needs 70 registers left alone, one wave per SIMD short of TWO workgroups per compute unit
// (16 waves each); held to 64 registers the two rounds of a batch of 512 searches run side by side.
template <typename VT, int DP, bool DIRECT> constexpr int small_waves_per_simd() {
  return (DIRECT && sizeof(VT) == 4 && DP == 16) ? 8 : small_waves<VT, DP>() / 4;
}

template <typename VT, int DP, bool DIRECT>
__global__ __launch_bounds__((64 * small_waves<VT, DP>())) __attribute__((amdgpu_waves_per_eu((small_waves_per_simd<VT, DP, DIRECT>()))))
void solve_small_kernel(
    const ProblemDev *__restrict__ probs, int64_t *d_opt, int32_t *d_n_stages, int64_t *d_est,
    int32_t *d_status) {
  const ProblemDev &pr = probs[blockIdx.x];
  constexpr VT INF = Lim<VT>::inf;
  constexpr int LS = DP + 1;  // row stride of a level in LDS: lanes (= columns) hit different banks
  constexpr int kSmallWaves = small_waves<VT, DP>();
  constexpr int NT = 64 * kSmallWaves;
  __shared__ int64_t sT[kSmallMaxN + 1], sP[kSmallMaxN + 1], sA[kSmallMaxN + 1], sC[kSmallMaxN + 1];
  __shared__ unsigned long long s_max_cut;
  __shared__ uint64_t scan[3][kSmallMaxN];
  // levels of V in LDS: the one being read and the one being folded into; the recomputing form keeps
  // a third, cleared while a level runs, so that a level costs one workgroup barrier instead of two
  constexpr int kLevelBufs = DIRECT ? 3 : 2;
  __shared__ VT lv[kLevelBufs][(kSmallMaxN + 1) * LS];
  __shared__ VT s_top[64];
  __shared__ int s_flags, s_wlo[2];
  // DIRECT: the stage times are recomputed from the prefix sums in LDS (as the recomputing level
  // kernel does), and the fits-in-memory bytes of all units stay in LDS too: no table is written and
  // the levels read nothing from memory
  constexpr int kUnits = kSmallMaxN + 64;  // 64 rows of chunk 0, then up to 128 rows of chunk 1
  __shared__ uint8_t s_rmin[DIRECT ? kUnits * 64 : 64];
  const int N = pr.N, D = pr.D, nch = pr.nch, S_eff = pr.S_eff;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- prefix sums and validation (as prefix_kernel) ----
  if (tid == 0) {
    s_flags = 0; s_wlo[0] = kNoRow; s_wlo[1] = kNoRow; s_max_cut = 0ull; sC[0] = 0;
    if (pr.o) pr.C[0] = 0;
  }
  int myflags = 0;
  __syncthreads();
  if (tid < N && pr.o) {  // per-cut send time (as prefix_kernel)
    const uint64_t c = cut_time(pr.o[tid], pr.bw, myflags);
    sC[tid + 1] = (tid + 1 < N) ? (int64_t)c : 0;
    pr.C[tid + 1] = sC[tid + 1];  // plan recovery values the stages from the prefix sums in memory
    if (tid + 1 < N && c) atomicMax(&s_max_cut, (unsigned long long)c);
  }
  if (tid < N) {
    const int64_t *in[3] = {pr.t, pr.p, pr.a};
    for (int w = 0; w < 3; ++w) {
      int64_t v = in[w][tid];
      if (v < 0) { myflags |= 1; v = 0; }
      uint64_t u = (uint64_t)v;
      if (u >= kSumLimit) { myflags |= 2; u = kSumLimit; }
      scan[w][tid] = u;
    }
  }
  __syncthreads();
  for (int off = 1; off < kSmallMaxN; off <<= 1) {
    uint64_t add[3] = {0, 0, 0};
    if (tid < N && tid >= off)
      for (int w = 0; w < 3; ++w) add[w] = scan[w][tid - off];
    __syncthreads();
    if (tid < N)
      for (int w = 0; w < 3; ++w) {
        const uint64_t v = scan[w][tid] + add[w];
        scan[w][tid] = v > kSumLimit ? kSumLimit : v;
      }
    __syncthreads();
  }
  if (tid < N) {
    if (scan[0][tid] >= kSumLimit || scan[1][tid] >= kSumLimit || scan[2][tid] >= kSumLimit) myflags |= 2;
    sT[tid + 1] = (int64_t)scan[0][tid]; sP[tid + 1] = (int64_t)scan[1][tid]; sA[tid + 1] = (int64_t)scan[2][tid];
    pr.T[tid + 1] = sT[tid + 1]; pr.P[tid + 1] = sP[tid + 1]; pr.A[tid + 1] = sA[tid + 1];
  }
  if (tid == 0) { sT[0] = sP[0] = sA[0] = 0; pr.T[0] = pr.P[0] = pr.A[0] = 0; }
  if (myflags) atomicOr(&s_flags, myflags);
  // level 1 buffer: "no plan" everywhere, padding columns 0
  for (int e = tid; e < (N + 1) * LS; e += NT) lv[0][e] = ((e % LS) < D) ? INF : (VT)0;
  if constexpr (DIRECT)  // level 2's buffer as well
    for (int e = tid; e < (N + 1) * LS; e += NT) lv[1][e] = ((e % LS) < D) ? INF : (VT)0;
  __syncthreads();
  int st = RANNC_DP_PROBLEM_OK;
  if (s_flags & 1) st = RANNC_DP_PROBLEM_NEGATIVE_INPUT;
  else if (s_flags & 2) st = RANNC_DP_PROBLEM_SUM_OVERFLOW;
  else if ((uint64_t)sT[N] + s_max_cut > (uint64_t)pr.time_limit) st = RANNC_DP_PROBLEM_TIME_TOO_LARGE;
  if (tid == 0) *pr.status = st;

  // ---- tables (as build_kernel): rows 0..min(63,N-1) of chunk 0, then rows 0..N-1 of chunk 1 ----
  const int R0 = min(64, N), RT = R0 + (nch > 1 ? N : 0);
  for (int f = wave; f < RT; f += kSmallWaves) {
    const int c = f >= R0, i = c ? f - R0 : f;
    const bool fits = build_unit<VT, DP>(pr, sT, sP, sA, pr.o ? sC : nullptr, i, c, lane, lv[0], LS, 0, nullptr,
                                         !DIRECT, DIRECT ? s_rmin + f * 64 : nullptr);
    if (fits && lane == 0) atomicMin(&s_wlo[c], i);
  }
  __syncthreads();
  if (tid < nch) pr.wlo[tid] = s_wlo[tid];
  const int64_t lvl = (int64_t)(N + 1) * DP;
  VT RANNC_GLOBAL *Vg = gptr((VT *)pr.V);
  const VT RANNC_GLOBAL *cost = gptr((const VT *)pr.cost);
  const uint8_t RANNC_GLOBAL *rmin = gptr((const uint8_t *)pr.rmin);
  // level 1 to memory
  for (int e = tid; e < (N + 1) * DP; e += NT) Vg[e] = lv[0][(e / DP) * LS + (e % DP)];
  if (tid == 0) s_top[0] = lv[0][N * LS + D - 1];

  // ---- levels 2..S_eff ----
  [[maybe_unused]] DirectConsts kc;
  if constexpr (DIRECT) direct_consts_init(kc);
  // passes of the recomputing form (see the level loop): P0 for the triangle of chunk 0, then F1 for
  // the rectangle and P1 for the triangle of chunk 1
  const int W0 = R0, W1 = nch > 1 ? N - 64 : 1;
  const int lg0 = W0 > 1 ? 32 - __builtin_clz(W0 - 1) : 0, lg1 = W1 > 1 ? 32 - __builtin_clz(W1 - 1) : 0;
  const int P0 = (W0 / 2 + (64 >> lg0)) >> (6 - lg0);
  const int F1 = nch > 1 ? 64 >> (6 - lg1) : 0;
  const int P1 = nch > 1 ? (W1 / 2 + (64 >> lg1)) >> (6 - lg1) : 0;
  [[maybe_unused]] const int RTP = P0 + F1 + P1;
  for (int s = 2; s <= S_eff; ++s) {
    // level s lives in buffer (s-1) mod kLevelBufs
    const VT *prev = lv[(s - 2) % kLevelBufs];  // level s-1
    VT *cur = lv[(s - 1) % kLevelBufs];         // level s
    const int rl = D - s + 1;
    if constexpr (!DIRECT) {
      for (int e = tid; e < (N + 1) * LS; e += NT) cur[e] = ((e % LS) < D) ? INF : (VT)0;
      lds_barrier();  // LDS only: the copy of the previous level to memory stays in flight
    }
    if constexpr (DIRECT) {
      // One pass of a wave = 64 (row, column) pairs, one per lane, so that no lane idles on the
      // triangular blocks.  A diagonal block of W columns (rows base..base+W-1) is cut into groups of
      // LG = 2^lg >= W lanes, G = 64 / LG groups to a pass; group number p (0..W/2) covers row base+p on
      // the lanes l >= p (columns l) and, for 0 < p < W-p, row base+W-p on the lanes l < p (columns
      // l+W-p): W lanes of work where a row alone has W-p.  The rectangular block of chunk 1 (rows
      // 0..63, W1 columns) runs G1 rows to a pass the same way.  Every lane reads its own a[] row
      // from LDS and folds its own column in, so a pass may mix rows freely.
      for (int f = wave; f < RTP; f += kSmallWaves) {
        const int c = f >= P0;
        if (64 * c + 64 < s) continue;
        int row, col;
        bool valid;
        if (c && f < P0 + F1) {
          const int l = lane & ((1 << lg1) - 1);
          row = ((f - P0) << (6 - lg1)) + (lane >> lg1);
          col = l;
          valid = l < W1;
        } else {
          const int W = c ? W1 : W0, lg = c ? lg1 : lg0;
          const int l = lane & ((1 << lg) - 1);
          const int p = ((c ? f - P0 - F1 : f) << (6 - lg)) + (lane >> lg);
          const bool second = l < p;
          valid = l < W && 2 * p <= W && (!second || 2 * p < W);
          row = 64 * c + (second ? W - p : p);
          col = second ? l + W - p : l;
        }
        if (!valid) { row = 64 * c; col = 0; }
        const int jj = 64 * c + col;
        const int rmn = s_rmin[((c ? R0 : 0) + row) * 64 + col];  // 255 outside the stage's range
        // the row must be able to end s-1 stages: i >= s-1, and some (s-1)-stage plan covers blocks 1..i
        const bool act = valid && rmn <= rl && row >= s - 1 && row >= s_wlo[c] && prev[row * LS + D - 1] != INF;
        if (__ballot(act) == 0ull) continue;
        const VT tij = (VT)(sT[min(jj + 1, N)] - sT[row]);
        // Narrower merge at late levels.  The first s-2 entries of a[] are INF (s-1 stages need s-1
        // devices) and only rl = D-s+1 replica counts and device totals are left, so the merge of
        // a[sig..sig+H-1] with c[1..H] on a network of H >= rl inputs gives every value the level
        // needs: its t-th output is W[d] for d - 1 = t + 1 + sig (the sig skipped entries are the
        // sig largest of the full merge).  sig <= s-2 skips only INF, sig <= DP-H stays inside the row.
#define RANNC_ROW(HH)                                                                                \
  {                                                                                                  \
    constexpr int H = (HH) <= DP ? (HH) : DP;                                                        \
    const int sig = H < DP ? min(s - 2, DP - H) : 0;                                                 \
    VT x[H];                                                                                         \
    row_merge_direct<VT, H, (H >= 8 ? H / 8 : 1), const VT *>(x, prev + row * LS + sig, tij, act ? rmn : 255, kc); \
    if (act && jj + 1 >= s) {                                                                        \
      /* no test per entry: columns D.. hold 0 and keep it, column DP (t + 1 + sig <= DP) is padding */ \
      VT *dst = cur + (jj + 1) * LS + 1 + sig;                                                       \
      _Pragma("unroll") for (int t = 0; t < H; ++t) atomicMin(&dst[t], x[t]);                        \
    }                                                                                                \
  }
        if (rl <= 8) RANNC_ROW(8)
        else if (rl <= 16) RANNC_ROW(16)
        else RANNC_ROW(32)
#undef RANNC_ROW
      }
    } else {
      for (int f = wave; f < RT; f += kSmallWaves) {
        const int c = f >= R0, i = c ? f - R0 : f;
        if (i < s - 1 || i < s_wlo[c] || 64 * c + 64 < s) continue;
        if (prev[i * LS + D - 1] == INF) continue;  // no (s-1)-stage plan covers blocks 1..i
        const int jj = 64 * c + lane;
        VT x[DP];
        const int64_t u = unit_index(nch, i, c);
        int rmn = 255;
        if (jj >= i && jj < N) rmn = rmin[u * 64 + lane];
        const bool act = rmn <= rl;
        if (__ballot(act) == 0ull) continue;
        const int col = act ? lane : __ffsll((long long)__ballot(act)) - 1;
        const VT RANNC_GLOBAL *unit = cost + u * 64 * D + col;
        const VT *arow = prev + i * LS;
        const VT off = act ? (VT)0 : INF;
#define RANNC_ROW(K)                                                                   \
  case K:                                                                              \
    if constexpr (8 * K <= DP) row_merge<VT, DP, K, const VT *>(x, unit, arow, off, rl); \
    break;
        switch ((rl + 7) >> 3) {
          RANNC_ROW(1) RANNC_ROW(2) RANNC_ROW(3) RANNC_ROW(4)
          RANNC_ROW(5) RANNC_ROW(6) RANNC_ROW(7) RANNC_ROW(8)
          default: break;
        }
#undef RANNC_ROW
        if (act && jj + 1 >= s) {
          // unconditional: folding INF in is a no-op and costs less than testing for it
#pragma unroll
          for (int t = 0; t < DP - 1; ++t)
            if (t + 1 <= D - 1) atomicMin(&cur[(jj + 1) * LS + t + 1], x[t]);
        }
      }
    }
    if constexpr (DIRECT) {
      // The next level's buffer held level s-2: its last readers were the passes of level s-1, which
      // the barrier before this level's passes closed, and its copy to memory was issued by these
      // same threads before their passes of level s-1.
      if (s < S_eff) {
        VT *next = lv[s % kLevelBufs];
        for (int e = tid; e < (N + 1) * LS; e += NT) next[e] = ((e % LS) < D) ? INF : (VT)0;
      }
    }
    lds_barrier();
    VT RANNC_GLOBAL *Vs = Vg + (int64_t)(s - 1) * lvl;
    for (int e = tid; e < (N + 1) * DP; e += NT) Vs[e] = cur[(e / DP) * LS + (e % DP)];
    if (tid == 0) s_top[s - 1] = cur[N * LS + D - 1];
  }
  __syncthreads();

  // ---- choice of the stage count (as select_kernel) ----
  if (wave == 0) {
    int64_t v = INT64_MAX;
    if (st == 0 && lane < S_eff) {
      const VT u = s_top[lane];
      v = (u == INF) ? INT64_MAX : (int64_t)u;
    }
    select_finish(pr, v, st, d_opt, d_n_stages, d_est, d_status);
  }
}

// ---------------------------------------------------------------------------------------
// DP level s >= 2, literal form: one thread per cell (j, d) scans every split point i
// (ascending) and every device count d' of the earlier stages (ascending), skipping infeasible
// predecessors and stages that do not fit, and keeps the first strict minimum -- the loops of
// Algorithm 1 as written.  Used as the reference level kernel (RANNC_DP_ALGO_SCAN) and to
// produce the (i, d') tables for export.  With write_v = 0 the value table is left alone and
// only the argmin arrays (canonical [(L+1)][N+1][D+1] layout of one problem) are written.
// ---------------------------------------------------------------------------------------
template <typename VT>
__global__ __launch_bounds__(64) void level_scan_kernel(const ProblemDev *__restrict__ probs, const int s,
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
  const VT *__restrict__ Vprev = (const VT *)pr.V + (int64_t)(s - 2) * lvl;
  const VT *__restrict__ cost = (const VT *)pr.cost;
  VT best = INF;
  int bi = -1, bd = -1;
  const int i_end = min(64 * c + 63, N - 1);
  for (int i = s - 1; i <= i_end; ++i) {
    const bool act = (jj >= i) && (jj < N);
    const int64_t u = unit_index(nch, i, c);
    const VT *__restrict__ unit = cost + u * 64 * D + lane;
    const int rmn = act ? (int)pr.rmin[u * 64 + lane] : 255;
    for (int dp = s - 1; dp <= d - 1; ++dp) {
      const VT a = Vprev[(int64_t)i * DP + dp - 1];
      if (a == INF) continue;  // earlier stages infeasible
      if (d - dp < rmn) continue;  // does not fit device memory
      const VT h = unit[(d - dp - 1) * 64];
      const VT v = vmax(a, h);
      if (v < best) { best = v; bi = i; bd = dp; }
    }
  }
  if (jj >= N || j < s) return;
  if (write_v) ((VT *)pr.V)[(int64_t)(s - 1) * lvl + (int64_t)j * DP + d - 1] = best;
  const int64_t e = ((int64_t)s * (N + 1) + j) * (D + 1) + d;
  if (arg_i) arg_i[e] = bi;
  if (arg_d) arg_d[e] = bd;
}

// Plan recovery for the split objective: the candidate kept by a cell is the first one, in scan
// order, whose sum equals the cell's value.  All threads of the workgroup evaluate the candidates
// of one cell, numbered in scan order, and the smallest matching number wins.
template <typename VT>
__device__ void traceback_split_body(const ProblemDev &pr, int plan_stride, int32_t *se, int32_t *rp,
                                     unsigned int *best_key, int forced) {
  constexpr VT INF = Lim<VT>::inf;
  const int N = pr.N, D = pr.D, DP = pr.DP, nch = pr.nch;
  const int tid = threadIdx.x;
  const int64_t lvl = (int64_t)(N + 1) * DP;
  const VT *V = (const VT *)pr.V, *VF = (const VT *)pr.VF, *VB = (const VT *)pr.VB;
  const VT *costf = (const VT *)pr.cost, *costb = (const VT *)pr.costb;
  int ns = (*pr.status == 0 && forced >= 0) ? (int)pr.res[1] : 0;  // forced < 0: no plan wanted
  if (forced > 0 && *pr.status == 0)
    ns = (forced <= pr.S_eff && V[(int64_t)(forced - 1) * lvl + (int64_t)N * DP + D - 1] != INF) ? forced : 0;
  for (int u = ns + tid; u < plan_stride; u += blockDim.x) { se[u] = -1; rp[u] = -1; }
  if (ns == 0) return;
  int j = N, d = D;
  for (int s = ns; s >= 2; --s) {
    if (tid == 0) *best_key = 0xFFFFFFFFu;
    __syncthreads();
    const VT v = V[(int64_t)(s - 1) * lvl + (int64_t)j * DP + d - 1];
    const int jj = j - 1, c = jj >> 6;
    const int nd = d - (s - 1);                       // d' = s-1 .. d-1
    const int total = (j - (s - 1)) * nd;             // i = s-1 .. j-1
    unsigned mine = 0xFFFFFFFFu;
    for (int e = tid; e < total && mine == 0xFFFFFFFFu; e += blockDim.x) {
      const int i = s - 1 + e / nd, dp = s - 1 + e % nd;
      const int64_t pc = (int64_t)(s - 2) * lvl + (int64_t)i * DP + dp - 1;
      if (V[pc] == INF) continue;
      const int64_t u = unit_index(nch, i, c);
      const int r = d - dp;
      if (r < (int)pr.rmin[u * 64 + (jj & 63)]) continue;
      const int64_t te = (u * D + (r - 1)) * 64 + (jj & 63);
      const VT f = vmax(VF[pc], costf[te]), b = vmax(VB[pc], costb[te]);
      if ((VT)(f + b) == v) mine = ((unsigned)i << 8) | (unsigned)dp;  // (i, d') ascends with e
    }
    if (mine != 0xFFFFFFFFu) atomicMin(best_key, mine);
    __syncthreads();
    const unsigned key = *best_key;
    __syncthreads();
    if (key == 0xFFFFFFFFu) {  // tables inconsistent: report no plan rather than walk on
      for (int u = tid; u < plan_stride; u += blockDim.x) { se[u] = -1; rp[u] = -1; }
      return;
    }
    const int i_sel = (int)(key >> 8), d_sel = (int)(key & 255u);
    if (tid == 0) { se[s - 1] = j; rp[s - 1] = d - d_sel; }
    j = i_sel;
    d = d_sel;
  }
  if (tid == 0) { se[0] = j; rp[0] = d; }
}

// ---------------------------------------------------------------------------------------
// Final choice of the stage count: opt = min over s of V[s][N][D], smallest s among equals.
// One wave per problem, lane s-1 reads V[s][N][D] (S_eff <= D <= 64).
// ---------------------------------------------------------------------------------------
// one wave: lane s-1 brings V[s][N][D] (INT64_MAX beyond S_eff or if the status is bad)
__device__ __forceinline__ void select_finish(const ProblemDev &pr, int64_t v, int st, int64_t *d_opt,
                                              int32_t *d_n_stages, int64_t *d_est, int32_t *d_status) {
  const int lane = threadIdx.x & 63;
  const int q = pr.q;
  // lexicographic minimum of (value, s): fewest stages among equal values
  int bs = lane + 1;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const int64_t ov = __shfl_xor(v, o);
    const int os = __shfl_xor(bs, o);
    if (ov < v || (ov == v && os < bs)) { v = ov; bs = os; }
  }
  if (lane != 0) return;
  const int64_t best = v;
  if (best == INT64_MAX) bs = 0;
  pr.res[0] = best;
  pr.res[1] = bs;
  d_opt[q] = best;
  d_n_stages[q] = bs;
  if (d_est) {
    int64_t e = INT64_MAX;
    if (bs > 0) {
      const int64_t f = (int64_t)pr.MB + bs - 1;
      e = (best != 0 && f > INT64_MAX / best) ? INT64_MAX : f * best;
    }
    d_est[q] = e;
  }
  if (d_status) d_status[q] = st;
}

__global__ __launch_bounds__(64) void select_kernel(const ProblemDev *__restrict__ probs,
                                                    int64_t *d_opt, int32_t *d_n_stages,
                                                    int64_t *d_est, int32_t *d_status) {
  const ProblemDev &pr = probs[blockIdx.x];
  const int lane = threadIdx.x;
  const int st = *pr.status;
  int64_t v = INT64_MAX;
  if (st == 0 && lane < pr.S_eff) {
    const int64_t lvl = (int64_t)(pr.N + 1) * pr.DP;
    const int64_t cell = (int64_t)pr.N * pr.DP + pr.D - 1;
    if (pr.bits == 32) {
      const uint32_t u = ((const uint32_t *)pr.V)[lane * lvl + cell];
      v = (u == Lim<uint32_t>::inf) ? INT64_MAX : (int64_t)u;
    } else {
      const uint64_t u = ((const uint64_t *)pr.V)[lane * lvl + cell];
      v = (u == Lim<uint64_t>::inf) ? INT64_MAX : (int64_t)u;
    }
  }
  select_finish(pr, v, st, d_opt, d_n_stages, d_est, d_status);
}

// ---------------------------------------------------------------------------------------
// Plan recovery (Algorithm 1's return value: the stage boundaries and replica counts behind the
// optimal table value).
// One workgroup per problem walks from (s*, N, D) down to level 1.  At each cell it finds the
// lexicographically smallest (i, d') with max(V[s-1][i][d'], h(i,j,d-d')) equal to the cell's
// value: the candidate that the ascending scan with strict "<" of Algorithm 1 would have kept.
// A wave owns a split point i and reads the row V[s-1][i][.] with one coalesced request (lane =
// d'-1).  Both that row and h(i,j,.) are non-increasing (the property the merge kernel rests on),
// so in row i the only candidate is the smallest d' whose earlier-stages value is <= the cell's
// value: one row read and one comparison of the stage's time per split point, and the reads of one
// pass (192 rows) do not depend on each other.
// ---------------------------------------------------------------------------------------
// Whether max(a, h) == v for the stage time h = ceil(x/r) + ceil(C/r) of Sec. III-C, given a <= v.
// The stage's time comes from the prefix sums (the table may not have been built); x is compared
// with multiples of r instead of being divided by it (a 64-bit division costs far more than the
// rest of a pass).  C is the same for every lane, so its branch does not diverge.
__device__ __forceinline__ bool stage_time_completes(uint64_t x, uint64_t C, int r, uint64_t a, uint64_t v) {
  uint64_t w = v;  // what ceil(x/r) may reach at most, and has to reach when a < v
  if (C) {
    const uint64_t hc = (C + (uint64_t)(r - 1)) / (uint64_t)r;
    if (hc > v) return false;
    w = v - hc;
  }
  // ceil(x/r) <= w  <=>  x <= w r
  if (__umul64hi(w, (uint64_t)r) == 0 && x > w * (uint64_t)r) return false;
  if (a == v || w == 0) return true;
  // ceil(x/r) >= w  <=>  x > (w-1) r
  return __umul64hi(w - 1, (uint64_t)r) == 0 && x > (w - 1) * (uint64_t)r;
}

// STAGED: everything the walk reads (the levels of V below the plan's, T, C, the window bounds, the
// fits-in-memory bytes) is first copied into the workgroup's LDS with one round of independent reads,
// and the walk then runs out of LDS.  For a search that small the walk is otherwise a chain of one
// memory round trip per stage out of a cold cache (about 1 us each).  lds: traceback_lds_bytes() bytes.
template <typename VT, int DP, bool STAGED>
__device__ void traceback_body(const ProblemDev &pr, int plan_stride, int32_t *se, int32_t *rp,
                               unsigned int *best_key, int forced, char *lds) {
  constexpr VT INF = Lim<VT>::inf;
  constexpr int KB = 12;  // rows per wave and pass; their reads are independent
  const int N = pr.N, D = pr.D, nch = pr.nch;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = blockDim.x >> 6;
  const int64_t lvl = (int64_t)(N + 1) * DP;
  const VT RANNC_GLOBAL *Vg = gptr((const VT *)pr.V);
  // forced > 0: the plan of exactly `forced` stages (Algorithm 1's own answer V[S][|B|][D]), if
  // that level holds one; forced = 0: the best level chosen by the solve; forced < 0: no plan wanted
  int ns = (*pr.status == 0 && forced >= 0) ? (int)pr.res[1] : 0;
  if (forced > 0 && *pr.status == 0)
    ns = (forced <= pr.S_eff && Vg[(int64_t)(forced - 1) * lvl + (int64_t)N * DP + D - 1] != INF) ? forced : 0;
  for (int u = ns + tid; u < plan_stride; u += blockDim.x) { se[u] = -1; rp[u] = -1; }
  if (ns == 0) return;
  using VP = std::conditional_t<STAGED, const VT *, const VT RANNC_GLOBAL *>;
  using TP = std::conditional_t<STAGED, const int64_t *, const int64_t RANNC_GLOBAL *>;
  using RP = std::conditional_t<STAGED, const uint8_t *, const uint8_t RANNC_GLOBAL *>;
  using WP = std::conditional_t<STAGED, const int32_t *, const int32_t RANNC_GLOBAL *>;
  VP V;
  TP T, C = nullptr;
  RP rmin;
  WP wlo;
  if constexpr (STAGED) {
    const int64_t nT = (((int64_t)(N + 1) * 8 + 31) / 32) * 32;
    char *w = lds;
    VT *Vl = (VT *)w; w += (int64_t)pr.S_eff * lvl * (int64_t)sizeof(VT);  // room for every level
    int64_t *Tl = (int64_t *)w; w += nT;
    int64_t *Cl = (int64_t *)w; w += nT;
    int32_t *Wl = (int32_t *)w; w += (((int64_t)nch * 4 + 31) / 32) * 32;
    uint8_t *Rl = (uint8_t *)w;
    // 16-byte copies (every array starts on a 256-byte boundary of the workspace; a level of V is
    // a multiple of 32 bytes)
    typedef uint32_t Quad __attribute__((ext_vector_type(4)));
    const Quad RANNC_GLOBAL *src = (const Quad RANNC_GLOBAL *)Vg;
    // eight reads in flight per lane (index clamped instead of tested, so that no branch separates them)
    const int64_t nquad = (int64_t)ns * lvl * (int64_t)sizeof(VT) / 16;
    for (int64_t e0 = tid; e0 < nquad; e0 += 8 * (int64_t)blockDim.x) {
      Quad r[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = src[min(e0 + k * (int64_t)blockDim.x, nquad - 1)];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (e0 + k * (int64_t)blockDim.x < nquad) ((Quad *)Vl)[e0 + k * (int64_t)blockDim.x] = r[k];
    }
    for (int e = tid; e <= N; e += blockDim.x) {
      Tl[e] = pr.T[e];
      if (pr.C) Cl[e] = pr.C[e];
    }
    for (int e = tid; e < nch; e += blockDim.x) Wl[e] = pr.wlo[e];
    const Quad RANNC_GLOBAL *rsrc = (const Quad RANNC_GLOBAL *)gptr((const uint8_t *)pr.rmin);
    for (int64_t e = tid; e < units_before(nch, N) * 4; e += blockDim.x) ((Quad *)Rl)[e] = rsrc[e];
    __syncthreads();
    V = Vl; T = Tl; rmin = Rl; wlo = Wl;
    if (pr.C) C = Cl;
  } else {
    V = Vg;
    T = gptr((const int64_t *)pr.T);
    rmin = gptr((const uint8_t *)pr.rmin);
    wlo = gptr((const int32_t *)pr.wlo);
    if (pr.C) C = gptr((const int64_t *)pr.C);
  }
  int j = N, d = D;
  for (int s = ns; s >= 2; --s) {
    VP Vp = V + (int64_t)(s - 2) * lvl;
    const int jj = j - 1, c = jj >> 6;
    const int64_t Tj = T[j];
    const uint64_t Cj = C ? (uint64_t)C[j] : 0ull;  // send time of the cut after block j (0 for j = N)
    if (tid == 0) *best_key = 0xFFFFFFFFu;
    lds_barrier();  // the waves meet through LDS only: the reads above and the plan stores stay in flight
    // the cell's value, the window bound and the first pass of rows are read together
    const VT v = V[(int64_t)(s - 1) * lvl + (int64_t)j * DP + d - 1];
    const int first = max(s - 1, min(wlo[c], j));  // earlier rows hold no stage that fits
    unsigned mine = 0xFFFFFFFFu;
    for (int top = j - 1; top >= s - 1; top -= nw * KB) {  // rows top, top-1, ... downwards
      VT a[KB];
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        const int i = top - (wave + nw * k);
        a[k] = (i >= s - 1 && lane < DP) ? Vp[(int64_t)i * DP + lane] : INF;  // lane = d'-1
      }
      // the row lane < KB is responsible for: its fits-in-memory byte and prefix sum are read in the
      // same round trip as the rows (their addresses depend on nothing that is loaded; a row
      // outside the range is clamped into it and ignored below)
      const int i = top - (wave + nw * lane);
      const int ic = min(max(i, s - 1), j - 1);
      int rmn = 0;
      int64_t Ti = 0;
      if (lane < KB) {  // the other lanes would only fetch lines nobody needs
        rmn = (int)rmin[unit_index(nch, ic, c) * 64 + (jj & 63)];
        Ti = T[ic];
      }
      // per row: smallest d' in [s-1, d-1] with a[d'] <= v (smaller d' cannot match, and if this
      // one does not match no larger one does: c only grows as r = d - d' shrinks); lane k then
      // checks row k against the stage time
      int my_d = 0;
      VT my_a = INF;
      // rows of this wave inside the window (they descend with k): the others cost nothing
      const int low = max(first, s - 1);
      const int kb = top - wave >= low ? (top - wave - low) / nw + 1 : 0;
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        // out of memory a test, not an exit: behind an exit the compiler moves each row's read to
        // its use, and the reads of a pass no longer overlap; out of LDS the exit is what is cheaper
        if constexpr (STAGED) {
          if (k >= kb) break;
        }
        const bool ok = k < kb && lane + 1 >= s - 1 && lane + 1 <= d - 1 && a[k] <= v;
        const unsigned long long m = __ballot(ok);
        if (m != 0ull) {
          const int q = __ffsll((long long)m) - 1;
          const VT aq = lane_bcast(a[k], q);
          if (lane == k) { my_d = q + 1; my_a = aq; }
        }
      }
      if (lane < KB && my_d != 0 && i >= first && v != INF) {
        const int r = d - my_d;
        if (r >= rmn && stage_time_completes((uint64_t)(Tj - Ti), Cj, r, (uint64_t)my_a, (uint64_t)v))
          mine = min(mine, ((unsigned)i << 8) | (unsigned)my_d);
      }
      if (top - nw * KB < first) break;  // the remaining rows lie below the window
    }
    if (mine != 0xFFFFFFFFu) atomicMin(best_key, mine);
    lds_barrier();
    const unsigned key = *best_key;
    lds_barrier();
    if (key == 0xFFFFFFFFu) {  // tables inconsistent: report no plan rather than walk on
      for (int u = tid; u < plan_stride; u += blockDim.x) { se[u] = -1; rp[u] = -1; }
      return;
    }
    const int i_sel = (int)(key >> 8), d_sel = (int)(key & 255u);
    if (tid == 0) { se[s - 1] = j; rp[s - 1] = d - d_sel; }
    j = i_sel;
    d = d_sel;
  }
  if (tid == 0) { se[0] = j; rp[0] = d; }
}

constexpr int kTracebackThreads = 1024;

// The plan of the one search the outer driver chose (the only one whose entry of the level array is
// not negative), copied behind its result record.  The record may live in host memory: it is only
// written here.
__device__ __forceinline__ void plan_to_record(int plan_stride, const int32_t *se, const int32_t *rp, int64_t *rec) {
  __syncthreads();  // the walk's stores, by this workgroup's first thread, are visible to all of it
  int32_t *plan = (int32_t *)(rec + 6);
  for (int u = threadIdx.x; u < plan_stride; u += blockDim.x) {
    plan[u] = se[u];
    plan[plan_stride + u] = rp[u];
  }
}

__global__ __launch_bounds__(kTracebackThreads) void traceback_kernel(
    const ProblemDev *__restrict__ probs, int plan_stride, int32_t *d_stage_end, int32_t *d_replicas,
    const int32_t *__restrict__ d_levels, int64_t *rec) {
  __shared__ unsigned int best_key;
  const ProblemDev pr = probs[blockIdx.x];  // by value: no reloads after the plan stores
  const int forced = d_levels ? d_levels[pr.q] : 0;
  int32_t *se = d_stage_end + (int64_t)pr.q * plan_stride;
  int32_t *rp = d_replicas + (int64_t)pr.q * plan_stride;
#define GO(T)                                                                                    \
  switch (pr.DP) {                                                                               \
    case 8: traceback_body<T, 8, false>(pr, plan_stride, se, rp, &best_key, forced, nullptr); break;   \
    case 16: traceback_body<T, 16, false>(pr, plan_stride, se, rp, &best_key, forced, nullptr); break; \
    case 32: traceback_body<T, 32, false>(pr, plan_stride, se, rp, &best_key, forced, nullptr); break; \
    default: traceback_body<T, 64, false>(pr, plan_stride, se, rp, &best_key, forced, nullptr); break; \
  }
  if (pr.VF) {  // split objective: first-match over all candidates
    if (pr.bits == 32) traceback_split_body<uint32_t>(pr, plan_stride, se, rp, &best_key, forced);
    else traceback_split_body<uint64_t>(pr, plan_stride, se, rp, &best_key, forced);
  } else if (pr.bits == 32) { GO(uint32_t) } else { GO(uint64_t) }
#undef GO
  if (rec && d_levels && forced >= 0) plan_to_record(plan_stride, se, rp, rec);
}

// Plan recovery out of LDS, for launches of few, small min-max searches (the host checks that every
// search of the launch fits traceback_lds_bytes() into the dynamic LDS it passes).
__global__ __launch_bounds__(kTracebackThreads) void traceback_lds_kernel(
    const ProblemDev *__restrict__ probs, int plan_stride, int32_t *d_stage_end, int32_t *d_replicas,
    const int32_t *__restrict__ d_levels, int64_t *rec) {
  __shared__ unsigned int best_key;
  extern __shared__ __align__(16) char staged[];
  const ProblemDev pr = probs[blockIdx.x];
  const int forced = d_levels ? d_levels[pr.q] : 0;
  int32_t *se = d_stage_end + (int64_t)pr.q * plan_stride;
  int32_t *rp = d_replicas + (int64_t)pr.q * plan_stride;
#define GO(T)                                                                                   \
  switch (pr.DP) {                                                                              \
    case 8: traceback_body<T, 8, true>(pr, plan_stride, se, rp, &best_key, forced, staged); break;    \
    case 16: traceback_body<T, 16, true>(pr, plan_stride, se, rp, &best_key, forced, staged); break;  \
    case 32: traceback_body<T, 32, true>(pr, plan_stride, se, rp, &best_key, forced, staged); break;  \
    default: traceback_body<T, 64, true>(pr, plan_stride, se, rp, &best_key, forced, staged); break;  \
  }
  if (pr.bits == 32) { GO(uint32_t) } else { GO(uint64_t) }
#undef GO
  if (rec && d_levels && forced >= 0) plan_to_record(plan_stride, se, rp, rec);
}

// ---------------------------------------------------------------------------------------
// Table export in the layout-independent form of the public header (parity and inspection).
// ---------------------------------------------------------------------------------------
template <typename VT>
__global__ __launch_bounds__(256) void export_kernel(const ProblemDev *__restrict__ prob, int which,
                                                     void *__restrict__ dst) {
  const ProblemDev &pr = *prob;
  const int N = pr.N, D = pr.D, DP = pr.DP, nch = pr.nch;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  constexpr VT INF = Lim<VT>::inf;
  const bool bad = *pr.status != 0;
  if (which == RANNC_DP_TABLE_COST || which == RANNC_DP_TABLE_FIT || which == RANNC_DP_TABLE_COST_BWD) {
    const VT *ctab = (const VT *)(which == RANNC_DP_TABLE_COST_BWD ? pr.costb : pr.cost);
    const int64_t total = (int64_t)N * (N + 1) / 2 * D;
    for (int64_t e = t0; e < total; e += stride) {
      const int r = (int)(e % D) + 1;
      const int64_t pair = e / D;  // j(j-1)/2 + i
      int j = (int)((1.0 + sqrt(1.0 + 8.0 * (double)pair)) * 0.5);
      while ((int64_t)j * (j - 1) / 2 > pair) --j;
      while ((int64_t)(j + 1) * j / 2 <= pair) ++j;
      const int i = (int)(pair - (int64_t)j * (j - 1) / 2);
      const int jj = j - 1;
      const int64_t u = unit_index(nch, i, jj >> 6);
      if (which == RANNC_DP_TABLE_FIT) {
        ((uint8_t *)dst)[e] = bad ? 0 : (uint8_t)(r >= (int)pr.rmin[u * 64 + (jj & 63)]);
      } else {
        const bool fit = !bad && r >= (int)pr.rmin[u * 64 + (jj & 63)];
        const VT v = fit ? ctab[(u * D + (r - 1)) * 64 + (jj & 63)] : INF;
        ((int64_t *)dst)[e] = (v == INF) ? INT64_MAX : (int64_t)v;
      }
    }
  } else if (which == RANNC_DP_TABLE_V || which == RANNC_DP_TABLE_MAX_FWD || which == RANNC_DP_TABLE_MAX_BWD) {
    const VT *vtab = (const VT *)(which == RANNC_DP_TABLE_V ? pr.V : which == RANNC_DP_TABLE_MAX_FWD ? pr.VF : pr.VB);
    const int64_t per = (int64_t)(N + 1) * (D + 1);
    const int64_t total = (int64_t)(pr.S_eff + 1) * per;
    const int64_t lvl = (int64_t)(N + 1) * DP;
    for (int64_t e = t0; e < total; e += stride) {
      const int s = (int)(e / per);
      const int j = (int)((e % per) / (D + 1));
      const int d = (int)(e % (D + 1));
      int64_t v = INT64_MAX;
      if (s == 0) v = (j == 0 && d == 0) ? 0 : INT64_MAX;
      else if (d >= 1 && !bad) {
        const VT u = vtab[(int64_t)(s - 1) * lvl + (int64_t)j * DP + d - 1];
        v = (u == INF) ? INT64_MAX : (int64_t)u;
      }
      ((int64_t *)dst)[e] = v;
    }
  }
}

// argmin export helpers: whole table to -1, then level 1 (the single stage 1..j on d devices
// has predecessor (0,0)); levels >= 2 come from level_scan_kernel.
template <typename VT>
__global__ __launch_bounds__(256) void arg_init_kernel(const ProblemDev *__restrict__ prob,
                                                       int32_t *__restrict__ arg) {
  const ProblemDev &pr = *prob;
  const int N = pr.N, D = pr.D, DP = pr.DP;
  const int64_t per = (int64_t)(N + 1) * (D + 1);
  const int64_t total = (int64_t)(pr.S_eff + 1) * per;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const bool bad = *pr.status != 0;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
    const int s = (int)(e / per);
    const int j = (int)((e % per) / (D + 1));
    const int d = (int)(e % (D + 1));
    int32_t v = -1;
    if (s == 1 && j >= 1 && d >= 1 && !bad) {
      if (((const VT *)pr.V)[(int64_t)j * DP + d - 1] != Lim<VT>::inf) v = 0;
    }
    arg[e] = v;
  }
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
hipError_t launch_prefix(const ProblemDev *probs, int Q, hipStream_t st) {
  hipLaunchKernelGGL(prefix_kernel, dim3(Q), dim3(256), 0, st, probs);
  return hipGetLastError();
}

hipError_t launch_fill(const ProblemDev *probs, int Q, hipStream_t st) {
  const int per = Q >= 256 ? 4 : Q >= 16 ? 32 : 256;
  for (int q0 = 0; q0 < Q; q0 += 65535) {
    const int nq = min(65535, Q - q0);
    hipLaunchKernelGGL(fill_kernel, dim3(per, nq), dim3(256), 0, st, probs + q0);
  }
  return hipGetLastError();
}

int merge_rows_per_item(int rows_per_wave) {
  if (rows_per_wave <= 0) return -1;  // chosen on the device
  return kMergeWaves * (rows_per_wave <= 1 ? 1 : rows_per_wave <= 2 ? 2 : rows_per_wave <= 4 ? 4 : rows_per_wave <= 8 ? 8 : rows_per_wave <= 12 ? 12 : 16);
}

// Grid of the sorted-merge level kernel = items of the largest search of the launch if nothing is
// pruned.  rows_per_item > 0: in items of that size.  Otherwise in the size that suits the launch
// as a whole: 4-row items (most workgroups) while that leaves the device short of work, larger ones
// (fewer folds and atomics per row) when the launch is full anyway.  The work list then takes the
// smallest item size that fits this grid.
int64_t merge_launch_rows(const LaunchShape &sh) {
  int64_t all_rows = 0;
  for (int c = 0; c < sh.max_nch; ++c) all_rows += min(64 * c + 64, sh.max_N);
  return all_rows * sh.nprob;
}

int merge_grid_items(const LaunchShape &sh, int rows_per_item, int slots, bool paired, int *rows_for_list) {
  // items of the largest search of the launch if nothing is pruned, in items of `rows` rows: the
  // segments of run_segments for windows that start at row 0 (a pruned window has no more rows in
  // either segment, so no more items at any size)
  auto items_at = [&](int rows) {
    int64_t items = 0;
    for (int c = 0; c < sh.max_nch; ++c) {
      const int hi = min(64 * c + 63, sh.max_N - 1);
      int n0 = hi + 1, n1 = 0;
      if (paired && hi >= 64 * c) { n0 = 64 * c; n1 = min(32, hi - 64 * c) + 1; }
      items += (n0 + rows - 1) / rows + (n1 + rows - 1) / rows;
    }
    return std::max<int64_t>(1, items);
  };
  int rows = rows_per_item;
  *rows_for_list = rows_per_item;
  if (rows <= 0) {
    const int64_t launch_rows = merge_launch_rows(sh);
    rows = launch_rows >= kMergeRows16From ? 16 : launch_rows >= kMergeRows8From ? 8 : kMergeMinRows;
    // A launch of the recomputing form over several searches with many rounds of workgroups: the
    // largest items that still leave three rounds if nothing is pruned, the same size for every
    // search of the launch.  Clearing the tile, the fold and the atomics are paid per item, and with
    // three rounds the partly filled last one costs little (config 5: 16 -> 64 rows, 157 -> 115 us
    // per level; the table form, bound by its reads, gains nothing: 100 -> 107 us at 32 devices).
    if (paired && sh.nprob > 1 && items_at(rows) * sh.nprob > slots)
      for (int r = 64; r > rows; r -= 4)
        if (items_at(r) * sh.nprob >= 3ll * slots) { rows = r; *rows_for_list = r; break; }
  }
  return (int)items_at(rows);
}

hipError_t launch_runs(const ProblemDev *probs, int Q, int rows_per_item, int max_items, int slots, bool paired,
                       hipStream_t st) {
  hipLaunchKernelGGL(runs_kernel, dim3(Q), dim3(256), 0, st, probs, rows_per_item, max_items, Q, slots, paired ? 1 : 0);
  return hipGetLastError();
}

// Workgroups of the sorted-merge level kernel that one compute unit holds at a time (by the
// registers of its four waves, one per SIMD; see the kernel's resource usage).
int merge_workgroups_per_cu(int bits, int DP, bool recompute) {
  if (bits == 32) {
    if (recompute) return DP == 64 ? 2 : DP == 32 ? 4 : DP == 16 ? 5 : 8;
    return DP == 64 ? 3 : DP == 32 ? 4 : DP == 16 ? 6 : 8;
  }
  return DP == 64 ? 2 : DP == 32 ? 3 : DP == 16 ? 4 : 8;
}

hipError_t launch_windows(const ProblemDev *probs, const LaunchShape &sh, hipStream_t st) {
  for (int q0 = 0; q0 < sh.nprob; q0 += 65535) {
    const int nq = min(65535, sh.nprob - q0);
    hipLaunchKernelGGL(windows_kernel, dim3(sh.max_nch, nq), dim3(256), 0, st, probs + q0);
  }
  return hipGetLastError();
}

constexpr int kBuildRowsFitOnly = 8;  // rows per wave when only the fits-in-memory part is built

template <typename VT, int DP>
static void build_go(const ProblemDev *p, const LaunchShape &sh, int parts, hipStream_t st) {
  const int rows = (parts & 2) ? 1 : kBuildRowsFitOnly;
  const int per_group = kBuildWaves * rows;
  for (int q0 = 0; q0 < sh.nprob; q0 += 65535) {
    const int nq = min(65535, sh.nprob - q0);
    const int groups = (sh.max_N + per_group - 1) / per_group, many = nq > 1;
    const dim3 grid = many ? dim3(nq, groups, sh.max_nch) : dim3(sh.max_nch, groups, 1), block(64 * kBuildWaves);
    if (rows == 1) hipLaunchKernelGGL((build_kernel<VT, DP, 1>), grid, block, 0, st, p + q0, parts, many);
    else hipLaunchKernelGGL((build_kernel<VT, DP, kBuildRowsFitOnly>), grid, block, 0, st, p + q0, parts, many);
  }
}

hipError_t launch_build(const ProblemDev *p, const LaunchShape &sh, int bits, int DP, int parts, hipStream_t st) {
  if (sh.max_N > 65535) return hipErrorInvalidValue;
#define GO(B, T)                                                   \
  if (bits == B) {                                                 \
    if (DP == 8) build_go<T, 8>(p, sh, parts, st);                 \
    else if (DP == 16) build_go<T, 16>(p, sh, parts, st);          \
    else if (DP == 32) build_go<T, 32>(p, sh, parts, st);          \
    else build_go<T, 64>(p, sh, parts, st);                        \
  }
  GO(32, uint32_t)
  GO(64, uint64_t)
#undef GO
  return hipGetLastError();
}

template <typename VT, int DP, bool DIRECT>
static void merge_go(const ProblemDev *p, const LaunchShape &sh, int s, int items, const ProblemDev *host_one,
                     hipStream_t st) {
  if (host_one && sh.nprob == 1) {
    hipLaunchKernelGGL((level_merge_one_kernel<VT, DP, DIRECT>), dim3((unsigned)items, 1, 1), dim3(64 * kMergeWaves), 0,
                       st, *host_one, s);
    return;
  }
  for (int q0 = 0; q0 < sh.nprob; q0 += 65535) {
    const int nq = min(65535, sh.nprob - q0);
    // (the table form keeps the items of a search together: workgroups that run at the same time
    // then read neighbouring units of few tables instead of one unit each of hundreds of tables,
    // which measured 10 % slower on config 5)
    if (DIRECT && nq > 1 && items <= 65535)
      hipLaunchKernelGGL((level_merge_kernel<VT, DP, DIRECT>), dim3(nq, 1, (unsigned)items), dim3(64 * kMergeWaves), 0,
                         st, p + q0, s, 0);
    else
      hipLaunchKernelGGL((level_merge_kernel<VT, DP, DIRECT>), dim3((unsigned)items, 1, nq), dim3(64 * kMergeWaves), 0,
                         st, p + q0, s, 1);
  }
}

hipError_t launch_level_merge(const ProblemDev *p, const LaunchShape &sh, int bits, int DP, int s, bool recompute,
                              int items, const ProblemDev *host_one, hipStream_t st) {
  if (recompute && bits != 32) return hipErrorInvalidValue;
#define GO(B, T, X)                                                            \
  if (bits == B && recompute == X) {                                           \
    if (DP == 8) merge_go<T, 8, X>(p, sh, s, items, host_one, st);               \
    else if (DP == 16) merge_go<T, 16, X>(p, sh, s, items, host_one, st);        \
    else if (DP == 32) merge_go<T, 32, X>(p, sh, s, items, host_one, st);        \
    else merge_go<T, 64, X>(p, sh, s, items, host_one, st);                      \
  }
  GO(32, uint32_t, false)
  GO(32, uint32_t, true)
  GO(64, uint64_t, false)
#undef GO
  return hipGetLastError();
}

int small_max_blocks() { return kSmallMaxN; }
// the one-launch kernel can recompute the stage times up to the 32-device class (beyond it the
// reciprocals and the merge do not fit the 128 registers of its sixteen waves): 32-bit values, or
// 64-bit values where the caller's bound on a search's total time keeps every stage time in the
// range the double-precision quotient is exact for
bool small_can_recompute(int bits, int DP, int64_t max_total_time) {
  return DP <= 32 && (bits == 32 || max_total_time <= kDirectWideMaxTime);
}

hipError_t launch_solve_small(const ProblemDev *p, int Q, int bits, int DP, bool direct, int64_t *d_opt,
                              int32_t *d_n_stages, int64_t *d_est, int32_t *d_status, hipStream_t st) {
  if (direct && DP > 32) return hipErrorInvalidValue;
#define GO(B, T, W, X)                                                                                 \
  if (bits == B && DP == W && direct == X)                                                             \
    hipLaunchKernelGGL((solve_small_kernel<T, W, X>), dim3(Q), dim3(64 * small_waves<T, W>()), 0, st, p, d_opt, \
                       d_n_stages, d_est, d_status);
  GO(32, uint32_t, 8, false) GO(32, uint32_t, 16, false) GO(32, uint32_t, 32, false) GO(32, uint32_t, 64, false)
  GO(64, uint64_t, 8, false) GO(64, uint64_t, 16, false) GO(64, uint64_t, 32, false) GO(64, uint64_t, 64, false)
  GO(32, uint32_t, 8, true) GO(32, uint32_t, 16, true) GO(32, uint32_t, 32, true)
  GO(64, uint64_t, 8, true) GO(64, uint64_t, 16, true) GO(64, uint64_t, 32, true)
#undef GO
  return hipGetLastError();
}

hipError_t launch_level_scan(const ProblemDev *p, const LaunchShape &sh, int bits, int s, int write_v,
                             int32_t *arg_i, int32_t *arg_d, hipStream_t st) {
  for (int q0 = 0; q0 < sh.nprob; q0 += 65535) {
    const int nq = min(65535, sh.nprob - q0);
    const dim3 grid(sh.max_nch, sh.max_D, nq);
    if (bits == 32)
      hipLaunchKernelGGL((level_scan_kernel<uint32_t>), grid, dim3(64), 0, st, p + q0, s, write_v, arg_i,
                         arg_d);
    else
      hipLaunchKernelGGL((level_scan_kernel<uint64_t>), grid, dim3(64), 0, st, p + q0, s, write_v, arg_i,
                         arg_d);
  }
  return hipGetLastError();
}

hipError_t launch_select(const ProblemDev *p, int Q, int64_t *d_opt, int32_t *d_n_stages,
                         int64_t *d_est, int32_t *d_status, hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(Q), dim3(64), 0, st, p, d_opt, d_n_stages, d_est, d_status);
  return hipGetLastError();
}

int64_t traceback_lds_bytes(int N, int DP, int S_eff, int bits) {
  const int nch = (N + 63) / 64;
  const int64_t nT = (((int64_t)(N + 1) * 8 + 31) / 32) * 32;
  return (int64_t)S_eff * (N + 1) * DP * (bits / 8) + 2 * nT + (((int64_t)nch * 4 + 31) / 32) * 32 +
         units_before(nch, N) * 64;
}

hipError_t launch_traceback(const ProblemDev *p, int Q, int plan_stride, int32_t *d_stage_end,
                            int32_t *d_replicas, const int32_t *d_levels, int64_t lds_bytes, int64_t *rec,
                            hipStream_t st) {
  if (lds_bytes > 0) {
    // more than the default 64 KiB of dynamic LDS has to be asked for once
    static const hipError_t attr = hipFuncSetAttribute((const void *)traceback_lds_kernel,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kTracebackLdsMax);
    if (attr != hipSuccess) return attr;
    if (lds_bytes > kTracebackLdsMax) return hipErrorInvalidValue;
    hipLaunchKernelGGL(traceback_lds_kernel, dim3(Q), dim3(kTracebackThreads), (size_t)lds_bytes, st, p, plan_stride,
                       d_stage_end, d_replicas, d_levels, rec);
  } else {
    hipLaunchKernelGGL(traceback_kernel, dim3(Q), dim3(kTracebackThreads), 0, st, p, plan_stride, d_stage_end,
                       d_replicas, d_levels, rec);
  }
  return hipGetLastError();
}

// V[s][N][D] for s = 1..S_eff of every problem (INT64_MAX: no plan of exactly s stages, or s
// beyond S_eff, or bad inputs): Algorithm 1's answer for each exact stage count.
__global__ __launch_bounds__(64) void level_values_kernel(const ProblemDev *__restrict__ probs, int stride,
                                                          int64_t *__restrict__ out) {
  const ProblemDev &pr = probs[blockIdx.x];
  const bool bad = *pr.status != 0;
  const int64_t lvl = (int64_t)(pr.N + 1) * pr.DP;
  const int64_t cell = (int64_t)pr.N * pr.DP + pr.D - 1;
  for (int k = threadIdx.x; k < stride; k += 64) {
    int64_t v = INT64_MAX;
    if (!bad && k < pr.S_eff) {
      if (pr.bits == 32) {
        const uint32_t u = ((const uint32_t *)pr.V)[k * lvl + cell];
        v = (u == Lim<uint32_t>::inf) ? INT64_MAX : (int64_t)u;
      } else {
        const uint64_t u = ((const uint64_t *)pr.V)[k * lvl + cell];
        v = (u == Lim<uint64_t>::inf) ? INT64_MAX : (int64_t)u;
      }
    }
    out[(int64_t)pr.q * stride + k] = v;
  }
}

hipError_t launch_level_values(const ProblemDev *p, int Q, int stride, int64_t *d_out, hipStream_t st) {
  hipLaunchKernelGGL(level_values_kernel, dim3(Q), dim3(64), 0, st, p, stride, d_out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Outer driver (Algorithm 2 "form_stage" of Sec. III-C), the loops over the solved batch: node
// counts n = 1, 2, 4, ... in turn, for each the stage counts S ascending over
// (devices_per_node*(n-1), devices_per_node*n], and for the first S that any search of that n can
// realise (V[S][N][D] finite), the search with the smallest (MB + S - 1) * V, the first one in
// batch order among equals.  That is the lexicographic minimum of (n, S, estimate, search index)
// over all feasible (search, S) pairs, S inside the range of the search's n: one wave, a lane per
// search (in rounds of 64) reads its values straight from the value tables (all reads of a lane
// are independent), then one reduction over the wave.
// Writes the record {q, S, first bad status in batch order or 0, 0, V, estimate}, the plan area
// behind it (-1 everywhere; the plan recovery fills in the chosen search's), and the level array
// of the plan recovery (S at the chosen search, -1 = no plan wanted elsewhere).  q = -1: infeasible.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void form_stage_select_kernel(
    const ProblemDev *__restrict__ probs, int Q, int stride, int N, int n_nodes, int devices_per_node,
    const int32_t *__restrict__ pair_n, const int32_t *__restrict__ pair_mb, int32_t *__restrict__ levels,
    int64_t *__restrict__ rec) {
  constexpr int NONE = 0x7fffffff;
  constexpr int kMaxRange = 64;  // devices_per_node <= RANNC_DP_MAX_DEVICES
  const int lane = threadIdx.x;
  int32_t *plan = (int32_t *)(rec + 6);
  for (int u = lane; u < 2 * stride; u += 64) plan[u] = -1;
  int bad_q = NONE, bad_st = 0;
  int best_k = NONE, best_q = NONE;  // k = n << 16 | S
  int64_t best_e = INT64_MAX, best_v = 0;
  for (int p = lane; p < Q; p += 64) {
    const ProblemDev &pr = probs[p];
    const int q = pr.q;
    levels[q] = -1;  // only the chosen search's plan is recovered
    const int st = *pr.status;
    if (st != 0) {
      if (q < bad_q) { bad_q = q; bad_st = st; }
      continue;
    }
    const int n = pair_n[q];
    const int64_t mb = pair_mb[q];
    const int lo = devices_per_node * (n - 1) + 1;
    const int hi = min(min(devices_per_node * n, N), pr.S_eff);
    const int64_t lvl = (int64_t)(pr.N + 1) * pr.DP, cell = (int64_t)pr.N * pr.DP + pr.D - 1;
    // the first S of the range that this search can realise (a smaller S always wins for one n)
    for (int S = lo; S <= hi && S < lo + kMaxRange; ++S) {
      int64_t v;
      if (pr.bits == 32) {
        const uint32_t u = ((const uint32_t *)pr.V)[(S - 1) * lvl + cell];
        v = (u == Lim<uint32_t>::inf) ? INT64_MAX : (int64_t)u;
      } else {
        const uint64_t u = ((const uint64_t *)pr.V)[(S - 1) * lvl + cell];
        v = (u == Lim<uint64_t>::inf) ? INT64_MAX : (int64_t)u;
      }
      if (v == INT64_MAX) continue;
      const int64_t f = mb + S - 1;
      const int64_t e = (v != 0 && f > INT64_MAX / v) ? INT64_MAX : f * v;
      const int k = n << 16 | S;
      if (k < best_k || (k == best_k && (e < best_e || (e == best_e && q < best_q)))) {
        best_k = k; best_e = e; best_v = v; best_q = q;
      }
      break;
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const int ok = __shfl_xor(best_k, o), oq = __shfl_xor(best_q, o);
    const int64_t oe = __shfl_xor(best_e, o), ov = __shfl_xor(best_v, o);
    if (ok < best_k || (ok == best_k && (oe < best_e || (oe == best_e && oq < best_q)))) {
      best_k = ok; best_e = oe; best_v = ov; best_q = oq;
    }
    const int obq = __shfl_xor(bad_q, o), obs = __shfl_xor(bad_st, o);
    if (obq < bad_q) { bad_q = obq; bad_st = obs; }
  }
  if (lane == 0) {
    const bool found = bad_q == NONE && best_q != NONE;
    if (found) levels[best_q] = best_k & 0xffff;
    rec[0] = found ? best_q : -1;
    rec[1] = found ? (best_k & 0xffff) : 0;
    rec[2] = bad_q == NONE ? 0 : bad_st;
    rec[3] = 0;
    rec[4] = found ? best_v : 0;
    rec[5] = found ? best_e : 0;
  }
}

hipError_t launch_form_stage_select(const ProblemDev *probs, int Q, int stride, int N, int n_nodes,
                                    int devices_per_node, const int32_t *pair_n, const int32_t *pair_mb,
                                    int32_t *levels, int64_t *rec, hipStream_t st) {
  hipLaunchKernelGGL(form_stage_select_kernel, dim3(1), dim3(64), 0, st, probs, Q, stride, N, n_nodes, devices_per_node,
                     pair_n, pair_mb, levels, rec);
  return hipGetLastError();
}

hipError_t launch_export(const ProblemDev *p, int which, int bits, void *d_dst, hipStream_t st) {
  const dim3 grid(1024), block(256);
  if (which != RANNC_DP_TABLE_ARG_I && which != RANNC_DP_TABLE_ARG_D) {
    if (bits == 32) hipLaunchKernelGGL((export_kernel<uint32_t>), grid, block, 0, st, p, which, d_dst);
    else hipLaunchKernelGGL((export_kernel<uint64_t>), grid, block, 0, st, p, which, d_dst);
  } else {
    if (bits == 32) hipLaunchKernelGGL((arg_init_kernel<uint32_t>), grid, block, 0, st, p, (int32_t *)d_dst);
    else hipLaunchKernelGGL((arg_init_kernel<uint64_t>), grid, block, 0, st, p, (int32_t *)d_dst);
  }
  return hipGetLastError();
}

}  // namespace rannc
