// Host orchestration behind the C ABI of include/rannc_dp.h: argument checks, workspace
// layout, and the sequence of kernel launches of one search (prefix sums and tables, one
// launch per DP level, final selection, plan recovery).  Nothing here computes any part of the
// recurrence; that is all in the kernel files (rannc_dp_kernels.hip, rannc_dp_split.hip, rannc_dp_compact.hip).
#include "../../include/rannc_dp.h"
#include "rannc_dp_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

using rannc::LaunchShape;
using rannc::ProblemDev;

namespace {

constexpr size_t kAlign = 256;
constexpr int64_t kNarrowMax = 4294967294LL;  // largest total time a 32-bit table can hold
constexpr int kStagingSlots = 2;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Sizes {  // bytes of one problem's regions inside the workspace
  size_t prefix, wlo, runs, ufit, misc, rmin, cost, V, keys;
  bool split;  // split objective: a fifth prefix array, a second stage-time table, two more value tables
  size_t total() const {
    return prefix * (split ? 5 : 4) + wlo + runs + ufit + misc + rmin + cost * (split ? 2 : 1) +
           V * (split ? 3 : 1) + keys;
  }
};

// false on arithmetic overflow
bool problem_sizes(int N, int D, int S_eff, int bits, bool split, bool packed, Sizes *o) {
  const int nch = (N + 63) / 64;
  const int DP = rannc::dp_class(D);
  const size_t esz = bits / 8;
  const unsigned __int128 rows = (unsigned __int128)rannc::units_before(nch, N) * 64;
  const unsigned __int128 cost = rows * (unsigned)D * esz;
  const unsigned __int128 V = (unsigned __int128)S_eff * (unsigned)(N + 1) * (unsigned)DP * esz;
  if (cost > ((unsigned __int128)1 << 46) || V > ((unsigned __int128)1 << 46)) return false;
  o->prefix = align_up((size_t)(N + 1) * 8);
  o->wlo = align_up((size_t)nch * 4);
  o->runs = align_up((size_t)(rannc::max_runs(nch) + 1) * 4);
  o->ufit = align_up((size_t)rannc::units_before(nch, N));
  o->misc = align_up(64);  // status word, result pair
  o->rmin = align_up((size_t)rows);
  o->cost = align_up((size_t)cost);
  o->V = align_up((size_t)V);
  o->split = split;
  o->keys = (split && packed) ? align_up((size_t)(N + 1) * (size_t)DP * 8) : 0;
  return true;
}

bool limits_ok(const rannc_dp_limits_t *l) {
  return l && l->max_problems >= 1 && l->max_blocks >= 1 && l->max_blocks <= 65535 &&
         l->max_devices >= 1 && l->max_devices <= RANNC_DP_MAX_DEVICES && l->max_stages >= 1 &&
         l->max_total_time_ns >= 0 && (l->flags & ~RANNC_DP_FLAG_SPLIT_OBJECTIVE) == 0 && l->algo >= RANNC_DP_ALGO_AUTO &&
         l->algo <= RANNC_DP_ALGO_RECOMPUTE && l->rows_per_wave >= 0 && l->rows_per_wave <= 16 &&
         l->one_launch_small >= 0 && l->one_launch_small <= 2 && l->single_stream >= 0 && l->single_stream <= 1 &&
         l->reserved == 0;
}

bool split_of(const rannc_dp_limits_t *l) { return (l->flags & RANNC_DP_FLAG_SPLIT_OBJECTIVE) != 0; }
// split objective: can the winners of a level be packed into 64-bit words (see the level kernel)
bool packed_of(const rannc_dp_limits_t *l) { return l->max_total_time_ns <= rannc::kSplitPackedMax; }
int bits_of(const rannc_dp_limits_t *l) { return l->max_total_time_ns <= kNarrowMax ? 32 : 64; }

size_t header_bytes(int Q) { return align_up((size_t)Q * sizeof(ProblemDev)); }

// Host-side validation of the batch descriptors against the limits.
int check_batch(const rannc_dp_limits_t *l, const rannc_dp_batch_t *b) {
  if (!b || b->n_problems < 1) return RANNC_DP_INVALID_ARG;
  if (!b->n_blocks || !b->n_devices || !b->max_stages || !b->n_microbatches || !b->mem_capacity ||
      !b->block_offset)
    return RANNC_DP_INVALID_ARG;
  if (b->n_problems > l->max_problems) return RANNC_DP_LIMIT_EXCEEDED;
  if (b->block_offset[0] < 0) return RANNC_DP_INVALID_ARG;
  if ((b->bandwidth_bytes_per_us == nullptr) != (b->cut_bytes == nullptr)) return RANNC_DP_INVALID_ARG;
  for (int q = 0; q < b->n_problems; ++q) {
    if (b->n_blocks[q] < 1 || b->n_devices[q] < 1 || b->max_stages[q] < 1 ||
        b->n_microbatches[q] < 1 || b->mem_capacity[q] < 0)
      return RANNC_DP_INVALID_ARG;
    if (b->bandwidth_bytes_per_us && b->bandwidth_bytes_per_us[q] < 1) return RANNC_DP_INVALID_ARG;
    if (b->block_offset[q + 1] - b->block_offset[q] != (int64_t)b->n_blocks[q])
      return RANNC_DP_INVALID_ARG;
    if (b->n_blocks[q] > l->max_blocks || b->n_devices[q] > l->max_devices ||
        std::min(b->max_stages[q], std::min(b->n_blocks[q], b->n_devices[q])) > l->max_stages)
      return RANNC_DP_LIMIT_EXCEEDED;
  }
  return RANNC_DP_OK;
}

}  // namespace

struct rannc_dp {
  rannc_dp_limits_t lim;
  int bits;
  char *ws;
  size_t ws_bytes;
  // pinned staging for the per-problem descriptors and problem lists, reused round-robin
  char *staging[kStagingSlots];
  hipEvent_t staging_free[kStagingSlots];
  bool staging_used[kStagingSlots];
  size_t staging_bytes;
  int next_slot;
  // state of the last successful solve
  bool solved;
  int Q;
  std::vector<ProblemDev> host_probs;  // in device order: grouped by DP class
  std::vector<int32_t> pos_of;         // position of the caller's problem q in that order
  ProblemDev *d_probs;
  // timing
  bool timing;
  hipEvent_t ev[4];
  bool ev_valid;
  int level_launches;
  // Device-count classes are independent chains of launches: with more than one class in a batch
  // the others run on streams of the handle (default priority), forked from and joined to the
  // caller's stream with events.  Off while per-phase timing is on (the phases are timed on the
  // caller's stream) and with RANNC_DP_STREAMS=0.
  char *fs_pin;          // pinned host mirror of the outer driver's device scratch (grown on demand)
  char *fs_pin_dev;      // the address the device reads and writes the mirror through, or null
  size_t fs_pin_bytes;
  hipStream_t aux[3];
  hipEvent_t fork_ev, join_ev[3];
  bool multi_stream;
  int n_cus;  // compute units of the device the handle was created on
  rannc_dp_solve_info_t info;  // of the last successful solve
  bool no_times[4];  // per device-count class of the last solve: the stage-time table was not built
  int tune_spw;  // > 0: override of the rows-per-wave heuristic (RANNC_DP_ROWS_PER_WAVE)
  int fused_small;  // one-launch kernel for classes of small searches: 1 = where it pays (default),
                    // 0 = never, 2 = whenever N <= 128 (RANNC_DP_FUSED_SMALL)
  int64_t call_total_bound;  // > 0 during the outer driver's solve: no search's total time exceeds it
};

extern "C" {

const char *rannc_dp_strerror(int status) {
  switch (status) {
    case RANNC_DP_OK: return "ok";
    case RANNC_DP_INVALID_ARG: return "invalid argument";
    case RANNC_DP_LIMIT_EXCEEDED: return "problem exceeds the limits of the handle";
    case RANNC_DP_WORKSPACE_TOO_SMALL: return "workspace too small for this batch";
    case RANNC_DP_OVERFLOW: return "size computation overflow";
    case RANNC_DP_HIP_ERROR: return "HIP runtime error";
    case RANNC_DP_BAD_STATE: return "no solved batch on this handle";
    case RANNC_DP_NO_HOST_MEMORY: return "out of host memory";
    default: return "unknown status";
  }
}

size_t rannc_dp_workspace_bytes(const rannc_dp_limits_t *l) {
  if (!limits_ok(l)) return 0;
  Sizes sz;
  const int S_eff = std::min(l->max_stages, std::min(l->max_blocks, l->max_devices));
  if (!problem_sizes(l->max_blocks, l->max_devices, S_eff, bits_of(l), split_of(l), packed_of(l), &sz)) return 0;
  const unsigned __int128 tot =
      (unsigned __int128)sz.total() * (unsigned)l->max_problems + header_bytes(l->max_problems);
  if (tot > ((unsigned __int128)1 << 47)) return 0;
  return (size_t)tot;
}

size_t rannc_dp_workspace_bytes_for(const rannc_dp_limits_t *l, const rannc_dp_batch_t *b) {
  if (!limits_ok(l) || check_batch(l, b) != RANNC_DP_OK) return 0;
  size_t tot = header_bytes(l->max_problems);
  for (int q = 0; q < b->n_problems; ++q) {
    Sizes sz;
    const int S_eff = std::min(b->max_stages[q], std::min(b->n_blocks[q], b->n_devices[q]));
    if (!problem_sizes(b->n_blocks[q], b->n_devices[q], S_eff, bits_of(l), split_of(l), packed_of(l), &sz)) return 0;
    tot += sz.total();
    if (tot > ((size_t)1 << 47)) return 0;
  }
  return tot;
}

int rannc_dp_create(const rannc_dp_limits_t *l, void *d_workspace, size_t workspace_bytes,
                    rannc_dp_t **out) {
  if (out) *out = nullptr;
  if (!out || !limits_ok(l) || !d_workspace || ((uintptr_t)d_workspace % kAlign) != 0)
    return RANNC_DP_INVALID_ARG;
  if (workspace_bytes < header_bytes(l->max_problems)) return RANNC_DP_WORKSPACE_TOO_SMALL;
  rannc_dp *h = new (std::nothrow) rannc_dp();
  if (!h) return RANNC_DP_NO_HOST_MEMORY;
  h->lim = *l;
  h->bits = bits_of(l);
  h->ws = (char *)d_workspace;
  h->ws_bytes = workspace_bytes;
  h->staging_bytes = header_bytes(l->max_problems);
  h->next_slot = 0;
  h->solved = false;
  h->Q = 0;
  h->timing = false;
  h->ev_valid = false;
  h->level_launches = 0;
  h->tune_spw = l->rows_per_wave;
  for (int k = 0; k < 4; ++k) h->no_times[k] = false;
  h->call_total_bound = 0;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
      (void)hipGetLastError();
      cus = 256;
    }
    h->n_cus = cus;
  }
  if (const char *e = std::getenv("RANNC_DP_ROWS_PER_WAVE")) h->tune_spw = std::atoi(e);
  h->fused_small = l->one_launch_small == 1 ? 0 : l->one_launch_small == 2 ? 2 : 1;
  if (const char *e = std::getenv("RANNC_DP_FUSED_SMALL")) h->fused_small = std::atoi(e);
  h->d_probs = (ProblemDev *)h->ws;
  h->fs_pin = nullptr;
  h->fs_pin_dev = nullptr;
  h->fs_pin_bytes = 0;
  h->multi_stream = l->single_stream == 0;
  if (const char *e = std::getenv("RANNC_DP_STREAMS")) h->multi_stream = std::atoi(e) != 0;
  int made_staging = 0, made_ev_s = 0, made_ev = 0, made_aux = 0, made_join = 0;
  bool made_fork = false;
  bool ok = true;
  for (int k = 0; k < kStagingSlots && ok; ++k) {
    h->staging_used[k] = false;
    ok = hipHostMalloc((void **)&h->staging[k], h->staging_bytes, hipHostMallocDefault) == hipSuccess;
    if (ok) ++made_staging;
  }
  for (int k = 0; k < kStagingSlots && ok; ++k) {
    ok = hipEventCreateWithFlags(&h->staging_free[k], hipEventDisableTiming) == hipSuccess;
    if (ok) ++made_ev_s;
  }
  for (int k = 0; k < 4 && ok; ++k) {
    ok = hipEventCreate(&h->ev[k]) == hipSuccess;
    if (ok) ++made_ev;
  }
  for (int k = 0; k < 3 && ok; ++k) {
    ok = hipStreamCreateWithFlags(&h->aux[k], hipStreamNonBlocking) == hipSuccess;
    if (ok) ++made_aux;
  }
  for (int k = 0; k < 3 && ok; ++k) {
    ok = hipEventCreateWithFlags(&h->join_ev[k], hipEventDisableTiming) == hipSuccess;
    if (ok) ++made_join;
  }
  if (ok) {
    ok = hipEventCreateWithFlags(&h->fork_ev, hipEventDisableTiming) == hipSuccess;
    made_fork = ok;
  }
  if (!ok) {
    for (int k = 0; k < made_aux; ++k) (void)hipStreamDestroy(h->aux[k]);
    for (int k = 0; k < made_join; ++k) (void)hipEventDestroy(h->join_ev[k]);
    if (made_fork) (void)hipEventDestroy(h->fork_ev);
    for (int k = 0; k < made_staging; ++k) (void)hipHostFree(h->staging[k]);
    for (int k = 0; k < made_ev_s; ++k) (void)hipEventDestroy(h->staging_free[k]);
    for (int k = 0; k < made_ev; ++k) (void)hipEventDestroy(h->ev[k]);
    delete h;
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  *out = h;
  return RANNC_DP_OK;
}

void rannc_dp_destroy(rannc_dp_t *h) {
  if (!h) return;
  for (int k = 0; k < kStagingSlots; ++k) {
    if (h->staging_used[k]) (void)hipEventSynchronize(h->staging_free[k]);
    (void)hipHostFree(h->staging[k]);
    (void)hipEventDestroy(h->staging_free[k]);
  }
  for (int k = 0; k < 4; ++k) (void)hipEventDestroy(h->ev[k]);
  for (int k = 0; k < 3; ++k) {
    (void)hipStreamSynchronize(h->aux[k]);
    (void)hipStreamDestroy(h->aux[k]);
    (void)hipEventDestroy(h->join_ev[k]);
  }
  (void)hipEventDestroy(h->fork_ev);
  if (h->fs_pin) (void)hipHostFree(h->fs_pin);
  delete h;
}

int rannc_dp_set_timing(rannc_dp_t *h, int enabled) {
  if (!h) return RANNC_DP_INVALID_ARG;
  h->timing = enabled != 0;
  return RANNC_DP_OK;
}

int rannc_dp_get_timing(rannc_dp_t *h, float *out_ms, int32_t *out_level_launches) {
  if (!h || !out_ms) return RANNC_DP_INVALID_ARG;
  if (!h->ev_valid) return RANNC_DP_BAD_STATE;
  if (hipEventSynchronize(h->ev[3]) != hipSuccess) return RANNC_DP_HIP_ERROR;
  for (int k = 0; k < 3; ++k)
    if (hipEventElapsedTime(&out_ms[k], h->ev[k], h->ev[k + 1]) != hipSuccess) return RANNC_DP_HIP_ERROR;
  if (out_level_launches) *out_level_launches = h->level_launches;
  return RANNC_DP_OK;
}

int rannc_dp_solve(rannc_dp_t *h, const rannc_dp_batch_t *b, void *hip_stream, int64_t *d_opt,
                   int32_t *d_n_stages, int64_t *d_est_iter_ns, int32_t *d_status) {
  if (!h || !d_opt || !d_n_stages) return RANNC_DP_INVALID_ARG;
  int rc = check_batch(&h->lim, b);
  if (rc != RANNC_DP_OK) return rc;
  if (!b->time_ns || !b->param_bytes || !b->act_bytes) return RANNC_DP_INVALID_ARG;
  const bool split = split_of(&h->lim);
  if (split != (b->time_bwd_ns != nullptr)) return RANNC_DP_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  const int Q = b->n_problems;

  // ---- device order: problems grouped by the padded device dimension their kernels are
  //      specialised for, so that one launch covers a contiguous slice of descriptors --------
  static const int kClasses[4] = {8, 16, 32, 64};
  std::vector<ProblemDev> probs;
  std::vector<int32_t> pos_of;
  try {
    probs.resize(Q);
    pos_of.resize(Q);
  } catch (...) {
    return RANNC_DP_NO_HOST_MEMORY;
  }
  int cls_start[5] = {0, 0, 0, 0, 0};
  for (int q = 0; q < Q; ++q)
    for (int k = 0; k < 4; ++k)
      if (rannc::dp_class(b->n_devices[q]) == kClasses[k]) ++cls_start[k + 1];
  for (int k = 0; k < 4; ++k) cls_start[k + 1] += cls_start[k];
  {
    int next[4] = {cls_start[0], cls_start[1], cls_start[2], cls_start[3]};
    for (int q = 0; q < Q; ++q)
      for (int k = 0; k < 4; ++k)
        if (rannc::dp_class(b->n_devices[q]) == kClasses[k]) pos_of[q] = next[k]++;
  }

  // ---- workspace layout -------------------------------------------------------------
  LaunchShape shape[4];
  std::memset(shape, 0, sizeof(shape));
  size_t off = header_bytes(h->lim.max_problems);
  for (int q = 0; q < Q; ++q) {
    const int N = b->n_blocks[q], D = b->n_devices[q];
    const int S_eff = std::min(b->max_stages[q], std::min(N, D));
    Sizes sz;
    if (!problem_sizes(N, D, S_eff, h->bits, split, packed_of(&h->lim), &sz)) return RANNC_DP_OVERFLOW;
    if (off + sz.total() > h->ws_bytes) return RANNC_DP_WORKSPACE_TOO_SMALL;
    ProblemDev &p = probs[pos_of[q]];
    std::memset(&p, 0, sizeof(p));
    p.N = N; p.D = D; p.S_eff = S_eff; p.MB = b->n_microbatches[q];
    p.DP = rannc::dp_class(D);
    p.nch = (N + 63) / 64;
    p.bits = h->bits;
    p.q = q;
    p.M = b->mem_capacity[q];
    p.time_limit = h->lim.max_total_time_ns;
    p.t = b->time_ns + b->block_offset[q];
    p.p = b->param_bytes + b->block_offset[q];
    p.a = b->act_bytes + b->block_offset[q];
    p.o = b->cut_bytes ? b->cut_bytes + b->block_offset[q] : nullptr;
    p.bw = b->cut_bytes ? b->bandwidth_bytes_per_us[q] : 0;
    char *base = h->ws + off;
    p.T = (int64_t *)base; base += sz.prefix;
    p.P = (int64_t *)base; base += sz.prefix;
    p.A = (int64_t *)base; base += sz.prefix;
    p.C = b->cut_bytes ? (int64_t *)base : nullptr; base += sz.prefix;
    if (split) {
      p.tb = b->time_bwd_ns + b->block_offset[q];
      p.TB = (int64_t *)base; base += sz.prefix;
    }
    p.wlo = (int32_t *)base; base += sz.wlo;
    p.runs = (int32_t *)base; base += sz.runs;
    p.ufit = (uint8_t *)base; base += sz.ufit;
    p.status = (int32_t *)base;
    p.res = (int64_t *)(base + 16); base += sz.misc;
    p.rmin = (uint8_t *)base; base += sz.rmin;
    p.cost = base; base += sz.cost;
    p.V = base; base += sz.V;
    if (split) {
      p.costb = base; base += sz.cost;
      p.VF = base; base += sz.V;
      p.VB = base; base += sz.V;
      if (sz.keys) { p.keys = base; base += sz.keys; }
    }
    off += sz.total();
    for (int k = 0; k < 4; ++k)
      if (p.DP == kClasses[k]) {
        LaunchShape &sh = shape[k];
        sh.nprob++;
        sh.max_N = std::max(sh.max_N, p.N);
        sh.max_nch = std::max(sh.max_nch, p.nch);
        sh.max_D = std::max(sh.max_D, p.D);
        sh.max_S_eff = std::max(sh.max_S_eff, p.S_eff);
      }
  }

  // ---- descriptors to the device ---------------------------------------------------
  const int slot = h->next_slot;
  h->next_slot = (slot + 1) % kStagingSlots;
  if (h->staging_used[slot] && hipEventSynchronize(h->staging_free[slot]) != hipSuccess)
    return RANNC_DP_HIP_ERROR;
  const size_t probs_bytes = (size_t)Q * sizeof(ProblemDev);
  std::memcpy(h->staging[slot], probs.data(), probs_bytes);
  h->solved = false;
  if (hipMemcpyAsync(h->ws, h->staging[slot], probs_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
      hipEventRecord(h->staging_free[slot], st) != hipSuccess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  h->staging_used[slot] = true;

  // ---- kernels ---------------------------------------------------------------------------
  const ProblemDev *dp = h->d_probs;
  const bool scan = h->lim.algo == RANNC_DP_ALGO_SCAN;
  // split objective: packed-key kernel wherever a cell's winner fits a 64-bit word (all 32-bit
  // handles, 64-bit ones up to 2^42 - 2 ns); RANNC_DP_ALGO_SCAN and larger time bounds take the
  // literal one
  const bool split_fast = split && !scan && packed_of(&h->lim);
  // stage times recomputed inside the level kernel instead of read from their table: where it
  // applies, on request, or (AUTO) for the classes whose launches are large enough to be bound by
  // throughput
  const bool can_recompute = !scan && !split && h->bits == 32 && !b->cut_bytes;
  bool recompute_cls[4];
  for (int k = 0; k < 4; ++k)
    recompute_cls[k] = can_recompute && (h->lim.algo == RANNC_DP_ALGO_RECOMPUTE ||
                                         (h->lim.algo == RANNC_DP_ALGO_AUTO &&
                                          rannc::merge_launch_rows(shape[k]) >=
                                              (shape[k].nprob > 1 ? rannc::kRecomputeRowsFromMany
                                                                  : rannc::kRecomputeRowsFrom)));
  bool ok = true;
  const bool timing = h->timing;
  h->ev_valid = false;
  h->level_launches = 0;
  if (timing) ok = ok && hipEventRecord(h->ev[0], st) == hipSuccess;
  // what the host knows about the total time of a search of this batch: the handle's bound, or the
  // outer driver's own sum over the inputs it has just scaled
  const int64_t total_bound = h->call_total_bound > 0 ? std::min(h->call_total_bound, h->lim.max_total_time_ns)
                                                      : h->lim.max_total_time_ns;
  bool fused[4] = {false, false, false, false};
  bool fused_direct[4] = {false, false, false, false};  // one-launch kernel that recomputes the stage times
  // estimated time of a class of few small searches (us): as one launch with recomputed stage times
  // (< 0: that kernel does not apply) and as launches per level
  double est_one[4] = {-1.0, -1.0, -1.0, -1.0}, est_levels[4] = {0.0, 0.0, 0.0, 0.0};
  for (int k = 0; k < 4; ++k) {
    const LaunchShape &sh = shape[k];
    if (!sh.nprob) continue;
    // Small searches: everything in one launch, one workgroup per search, where that measured
    // faster than the launches per level (MI355X; N = 16..128, D = 8..64, 1..512 searches per class).
    {
      const int64_t rows = std::min(sh.max_N, 64) + (sh.max_nch > 1 ? sh.max_N : 0);
      const int levels = sh.max_S_eff - 1;
      const int cls = kClasses[k];
      // the launches per level of a few small searches: 14 us in front of the levels, 4.4 us a level
      const double launches_us = 14.0 + 4.4 * levels;
      const bool direct_ok = !scan && !split && !b->cut_bytes && h->lim.algo != RANNC_DP_ALGO_MERGE &&
                             rannc::small_can_recompute(h->bits, cls, total_bound);
      const bool heavy = h->bits / 8 * cls >= 256;  // the variants that run eight waves per search
      bool tiny;
      if (direct_ok) {
        // Stage times recomputed: the levels read nothing from memory.  The kernel runs a level as
        // passes of 64 (row, column) pairs packed from the triangular and rectangular blocks, sixteen
        // waves at a time.  Least-squares fit over a sweep (N = 8..128, D = 8, 16, 32, S = 2..D, 1 and
        // 8 searches; rms 3.7 us): 12 us + 0.04 us per table row in front, then per level a constant
        // and a price per pass that follow the width of the merge the level still needs (32 / 16 / 8
        // inputs), the passes of the first round of sixteen dearer than the later ones.  The launches
        // per level on the same sweep: 21 us + 4.4 us per level + 0.05 us per block.
        auto tri = [](int W) {
          int lg = 0;
          while ((1 << lg) < W) ++lg;
          return (W / 2 + (64 >> lg)) >> (6 - lg);
        };
        int passes = tri(std::min(sh.max_N, 64));
        if (sh.max_N > 64) {
          int lg = 0;
          while ((1 << lg) < sh.max_N - 64) ++lg;
          passes += (64 >> (6 - lg)) + tri(sh.max_N - 64);
        }
        const double work = 0.17 * std::min(passes, 16) + 0.105 * std::max(passes - 16, 0);
        const bool w64 = h->bits == 64;  // the same fit on 64-bit values (rms 5.7 us; eight waves at 32 devices)
        double us = w64 ? 13.0 + 0.02 * (double)rows : 12.0 + 0.04 * (double)rows;
        for (int s = 2; s <= sh.max_S_eff; ++s) {
          const int rl = sh.max_D - s + 1;
          if (w64) us += rl <= 8 ? 0.33 + 0.63 * work : rl <= 16 ? 1.1 + 0.9 * work : 1.45 + 1.62 * work;
          else us += rl <= 8 ? 0.43 + 0.45 * work : rl <= 16 ? 0.68 + 0.61 * work : 1.5 + 0.91 * work;
        }
        est_one[k] = us;
        tiny = us <= (w64 ? 22.0 + 5.5 * levels + 0.06 * sh.max_N : 21.0 + 4.4 * levels + 0.05 * sh.max_N);
      } else if (heavy) {
        // 64 devices, or 64-bit values from 32 devices on, stage times from the table: a level costs
        // about 7 us plus 1.7 us per pass of eight rows, more than a launch; only two or three levels
        // are cheaper in one launch
        tiny = rows <= (h->bits == 64 ? 16 : 32) && (7.0 + 1.7 * (double)((rows + 7) / 8)) * levels <= launches_us;
      } else {
        // stage times from the table, sixteen waves (sweep over N = 8..128, D = 8, 16, S = 2..D)
        tiny = rows <= 64 && rows * levels <= (h->bits == 64 ? 240 : 480);
      }
      // hundreds of searches: the launches per level are throughput-bound as well
      const bool batch = sh.nprob >= 256 && (cls <= 16 || sh.max_N <= 64) && !(h->bits == 64 && cls == 64);
      fused[k] = !scan && !split && sh.max_N <= rannc::small_max_blocks() &&
                 (h->fused_small == 1 ? (batch || tiny) : h->fused_small == 2);
      fused_direct[k] = fused[k] && direct_ok;
      est_levels[k] = h->bits == 64 ? 22.0 + 5.5 * levels + 0.06 * sh.max_N : 21.0 + 4.4 * levels + 0.05 * sh.max_N;
    }
  }
  // Classes in the shadow of the longest one.  The classes of a batch run side by side on streams
  // of their own, so the call takes as long as its longest class -- or as long as the host needs to
  // enqueue everything: a class of launches per level costs the host some 3 us per launch (outer
  // driver at 128 blocks: 118 launches, 0.385 ms per call for 0.27 ms of device time).  A class of
  // few searches that is not the longest and would finish as ONE launch within the longest class's
  // time takes the one-launch kernel even where its own launches per level would be faster.
  bool share_stream = true;  // the one-launch classes besides the first share one stream
  if (h->fused_small == 1 && h->multi_stream && !timing) {
    double longest = 0.0;
    int crit = -1;
    for (int k = 0; k < 4; ++k) {
      if (!shape[k].nprob) continue;
      const double t = fused[k] && est_one[k] >= 0.0 ? est_one[k] : est_levels[k];
      if (t > longest) { longest = t; crit = k; }
    }
    for (int k = 0; k < 4; ++k)
      if (shape[k].nprob && k != crit && !fused[k] && est_one[k] >= 0.0 && est_one[k] <= longest &&
          shape[k].nprob <= 64 && shape[k].max_N <= rannc::small_max_blocks())
        fused[k] = fused_direct[k] = true;
    double sum = 0.0;
    for (int k = 0; k < 4; ++k)
      if (shape[k].nprob && fused[k] && k != crit && est_one[k] >= 0.0) sum += est_one[k];
    share_stream = sum <= longest;
  }
  // one stream per device-count class: the largest class stays on the caller's stream
  hipStream_t cs[4] = {st, st, st, st};
  int n_aux = 0;
  if (h->multi_stream && !timing) {
    // (the other classes that run as ONE launch each share a stream where together they stay within
    // the longest class's time: every stream costs a wait on the fork event and one on its join
    // event, 10 us of host time each)
    bool first = true;
    int shared = -1;
    for (int k = 3; k >= 0; --k) {
      if (!shape[k].nprob) continue;
      if (first) { first = false; continue; }
      if (fused[k] && share_stream) {
        if (shared < 0) shared = n_aux++;
        cs[k] = h->aux[shared];
      } else {
        cs[k] = h->aux[n_aux++];
      }
    }
    if (n_aux > 0) {
      ok = ok && hipEventRecord(h->fork_ev, st) == hipSuccess;  // descriptors are on the device
      for (int a = 0; a < n_aux && ok; ++a) ok = hipStreamWaitEvent(h->aux[a], h->fork_ev, 0) == hipSuccess;
    }
  }
  int merge_items[4] = {1, 1, 1, 1};
  for (int k = 0; k < 4 && ok; ++k) {
    const LaunchShape &sh = shape[k];
    if (!sh.nprob) continue;
    const ProblemDev *cp = dp + cls_start[k];
    const hipStream_t st = cs[k];  // this class's stream
    if (fused[k]) continue;
    ok = rannc::launch_prefix(cp, sh.nprob, st) == hipSuccess;
    ok = ok && rannc::launch_fill(cp, sh.nprob, st) == hipSuccess;
    ok = ok && rannc::launch_build(cp, sh, h->bits, kClasses[k], recompute_cls[k] ? 1 : 3, st) == hipSuccess;
    ok = ok && rannc::launch_windows(cp, sh, st) == hipSuccess;  // also used by traceback
    if (split) {
      ok = ok && rannc::launch_split_level1(cp, sh, h->bits, st) == hipSuccess;
      if (split_fast) ok = ok && rannc::launch_runs(cp, sh.nprob, rannc::split_rows_per_item(sh, h->n_cus), 0, 0, false, st) == hipSuccess;
    }
    if (scan || split) continue;
    // Rows per item of the level kernel: chosen on the device from the size of the windows unless
    // the handle fixes it, or the host does for a launch of many rounds (merge_grid_items).
    const int slots = h->n_cus * rannc::merge_workgroups_per_cu(h->bits, kClasses[k], recompute_cls[k]);
    int rows_for_list = -1;
    merge_items[k] = rannc::merge_grid_items(sh, rannc::merge_rows_per_item(h->tune_spw), slots, recompute_cls[k],
                                             &rows_for_list);
    ok = ok && rannc::launch_runs(cp, sh.nprob, rows_for_list, merge_items[k], slots, recompute_cls[k], st) == hipSuccess;
  }
  if (timing) ok = ok && hipEventRecord(h->ev[1], st) == hipSuccess;
  int max_levels = 0;
  for (int k = 0; k < 4; ++k) {
    if (fused[k]) {
      ok = ok && rannc::launch_solve_small(dp + cls_start[k], shape[k].nprob, h->bits, kClasses[k], fused_direct[k], d_opt,
                                           d_n_stages, d_est_iter_ns, d_status, cs[k]) == hipSuccess;
      h->level_launches++;
    } else {
      max_levels = std::max(max_levels, shape[k].max_S_eff);
    }
  }
  for (int s = 2; s <= max_levels && ok; ++s) {
    for (int k = 0; k < 4 && ok; ++k) {
      const LaunchShape &sh = shape[k];
      if (!sh.nprob || sh.max_S_eff < s || fused[k]) continue;
      const hipStream_t st = cs[k];
      if (split_fast)
        ok = rannc::launch_level_split_fast(dp + cls_start[k], sh, h->bits, kClasses[k], s,
                                            rannc::split_rows_per_item(sh, h->n_cus), st) == hipSuccess;
      else if (split)
        ok = rannc::launch_level_split(dp + cls_start[k], sh, h->bits, s, 1, nullptr, nullptr, st) ==
             hipSuccess;
      else if (scan)
        ok = rannc::launch_level_scan(dp + cls_start[k], sh, h->bits, s, 1, nullptr, nullptr, st) ==
             hipSuccess;
      else
        ok = rannc::launch_level_merge(dp + cls_start[k], sh, h->bits, kClasses[k], s, recompute_cls[k], merge_items[k],
                                       // measured: c4 (64 devices) 0.410 -> 0.401 ms; c3, c2 (32, 16 devices,
                                       // launches of 4-6 us) 1-2 us slower per solve with the larger argument block
                                       sh.nprob == 1 && kClasses[k] == 64 ? &probs[cls_start[k]] : nullptr, st) == hipSuccess;
      h->level_launches++;
    }
  }
  if (timing) ok = ok && hipEventRecord(h->ev[2], st) == hipSuccess;
  for (int k = 0; k < 4 && ok; ++k)
    if (shape[k].nprob && !fused[k])
      ok = rannc::launch_select(dp + cls_start[k], shape[k].nprob, d_opt, d_n_stages, d_est_iter_ns,
                                d_status, cs[k]) == hipSuccess;
  for (int a = 0; a < n_aux && ok; ++a)  // join: the caller's stream continues after every class
    ok = hipEventRecord(h->join_ev[a], h->aux[a]) == hipSuccess &&
         hipStreamWaitEvent(st, h->join_ev[a], 0) == hipSuccess;
  if (timing) ok = ok && hipEventRecord(h->ev[3], st) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    // nothing of this solve may still run on the handle's streams when the caller sees the error
    for (int a = 0; a < n_aux; ++a) (void)hipStreamSynchronize(h->aux[a]);
    return RANNC_DP_HIP_ERROR;
  }
  h->ev_valid = timing;
  for (int k = 0; k < 4; ++k) {
    h->no_times[k] = fused[k] ? fused_direct[k] : recompute_cls[k];
    h->info.n_problems[k] = shape[k].nprob;
    h->info.level_kernel[k] = !shape[k].nprob ? RANNC_DP_KERNEL_NONE
                              : fused[k]      ? (fused_direct[k] ? RANNC_DP_KERNEL_ONE_LAUNCH_RECOMPUTE : RANNC_DP_KERNEL_ONE_LAUNCH)
                              : split_fast    ? RANNC_DP_KERNEL_SPLIT
                              : split         ? RANNC_DP_KERNEL_SPLIT_SCAN
                              : scan          ? RANNC_DP_KERNEL_SCAN
                              : recompute_cls[k] ? RANNC_DP_KERNEL_MERGE_RECOMPUTE
                                                 : RANNC_DP_KERNEL_MERGE_TABLE;
  }
  h->host_probs.swap(probs);
  h->pos_of.swap(pos_of);
  h->Q = Q;
  h->solved = true;
  return RANNC_DP_OK;
}

constexpr int kTracebackStagedMaxProblems = 64;
// outer driver: inputs of up to this many bytes are read by the kernels out of the pinned host mirror
constexpr size_t kFsReadInPlaceMax = 32 << 10;

int rannc_dp_solve_info(rannc_dp_t *h, rannc_dp_solve_info_t *out) {
  if (!h || !out) return RANNC_DP_INVALID_ARG;
  if (!h->solved) return RANNC_DP_BAD_STATE;
  *out = h->info;
  return RANNC_DP_OK;
}

// rec: the outer driver's result record on the device (the chosen search's plan is also written
// behind it), or null
static int traceback_impl(rannc_dp_t *h, void *hip_stream, const int32_t *d_levels, int32_t plan_stride,
                          int32_t *d_stage_end, int32_t *d_replicas, int64_t *d_rec) {
  if (!h || !d_stage_end || !d_replicas || plan_stride < 1) return RANNC_DP_INVALID_ARG;
  if (!h->solved) return RANNC_DP_BAD_STATE;
  // A few small min-max searches: the walk runs out of LDS (one round of reads instead of one
  // memory round trip per stage).  Many searches fill the device anyway, and a workgroup that holds
  // most of a compute unit's LDS would then only lower the number in flight.
  int64_t lds_bytes = 0;
  bool staged = h->Q <= kTracebackStagedMaxProblems;
  for (int q = 0; q < h->Q; ++q) {
    const ProblemDev &p = h->host_probs[q];
    if (p.S_eff > plan_stride) return RANNC_DP_INVALID_ARG;
    const int64_t need = rannc::traceback_lds_bytes(p.N, p.DP, p.S_eff, p.bits);
    staged = staged && !p.VF && need <= rannc::kTracebackLdsMax;
    lds_bytes = std::max(lds_bytes, need);
  }
  if (!staged) lds_bytes = 0;
  if (rannc::launch_traceback(h->d_probs, h->Q, plan_stride, d_stage_end, d_replicas, d_levels, lds_bytes, d_rec,
                              (hipStream_t)hip_stream) != hipSuccess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  return RANNC_DP_OK;
}

int rannc_dp_traceback_at(rannc_dp_t *h, void *hip_stream, const int32_t *d_levels, int32_t plan_stride,
                          int32_t *d_stage_end, int32_t *d_replicas) {
  return traceback_impl(h, hip_stream, d_levels, plan_stride, d_stage_end, d_replicas, nullptr);
}

int rannc_dp_traceback(rannc_dp_t *h, void *hip_stream, int32_t plan_stride, int32_t *d_stage_end,
                       int32_t *d_replicas) {
  return rannc_dp_traceback_at(h, hip_stream, nullptr, plan_stride, d_stage_end, d_replicas);
}

int rannc_dp_level_values(rannc_dp_t *h, void *hip_stream, int32_t stride, int64_t *d_values) {
  if (!h || !d_values || stride < 1) return RANNC_DP_INVALID_ARG;
  if (!h->solved) return RANNC_DP_BAD_STATE;
  for (int q = 0; q < h->Q; ++q)
    if (h->host_probs[q].S_eff > stride) return RANNC_DP_INVALID_ARG;
  if (rannc::launch_level_values(h->d_probs, h->Q, stride, d_values, (hipStream_t)hip_stream) != hipSuccess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  return RANNC_DP_OK;
}

// ---- Algorithm 2 ("form_stage"): host-level driver over one batched solve ---------------------
namespace {

struct FsPair { int n, MB; int64_t b; };

// the (n, MB) pairs Algorithm 2 can visit, in its order; false if the input is invalid
bool fs_pairs(const rannc_dp_form_stage_in_t *in, std::vector<FsPair> *out, int *max_D) {
  if (!in || in->n_blocks < 1 || in->n_nodes < 1 || in->devices_per_node < 1 || in->batch_size < 1 ||
      in->mem_capacity < 0 || in->reserved != 0)
    return false;
  if (in->cut_bytes_per_sample && in->bandwidth_bytes_per_us < 1) return false;
  *max_D = 0;
  for (int64_t n = 1; n <= in->n_nodes; n *= 2) {
    const int64_t D = (int64_t)in->devices_per_node * n;
    if (D > RANNC_DP_MAX_DEVICES) return false;
    *max_D = (int)D;
    const int64_t R = in->n_nodes / n;
    for (int64_t MB = 1; MB <= in->batch_size / R; MB *= 2) {
      if (out) out->push_back({(int)n, (int)MB, in->batch_size / R / MB});
      if (MB > (1 << 29)) break;
    }
  }
  return true;
}

size_t fs_scratch(int Q, int N, int stride) {
  size_t b = 0;
  b += 5 * align_up((size_t)Q * N * 8);       // scaled time, param, act, cut bytes, backward time
  b += align_up((size_t)Q * 8);               // n and MB of every search (int32 each; travels up with the inputs)
  b += 2 * align_up((size_t)Q * 8);           // opt, (n_stages + status as int32 pairs)
  b += align_up((size_t)Q * stride * 8);      // per-level values
  b += align_up((size_t)Q * 4);               // forced levels
  b += 2 * align_up((size_t)Q * stride * 4);  // plans of the batch
  b += align_up(6 * 8 + (size_t)stride * 8);  // result record and the chosen plan (travels down)
  return b;
}

}  // namespace

int32_t rannc_dp_form_stage_problems(const rannc_dp_form_stage_in_t *in) {
  std::vector<FsPair> pairs;
  int max_D = 0;
  try {
    if (!fs_pairs(in, &pairs, &max_D)) return 0;
  } catch (...) {
    return 0;
  }
  return (int32_t)pairs.size();
}

size_t rannc_dp_form_stage_scratch_bytes(const rannc_dp_form_stage_in_t *in) {
  const int Q = rannc_dp_form_stage_problems(in);
  int max_D = 0;
  if (Q == 0 || !fs_pairs(in, nullptr, &max_D)) return 0;
  return fs_scratch(Q, in->n_blocks, max_D);
}

int rannc_dp_form_stage(rannc_dp_t *h, const rannc_dp_form_stage_in_t *in, void *hip_stream,
                        void *d_scratch, size_t scratch_bytes, rannc_dp_form_stage_out_t *out,
                        int32_t *stage_end, int32_t *replicas, int32_t plan_stride) {
  if (!h || !in || !out || !stage_end || !replicas || !d_scratch) return RANNC_DP_INVALID_ARG;
  if (!in->time_per_sample_ns || !in->act_bytes_per_sample || !in->param_bytes) return RANNC_DP_INVALID_ARG;
  std::vector<FsPair> pairs;
  int max_D = 0;
  std::vector<int64_t> hbw, hM, hoff;
  const bool comm = in->cut_bytes_per_sample != nullptr;
  std::vector<int32_t> hN, hD, hS, hMB;
  const int N = in->n_blocks;
  try {
    if (!fs_pairs(in, &pairs, &max_D)) return RANNC_DP_INVALID_ARG;
  } catch (...) {
    return RANNC_DP_NO_HOST_MEMORY;
  }
  const int Q = (int)pairs.size();
  if (Q == 0) return RANNC_DP_INVALID_ARG;
  const bool split = in->time_bwd_per_sample_ns != nullptr;
  if (split != split_of(&h->lim)) return RANNC_DP_INVALID_ARG;
  const int stride = max_D;
  if (plan_stride < std::min(stride, N)) return RANNC_DP_INVALID_ARG;
  // before anything is sized by them (the batched solve would refuse the same)
  if (N > h->lim.max_blocks || max_D > h->lim.max_devices || Q > h->lim.max_problems ||
      std::min(N, max_D) > h->lim.max_stages)
    return RANNC_DP_LIMIT_EXCEEDED;
  const size_t need = fs_scratch(Q, N, stride);
  if (scratch_bytes < need) return RANNC_DP_WORKSPACE_TOO_SMALL;
  if (((uintptr_t)d_scratch % kAlign) != 0) return RANNC_DP_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  // pinned host mirror of the device scratch: same layout, so inputs go up and results come down
  // in one copy each
  if (h->fs_pin_bytes < need) {
    if (h->fs_pin) {
      if (hipStreamSynchronize(st) != hipSuccess) return RANNC_DP_HIP_ERROR;  // an earlier call's copies
      (void)hipHostFree(h->fs_pin);
      h->fs_pin = nullptr;
      h->fs_pin_dev = nullptr;
      h->fs_pin_bytes = 0;
    }
    if (hipHostMalloc((void **)&h->fs_pin, need, hipHostMallocMapped | hipHostMallocPortable) != hipSuccess) {
      (void)hipGetLastError();
      h->fs_pin = nullptr;
      return RANNC_DP_NO_HOST_MEMORY;
    }
    h->fs_pin_bytes = need;
    // the device's view of the mirror; without one the call copies in both directions
    if (hipHostGetDevicePointer((void **)&h->fs_pin_dev, h->fs_pin, 0) != hipSuccess) {
      (void)hipGetLastError();
      h->fs_pin_dev = nullptr;
    }
  }
  try {
    if (comm) hbw.assign(Q, in->bandwidth_bytes_per_us);
    hM.assign(Q, in->mem_capacity); hoff.resize(Q + 1);
    hN.assign(Q, N); hD.resize(Q); hS.resize(Q); hMB.resize(Q);
  } catch (...) {
    return RANNC_DP_NO_HOST_MEMORY;
  }
  // layout of the scratch (device) and of its mirror (host)
  const size_t a_in = align_up((size_t)Q * N * 8);
  const size_t o_pair = 0, o_t = align_up((size_t)Q * 8);
  const size_t o_p = o_t + a_in, o_a = o_t + 2 * a_in, o_o = o_t + 3 * a_in, o_b = o_t + 4 * a_in;
  const size_t o_opt = o_t + 5 * a_in;
  const size_t o_ns = o_opt + align_up((size_t)Q * 8);
  const size_t o_vals = o_ns + align_up((size_t)Q * 8);  // (room of an earlier layout; rannc_dp_form_stage_scratch_bytes counts it)
  const size_t o_lev = o_vals + align_up((size_t)Q * stride * 8);
  const size_t o_se = o_lev + align_up((size_t)Q * 4);
  const size_t o_rp = o_se + align_up((size_t)Q * stride * 4);
  const size_t o_rec = o_rp + align_up((size_t)Q * stride * 4);
  char *dev = (char *)d_scratch, *pin = h->fs_pin;
  int64_t *ht = (int64_t *)(pin + o_t), *hp = (int64_t *)(pin + o_p), *ha = (int64_t *)(pin + o_a);
  int64_t *ho = (int64_t *)(pin + o_o), *hb = (int64_t *)(pin + o_b);
  int32_t *hpn = (int32_t *)(pin + o_pair), *hpm = hpn + Q;
  // per-microbatch inputs of every (n, MB): b samples on one pipeline replica
  const __int128 lim = (__int128)1 << 62;
  __int128 max_total = 0;  // largest total time of a search (forward, no communication term: what the
                           // kernels that care about it are restricted to)
  for (int q = 0; q < Q; ++q) {
    __int128 total = 0;
    hD[q] = in->devices_per_node * pairs[q].n;
    hS[q] = hD[q];
    hMB[q] = pairs[q].MB;
    hpn[q] = pairs[q].n;
    hpm[q] = pairs[q].MB;
    hoff[q] = (int64_t)q * N;
    for (int k = 0; k < N; ++k) {
      const int64_t ts = in->time_per_sample_ns[k], as = in->act_bytes_per_sample[k];
      if (ts < 0 || as < 0 || in->param_bytes[k] < 0) return RANNC_DP_INVALID_ARG;
      if ((__int128)ts * pairs[q].b >= lim || (__int128)as * pairs[q].b >= lim) return RANNC_DP_OVERFLOW;
      ht[(size_t)q * N + k] = ts * pairs[q].b;
      total += (__int128)ts * pairs[q].b;
      ha[(size_t)q * N + k] = as * pairs[q].b;
      hp[(size_t)q * N + k] = in->param_bytes[k];
      if (split) {
        const int64_t tb = in->time_bwd_per_sample_ns[k];
        if (tb < 0) return RANNC_DP_INVALID_ARG;
        if ((__int128)tb * pairs[q].b >= lim) return RANNC_DP_OVERFLOW;
        hb[(size_t)q * N + k] = tb * pairs[q].b;
      }
      if (comm) {
        const int64_t os = in->cut_bytes_per_sample[k];
        if (os < 0) return RANNC_DP_INVALID_ARG;
        if ((__int128)os * pairs[q].b > (lim - 1) / 1000) return RANNC_DP_OVERFLOW;
        ho[(size_t)q * N + k] = os * pairs[q].b;
      }
    }
    max_total = std::max(max_total, total);
  }
  hoff[Q] = (int64_t)Q * N;
  // The (n, MB) of every search and the block arrays in use are contiguous: one copy up.  Small
  // inputs (the paper's 32 blocks: 18 KB) are not copied at all: the mirror is pinned host memory
  // that the device reads through the same address, every word once, which costs the kernels a
  // bus round trip and saves the call a copy in front of its first kernel.
  const size_t in_bytes = o_t + (split ? 5 : comm ? 4 : 3) * a_in;
  char *pin_dev = h->fs_pin_dev;
  const bool in_place = pin_dev && in_bytes <= kFsReadInPlaceMax;
  if (!in_place && hipMemcpyAsync(dev, pin, in_bytes, hipMemcpyHostToDevice, st) != hipSuccess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  const char *src = in_place ? pin_dev : dev;
  int64_t *d_opt = (int64_t *)(dev + o_opt);
  int32_t *d_ns = (int32_t *)(dev + o_ns), *d_st = d_ns + Q;
  int32_t *d_lev = (int32_t *)(dev + o_lev), *d_se = (int32_t *)(dev + o_se), *d_rp = (int32_t *)(dev + o_rp);
  const int32_t *d_pn = (const int32_t *)(src + o_pair), *d_pm = d_pn + Q;
  // the result record and the chosen plan behind it are written by the kernels straight into the
  // mirror (they only write it): no copy down, the wait for the stream is all that is left
  int64_t *d_rec = (int64_t *)((pin_dev ? pin_dev : dev) + o_rec);
  rannc_dp_batch_t b;
  b.n_problems = Q;
  b.n_blocks = hN.data(); b.n_devices = hD.data(); b.max_stages = hS.data();
  b.n_microbatches = hMB.data(); b.mem_capacity = hM.data(); b.block_offset = hoff.data();
  b.time_ns = (const int64_t *)(src + o_t); b.param_bytes = (const int64_t *)(src + o_p);
  b.act_bytes = (const int64_t *)(src + o_a);
  b.bandwidth_bytes_per_us = comm ? hbw.data() : nullptr;
  b.cut_bytes = comm ? (const int64_t *)(src + o_o) : nullptr;
  b.time_bwd_ns = split ? (const int64_t *)(src + o_b) : nullptr;
  // Everything on the device, in stream order: the batched search, Algorithm 2's loops over the
  // values V[S][N][D] of every search and S (first n, then first S with a feasible MB; among those
  // the smallest (MB + S - 1) * V, the first found among equals), and the plan of the chosen
  // (n, MB, S), which the plan recovery also writes behind the record.  Three launches behind the
  // search's own, one copy down, one wait.
  h->call_total_bound = max_total < lim ? (int64_t)max_total : 0;
  int rc = rannc_dp_solve(h, &b, hip_stream, d_opt, d_ns, nullptr, d_st);
  h->call_total_bound = 0;
  if (rc == RANNC_DP_OK &&
      rannc::launch_form_stage_select(h->d_probs, Q, stride, N, in->n_nodes, in->devices_per_node, d_pn, d_pm,
                                      d_lev, d_rec, st) != hipSuccess) {
    (void)hipGetLastError();
    rc = RANNC_DP_HIP_ERROR;
  }
  if (rc == RANNC_DP_OK) rc = traceback_impl(h, hip_stream, d_lev, stride, d_se, d_rp, d_rec);
  if (rc != RANNC_DP_OK) {
    (void)hipStreamSynchronize(st);  // the mirror may be refilled by the next call
    return rc;
  }
  if ((!pin_dev && hipMemcpyAsync(pin + o_rec, dev + o_rec, 6 * 8 + (size_t)stride * 8, hipMemcpyDeviceToHost, st) !=
                       hipSuccess) ||
      hipStreamSynchronize(st) != hipSuccess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  const int64_t *rec = (const int64_t *)(pin + o_rec);
  const int stq = (int)rec[2];
  if (stq == RANNC_DP_PROBLEM_NEGATIVE_INPUT) return RANNC_DP_INVALID_ARG;
  if (stq != RANNC_DP_PROBLEM_OK) return RANNC_DP_OVERFLOW;  // sums or times beyond the handle's width
  std::memset(out, 0, sizeof(*out));
  for (int u = 0; u < plan_stride; ++u) stage_end[u] = replicas[u] = -1;
  const int q_sel = (int)rec[0], S_sel = (int)rec[1];
  if (q_sel < 0) return RANNC_DP_OK;  // infeasible: out->feasible = 0
  const int32_t *hse = (const int32_t *)(rec + 6), *hrp = hse + stride;
  out->feasible = 1;
  out->n = pairs[q_sel].n;
  out->devices = hD[q_sel];
  out->replica_factor = in->n_nodes / pairs[q_sel].n;
  out->n_stages = S_sel;
  out->n_microbatches = pairs[q_sel].MB;
  out->stage_time_ns = rec[4];
  out->est_iter_ns = rec[5];
  for (int u = 0; u < std::min(stride, (int)plan_stride); ++u) { stage_end[u] = hse[u]; replicas[u] = hrp[u]; }
  return RANNC_DP_OK;
}

size_t rannc_dp_compact_workspace_bytes(int32_t n_groups) {
  if (n_groups < 1 || n_groups > 65535) return 0;
  return rannc::compact_workspace_bytes(n_groups);
}

int rannc_dp_compact(void *hip_stream, int32_t n_groups, int32_t k, int32_t max_walks, int64_t mem_capacity,
                     const int64_t *d_time_ns, const int64_t *d_param_bytes, const int64_t *d_act_bytes,
                     void *d_workspace, size_t workspace_bytes, int32_t *d_n_blocks, int32_t *d_block_end,
                     int64_t *d_time_out, int64_t *d_param_out, int64_t *d_act_out, int32_t *d_status) {
  if (n_groups < 1 || n_groups > 65535 || k < 1 || max_walks < 0 || mem_capacity < 0) return RANNC_DP_INVALID_ARG;
  if (!d_time_ns || !d_param_bytes || !d_act_bytes || !d_workspace || !d_n_blocks || !d_block_end ||
      !d_time_out || !d_param_out || !d_act_out || !d_status)
    return RANNC_DP_INVALID_ARG;
  if (((uintptr_t)d_workspace % kAlign) != 0) return RANNC_DP_INVALID_ARG;
  if (workspace_bytes < rannc::compact_workspace_bytes(n_groups)) return RANNC_DP_WORKSPACE_TOO_SMALL;
  if (rannc::launch_compact(n_groups, k, mem_capacity, max_walks, d_time_ns, d_param_bytes, d_act_bytes,
                            d_workspace, d_n_blocks, d_block_end, d_time_out, d_param_out, d_act_out, d_status,
                            (hipStream_t)hip_stream) != hipSuccess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  return RANNC_DP_OK;
}

// ---- compaction for callers that cannot allocate: workspace in a static device array ----------
namespace {

constexpr size_t kCompactStaticBytes = rannc::compact_workspace_bytes(RANNC_DP_COMPACT_STATIC_MAX_GROUPS);
// Workspace of rannc_dp_compact_static.  Every device the library runs on holds its own copy at its
// own address until the process ends; host code never uses this name as an address (it is only a
// handle for hipGetSymbolAddress), kernels get the looked-up pointer as an argument.
static __device__ __align__(256) unsigned char scratch[kCompactStaticBytes];

constexpr int kMaxDevicesPerProcess = 64;
std::atomic<void *> scratch_of_device[kMaxDevicesPerProcess];

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevicesPerProcess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  void *ptr = scratch_of_device[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return RANNC_DP_HIP_ERROR;
    }
    scratch_of_device[dev].store(ptr, std::memory_order_release);  // two racing threads store the same address
  }
  *out = ptr;
  return RANNC_DP_OK;
}

}  // namespace

int rannc_dp_compact_static(void *hip_stream, int32_t n_groups, int32_t k, int32_t max_walks, int64_t mem_capacity,
                            const int64_t *d_time_ns, const int64_t *d_param_bytes, const int64_t *d_act_bytes,
                            int32_t *d_n_blocks, int32_t *d_block_end, int64_t *d_time_out, int64_t *d_param_out,
                            int64_t *d_act_out, int32_t *d_status) {
  if (n_groups < 1 || k < 1 || max_walks < 0 || mem_capacity < 0) return RANNC_DP_INVALID_ARG;
  if (n_groups > RANNC_DP_COMPACT_STATIC_MAX_GROUPS) return RANNC_DP_LIMIT_EXCEEDED;
  if (!d_time_ns || !d_param_bytes || !d_act_bytes || !d_n_blocks || !d_block_end || !d_time_out ||
      !d_param_out || !d_act_out || !d_status)
    return RANNC_DP_INVALID_ARG;
  void *ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != RANNC_DP_OK) return rc;
  // the kernel initialises every word of the workspace it later reads, so nothing has to be cleared
  if (rannc::launch_compact(n_groups, k, mem_capacity, max_walks, d_time_ns, d_param_bytes, d_act_bytes, ws,
                            d_n_blocks, d_block_end, d_time_out, d_param_out, d_act_out, d_status,
                            (hipStream_t)hip_stream) != hipSuccess) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  return RANNC_DP_OK;
}

int rannc_dp_read_table(rannc_dp_t *h, int which, int32_t problem, void *d_dst, size_t bytes,
                        void *hip_stream) {
  if (!h || !d_dst) return RANNC_DP_INVALID_ARG;
  if (!h->solved) return RANNC_DP_BAD_STATE;
  if (problem < 0 || problem >= h->Q) return RANNC_DP_INVALID_ARG;
  const int pos = h->pos_of[problem];
  const ProblemDev &p = h->host_probs[pos];
  const size_t tri = (size_t)p.N * (size_t)(p.N + 1) / 2 * (size_t)p.D;
  const size_t cells = (size_t)(p.S_eff + 1) * (size_t)(p.N + 1) * (size_t)(p.D + 1);
  size_t want = 0;
  switch (which) {
    case RANNC_DP_TABLE_COST_BWD:
      if (!p.costb) return RANNC_DP_INVALID_ARG;
      want = tri * 8;
      break;
    case RANNC_DP_TABLE_MAX_FWD:
    case RANNC_DP_TABLE_MAX_BWD:
      if (!p.VF) return RANNC_DP_INVALID_ARG;
      want = cells * 8;
      break;
    case RANNC_DP_TABLE_COST: want = tri * 8; break;
    case RANNC_DP_TABLE_FIT: want = tri; break;
    case RANNC_DP_TABLE_V: want = cells * 8; break;
    case RANNC_DP_TABLE_ARG_I:
    case RANNC_DP_TABLE_ARG_D: want = cells * 4; break;
    default: return RANNC_DP_INVALID_ARG;
  }
  if (bytes != want) return RANNC_DP_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  bool ok = true;
  int cls = 0;
  while (cls < 3 && p.DP != (8 << cls)) ++cls;
  if (h->no_times[cls] && (which == RANNC_DP_TABLE_COST || which == RANNC_DP_TABLE_ARG_I || which == RANNC_DP_TABLE_ARG_D)) {
    // the solve recomputed the stage times instead of tabulating them: tabulate this search's now
    LaunchShape one;
    one.nprob = 1; one.max_N = p.N; one.max_nch = p.nch; one.max_D = p.D; one.max_S_eff = p.S_eff;
    ok = rannc::launch_build(h->d_probs + pos, one, p.bits, p.DP, 2, st) == hipSuccess;
  }
  ok = ok && rannc::launch_export(h->d_probs + pos, which, p.bits, d_dst, st) == hipSuccess;
  if (which == RANNC_DP_TABLE_ARG_I || which == RANNC_DP_TABLE_ARG_D) {
    LaunchShape sh;
    sh.nprob = 1; sh.max_N = p.N; sh.max_nch = p.nch; sh.max_D = p.D; sh.max_S_eff = p.S_eff;
    int32_t *ai = which == RANNC_DP_TABLE_ARG_I ? (int32_t *)d_dst : nullptr;
    int32_t *ad = which == RANNC_DP_TABLE_ARG_D ? (int32_t *)d_dst : nullptr;
    for (int s = 2; s <= p.S_eff && ok; ++s)
      ok = (p.VF ? rannc::launch_level_split(h->d_probs + pos, sh, p.bits, s, 0, ai, ad, st)
                 : rannc::launch_level_scan(h->d_probs + pos, sh, p.bits, s, 0, ai, ad, st)) == hipSuccess;
  }
  if (!ok) {
    (void)hipGetLastError();
    return RANNC_DP_HIP_ERROR;
  }
  return RANNC_DP_OK;
}

}  // extern "C"
