/*
 * CPU oracle for the stage-level partition search of RaNNC (Sec. III-C, Algorithm 1).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct reference that the
 * tests, the smoke check and the benchmark's cpu_baseline leg compare the HIP path against.
 * It shares no code with the HIP path and the product never calls it.
 *
 * What it computes (all values int64, no floating point):
 *
 *   blocks k = 1..N with time t_k, persistent bytes p_k, per-microbatch transient bytes a_k;
 *   prefix sums T, P, A (T[0] = 0);
 *   a stage holding blocks i+1..j with r replicas (Sec. III-C: consecutive blocks
 *   b_{i-1} < k <= b_i, replica count sd_i) has
 *       h(i,j,r) = ceil((T[j]-T[i]) / r)                  stage time
 *       m(i,j,r) = (P[j]-P[i]) + ceil((A[j]-A[i]) / r)    stage memory
 *   and fits iff m <= M (Algorithm 1 skips a candidate only when m > M).
 *   Optional communication term (Sec. III-C counts the time to send a stage's outputs to the
 *   following stage into its execution time; Sec. III-B estimates it from the sizes of the
 *   values and the bandwidth): with o_k = bytes that cross the cut after block k for one
 *   microbatch and bandwidth w in bytes per microsecond, every stage that ends at j < N has
 *       h(i,j,r) = ceil((T[j]-T[i]) / r) + ceil(1000 * o_j / (r * w))   [ns]
 *   (each replica sends 1/r of the microbatch); the stage that ends at j = N has no follower
 *   and sends nothing.
 *   The additive form is the paper's own stand-in for profile() in Sec. IV-D (sums over the
 *   members of a stage); the replica divides the per-replica batch, hence time and transient
 *   memory, and leaves the persistent part alone.
 *
 *   Recurrence of Sec. III-C:
 *       V[s][j][d] = min over 0<=i<j, 0<=d'<d, V[s-1][i][d'] finite, stage (i,j,d-d') fits
 *                    of max(V[s-1][i][d'], h(i,j,d-d'))
 *   with V[0][0][0] = 0 and every other V[0][.][.] infinite (a plan must start at block 1
 *   with no devices spent: b_0 = 0 in Sec. III-C).  The loops run in the order of
 *   Algorithm 1 (s, then block count, then device total, then the split point ascending, then
 *   the devices of the earlier stages ascending) with the strict "<" of Algorithm 1, so among
 *   equal candidates the first one scanned is kept: the lexicographically smallest (i, d').
 *   The device-count loop is written ascending here; cells of one level are independent, so
 *   its direction does not change any value.  The d_min early break and the loop-range
 *   trimming of Algorithm 1 are search-space pruning for an expensive profiler, not part of
 *   the objective, and are not applied.
 *
 *   Answer: opt = min over 1 <= s <= min(S,N,D) of V[s][N][D], ties to the smallest s;
 *   INFEASIBLE (opt = INT64_MAX, 0 stages) if no level is finite.  The plan is recovered by
 *   following the stored (i, d') back from (s*, N, D).
 *
 *   Split objective (Algorithm 1 as printed): with separate forward and backward block times
 *   (two stage-time tables hf, hb), every cell also carries the largest forward and the largest
 *   backward stage time of its chosen plan, tf and tb.  A candidate (i, d') is valued
 *       v = max(tf[s-1][i][d'], hf(i,j,d-d')) + max(tb[s-1][i][d'], hb(i,j,d-d'))
 *   and replaces the cell's (V, tf, tb) when v is strictly smaller, candidates scanned in the
 *   same order as above.  Only ONE (tf, tb) pair survives per cell, so from the third level on
 *   this is a heuristic for min over plans of (max forward + max backward), not its exact
 *   minimum; rannc_oracle_dp_split therefore follows the algorithm's steps in its own order.
 *   What the mathematics still fixes (and the tests pin): levels 1 and 2 are exact; equal or
 *   all-zero backward times reduce to the min-max search above; every value is the value of the
 *   plan it comes with and never below the exact minimum.
 *
 * Pins (tests/test_oracle_*.py): brute-force enumeration of every plan from the definition,
 * closed forms (one stage; memory not binding; the textbook linear-partition problem),
 * invariants, and a separately written per-cell check of the canonical argmin.
 *
 * Layouts (caller allocates everything):
 *   cost, fit : packed lower triangle, entry (j,i,r), 1<=j<=N, 0<=i<j, 1<=r<=D at
 *               ((j*(j-1)/2 + i) * D + (r-1));  cost int64, fit uint8 (1 = fits)
 *   V         : int64 [(S_eff+1)][(N+1)][(D+1)]
 *   arg_i, arg_d : int32, same shape; -1 where no admissible candidate exists
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_INF INT64_MAX
#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_OVERFLOW (-4)

/* n_threads > 0: that many OpenMP threads; otherwise the number the process started with (an
 * earlier call's explicit count must not stick). */
static void set_threads(int32_t n_threads) {
#ifdef _OPENMP
  static int at_start = 0;
  if (!at_start) at_start = omp_get_max_threads();
  omp_set_num_threads(n_threads > 0 ? n_threads : at_start);
#else
  (void)n_threads;
#endif
}

static int64_t ceil_div(int64_t x, int64_t r) { return (x + r - 1) / r; } /* x >= 0, r >= 1 */

/* Inclusive prefix sums X[0] = 0, X[k] = x_1 + .. + x_k.  Rejects negative entries and
 * totals of 2^62 or more. */
int rannc_oracle_prefix(int32_t N, const int64_t *x, int64_t *X) {
  if (N < 1 || !x || !X) return ORACLE_BAD_ARG;
  const int64_t LIM = (int64_t)1 << 62;
  X[0] = 0;
  for (int32_t k = 1; k <= N; ++k) {
    int64_t v = x[k - 1];
    if (v < 0) return ORACLE_BAD_ARG;
    if (v >= LIM - X[k - 1]) return ORACLE_OVERFLOW;
    X[k] = X[k - 1] + v;
  }
  return ORACLE_OK;
}

size_t rannc_oracle_table_entries(int32_t N, int32_t D) {
  return (size_t)N * (size_t)(N + 1) / 2 * (size_t)D;
}

/* Stage time and fits-in-memory tables straight from the definitions above. */
int rannc_oracle_tables(int32_t N, int32_t D, const int64_t *T, const int64_t *P,
                        const int64_t *A, int64_t M, const int64_t *o, int64_t w, int64_t *cost,
                        uint8_t *fit) {
  if (N < 1 || D < 1 || M < 0 || !T || !P || !A || !cost || !fit) return ORACLE_BAD_ARG;
  if (o) { /* o[k-1] = bytes crossing the cut after block k; w = bytes per microsecond */
    if (w < 1) return ORACLE_BAD_ARG;
    for (int32_t k = 0; k < N; ++k) {
      if (o[k] < 0) return ORACLE_BAD_ARG;
      if (o[k] > (((int64_t)1 << 62) - 1) / 1000) return ORACLE_OVERFLOW;
    }
  }
  for (int64_t j = 1; j <= N; ++j)
    for (int64_t i = 0; i < j; ++i)
      for (int64_t r = 1; r <= D; ++r) {
        size_t e = (size_t)((j * (j - 1) / 2 + i) * D + (r - 1));
        int64_t h = ceil_div(T[j] - T[i], r);
        if (o && j < N) { /* time to send this replica's share of the cut's bytes */
          __int128 den = (__int128)r * w, num = (__int128)1000 * o[j - 1];
          h += (int64_t)((num + den - 1) / den);
        }
        int64_t m = (P[j] - P[i]) + ceil_div(A[j] - A[i], r);
        cost[e] = h;
        fit[e] = (uint8_t)(m <= M);
      }
  return ORACLE_OK;
}

/* The five nested loops, levels 1..n_levels (n_levels <= min(S,N,D)).  Level 0 is set here. */
int rannc_oracle_dp(int32_t N, int32_t D, int32_t n_levels, const int64_t *cost,
                    const uint8_t *fit, int64_t *V, int32_t *arg_i, int32_t *arg_d,
                    int32_t n_threads) {
  if (N < 1 || D < 1 || n_levels < 0 || !cost || !fit || !V || !arg_i || !arg_d)
    return ORACLE_BAD_ARG;
  const size_t ND = (size_t)(N + 1) * (size_t)(D + 1);
#define CELL(s, j, d) ((size_t)(s) * ND + (size_t)(j) * (size_t)(D + 1) + (size_t)(d))
  for (size_t e = 0; e < ((size_t)n_levels + 1) * ND; ++e) {
    V[e] = ORACLE_INF;
    arg_i[e] = -1;
    arg_d[e] = -1;
  }
  V[CELL(0, 0, 0)] = 0;
  set_threads(n_threads);
  for (int32_t s = 1; s <= n_levels; ++s) {
    /* cells (j, d) of one level depend only on level s-1 */
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int32_t j = s; j <= N; ++j) {
      for (int32_t d = s; d <= D; ++d) {
        int64_t best = ORACLE_INF;
        int32_t bi = -1, bd = -1;
        for (int32_t i = s - 1; i <= j - 1; ++i) {
          for (int32_t dp = s - 1; dp <= d - 1; ++dp) {
            int64_t prev = V[CELL(s - 1, i, dp)];
            if (prev == ORACLE_INF) continue; /* earlier stages infeasible */
            size_t e = (size_t)(((int64_t)j * (j - 1) / 2 + i) * D + (d - dp - 1));
            if (!fit[e]) continue; /* does not fit device memory */
            int64_t v = prev > cost[e] ? prev : cost[e];
            if (v < best) {
              best = v;
              bi = i;
              bd = dp;
            }
          }
        }
        V[CELL(s, j, d)] = best;
        arg_i[CELL(s, j, d)] = bi;
        arg_d[CELL(s, j, d)] = bd;
      }
    }
  }
#undef CELL
  return ORACLE_OK;
}

/* A plan for blocks 1..j on d devices as Algorithm 1 with separate forward and backward maxima sees
 * it: its longest forward and backward stage times, and where its last stage begins (split point i,
 * devices dp spent before it).  none = no such plan. */
typedef struct {
  int64_t fwd, bwd;
  int32_t i, dp;
  int none;
} split_plan_t;

/* Which of two plans for the same cell the algorithm keeps: the smaller sum of the two maxima; among
 * equal sums the one it meets first, i.e. the smaller split point, then the fewer devices before the
 * last stage (it walks both upwards and replaces only on a strictly smaller sum). */
static int split_plan_wins(const split_plan_t *x, const split_plan_t *y) {
  if (x->none || y->none) return !x->none;
  const int64_t sx = x->fwd + x->bwd, sy = y->fwd + y->bwd;
  if (sx != sy) return sx < sy;
  if (x->i != y->i) return x->i < y->i;
  return x->dp < y->dp;
}

/* Algorithm 1 with the forward and backward maxima carried separately (see the header): costf and
 * costb are two stage-time tables in the layout of `cost`, TF and TB have the shape of V and hold
 * the largest forward / backward stage time of the plan behind each cell (0 at level 0's origin,
 * INF where V is).  A cell keeps ONE plan (split_plan_wins), and only that plan is extended at the
 * next level: the heuristic of the printed algorithm, not an exact minimum. */
int rannc_oracle_dp_split(int32_t N, int32_t D, int32_t n_levels, const int64_t *costf,
                          const int64_t *costb, const uint8_t *fit, int64_t *V, int64_t *TF,
                          int64_t *TB, int32_t *arg_i, int32_t *arg_d, int32_t n_threads) {
  if (N < 1 || D < 1 || n_levels < 0 || !costf || !costb || !fit || !V || !TF || !TB || !arg_i ||
      !arg_d)
    return ORACLE_BAD_ARG;
  const size_t ND = (size_t)(N + 1) * (size_t)(D + 1);
#define CELL(s, j, d) ((size_t)(s) * ND + (size_t)(j) * (size_t)(D + 1) + (size_t)(d))
  for (size_t e = 0; e < ((size_t)n_levels + 1) * ND; ++e) {
    V[e] = TF[e] = TB[e] = ORACLE_INF;
    arg_i[e] = -1;
    arg_d[e] = -1;
  }
  V[CELL(0, 0, 0)] = TF[CELL(0, 0, 0)] = TB[CELL(0, 0, 0)] = 0;
  set_threads(n_threads);
  for (int32_t s = 1; s <= n_levels; ++s) {
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int32_t j = s; j <= N; ++j) {
      for (int32_t d = s; d <= D; ++d) {
        split_plan_t kept = {0, 0, -1, -1, 1};
        /* every way to end at (j, d): the kept plan of s-1 stages for blocks 1..i on dp devices,
         * followed by the stage (i, j] on the remaining d - dp devices */
        for (int32_t i = s - 1; i < j; ++i) {
          for (int32_t dp = s - 1; dp < d; ++dp) {
            const size_t before = CELL(s - 1, i, dp);
            const size_t stage = (size_t)(((int64_t)j * (j - 1) / 2 + i) * D) + (size_t)(d - dp - 1);
            if (V[before] == ORACLE_INF || !fit[stage]) continue; /* nothing to extend / stage too large */
            split_plan_t cand;
            cand.fwd = TF[before] > costf[stage] ? TF[before] : costf[stage];
            cand.bwd = TB[before] > costb[stage] ? TB[before] : costb[stage];
            cand.i = i;
            cand.dp = dp;
            cand.none = 0;
            if (split_plan_wins(&cand, &kept)) kept = cand;
          }
        }
        if (!kept.none) {
          const size_t c = CELL(s, j, d);
          V[c] = kept.fwd + kept.bwd;
          TF[c] = kept.fwd;
          TB[c] = kept.bwd;
          arg_i[c] = kept.i;
          arg_d[c] = kept.dp;
        }
      }
    }
  }
#undef CELL
  return ORACLE_OK;
}

/* Min-max value of cell (s, b, d) from level s-1 (the recurrence of Sec. III-C over every split
 * point and device split); *scanned counts the predecessor cells looked at. */
static int64_t minmax_cell(int32_t D, size_t ND, const int64_t *V, const int64_t *cost, const uint8_t *fit,
                           int32_t s, int32_t b, int32_t d, int64_t *scanned) {
  int64_t best = ORACLE_INF;
  for (int32_t from = s - 1; from < b; ++from) {
    for (int32_t used = s - 1; used < d; ++used) {
      ++*scanned;
      const int64_t earlier = V[(size_t)(s - 1) * ND + (size_t)from * (size_t)(D + 1) + (size_t)used];
      const size_t stage = (size_t)(((int64_t)b * (b - 1) / 2 + from) * D) + (size_t)(d - used - 1);
      if (earlier == ORACLE_INF || !fit[stage]) continue;
      const int64_t slowest = earlier > cost[stage] ? earlier : cost[stage];
      if (slowest < best) best = slowest;
    }
  }
  return best;
}

/* Algorithm 1 for EXACTLY S stages with the search-space pruning it prints (a study, not part of
 * the search the HIP path runs).  Level s looks only at block counts that leave a block for each
 * of the S-s later stages and at device totals that leave a device for each of them; the totals
 * are tried from the largest down, and the first cell anywhere that has no solution raises a
 * floor (d_min, kept for the rest of the run) to just above its device total and ends that
 * descent.  V has the shape [(S+1)][N+1][D+1]; cells that are never visited stay INF.
 * stats[0] = cells visited, stats[1] = candidates (b', d') scanned, stats[2] = final d_min. */
int rannc_oracle_dp_pruned(int32_t N, int32_t D, int32_t S, const int64_t *cost, const uint8_t *fit,
                           int64_t *V, int64_t *stats) {
  if (N < 1 || D < 1 || S < 1 || S > N || S > D || !cost || !fit || !V || !stats) return ORACLE_BAD_ARG;
  const size_t ND = (size_t)(N + 1) * (size_t)(D + 1);
  for (size_t e = 0; e < ((size_t)S + 1) * ND; ++e) V[e] = ORACLE_INF;
  V[0] = 0; /* cell (0, 0, 0) */
  int32_t floor_d = 1; /* d_min */
  int64_t cells = 0, cands = 0;
  for (int32_t s = 1; s <= S; ++s) {
    const int32_t later = S - s; /* stages still to come: each needs a block and a device */
    for (int32_t b = s; b + later <= N; ++b) {
      int32_t d = D - later;
      while (d >= s && d >= floor_d) {
        ++cells;
        const int64_t v = minmax_cell(D, ND, V, cost, fit, s, b, d, &cands);
        V[(size_t)s * ND + (size_t)b * (size_t)(D + 1) + (size_t)d] = v;
        if (v == ORACLE_INF) {
          floor_d = d + 1;
          break;
        }
        --d;
      }
    }
  }
  stats[0] = cells;
  stats[1] = cands;
  stats[2] = floor_d;
  return ORACLE_OK;
}

/* Best level for the full chain on all D devices; smallest s among equals. */
int rannc_oracle_select(int32_t N, int32_t D, int32_t n_levels, const int64_t *V,
                        int64_t *opt, int32_t *n_stages) {
  if (!V || !opt || !n_stages) return ORACLE_BAD_ARG;
  const size_t ND = (size_t)(N + 1) * (size_t)(D + 1);
  int64_t best = ORACLE_INF;
  int32_t bs = 0;
  for (int32_t s = 1; s <= n_levels; ++s) {
    int64_t v = V[(size_t)s * ND + (size_t)N * (size_t)(D + 1) + (size_t)D];
    if (v < best) {
      best = v;
      bs = s;
    }
  }
  *opt = best;
  *n_stages = bs;
  return ORACLE_OK;
}

/* Follow the stored (i, d') from (n_stages, N, D) down to level 0.  stage_end[u-1] = b_u
 * (1-based count of blocks covered by stages 1..u), replicas[u-1] = devices of stage u;
 * slots from n_stages up to max_slots-1 are set to -1. */
int rannc_oracle_traceback(int32_t N, int32_t D, int32_t n_stages, const int32_t *arg_i,
                           const int32_t *arg_d, int32_t max_slots, int32_t *stage_end,
                           int32_t *replicas) {
  if (!arg_i || !arg_d || !stage_end || !replicas || n_stages > max_slots) return ORACLE_BAD_ARG;
  const size_t ND = (size_t)(N + 1) * (size_t)(D + 1);
  for (int32_t u = 0; u < max_slots; ++u) stage_end[u] = replicas[u] = -1;
  int32_t j = N, d = D;
  for (int32_t s = n_stages; s >= 1; --s) {
    size_t c = (size_t)s * ND + (size_t)j * (size_t)(D + 1) + (size_t)d;
    int32_t i = arg_i[c], dp = arg_d[c];
    if (i < 0 || dp < 0) return ORACLE_BAD_ARG;
    stage_end[s - 1] = j;
    replicas[s - 1] = d - dp;
    j = i;
    d = dp;
  }
  if (n_stages > 0 && (j != 0 || d != 0)) return ORACLE_BAD_ARG;
  return ORACLE_OK;
}

/* Compaction step of the block-level phase (Sec. III-B, last paragraph before the stage-level
 * search), on a chain: G groups in topological order with computation time t, persistent bytes p
 * and transient bytes a each; target k blocks; device memory M.  Steps, in the paper's order:
 * the current groups are listed by ascending computation time (equal times: by position); each
 * listed group v that still stands as listed (it has neither been absorbed nor grown since) picks,
 * of its left and right neighbours in the chain, the one whose current computation time is
 * smaller (equal: the left one; only one neighbour: that one); if the union fits the device
 * memory (all persistent plus all transient bytes <= M) the two are merged into one group at
 * their place in the chain, times and bytes added up; the procedure ends as soon as k groups are
 * left.  A union is not put back into the list it was formed from.
 * Readings where the text is silent: the other neighbour is not tried when the chosen one does
 * not fit; memory of a group = p + a (one replica, the whole microbatch); a group that was merged
 * INTO (it absorbed a neighbour on that neighbour's turn) has changed and is no longer the listed
 * group either.  "Repeats this process for every v in the sorted list until |G| = k" leaves open
 * what happens when the list runs out above k groups: with max_passes <= 0 the groups that now
 * exist are listed again by their current times and the walk repeats, until k groups are left or a
 * whole walk merges nothing (then every group's chosen union exceeds M and no further walk could
 * differ); max_passes = n > 0 stops after n walks (n = 1: one walk over the initial list, which at
 * most about halves the number of groups).
 * Output: n_out groups, group u covering the input groups end[u-1]+1 .. end[u] (end[-1] = 0). */
int rannc_oracle_compact(int32_t G, const int64_t *t, const int64_t *p, const int64_t *a, int32_t k,
                         int64_t M, int32_t max_passes, int32_t *n_out, int32_t *end) {
  if (G < 1 || k < 1 || M < 0 || !t || !p || !a || !n_out || !end) return ORACLE_BAD_ARG;
  int64_t *ct = malloc(sizeof(int64_t) * (size_t)G), *cm = malloc(sizeof(int64_t) * (size_t)G);
  int32_t *prev = malloc(sizeof(int32_t) * (size_t)G), *next = malloc(sizeof(int32_t) * (size_t)G);
  int32_t *order = malloc(sizeof(int32_t) * (size_t)G);
  uint8_t *listed = malloc((size_t)G); /* still the group that was listed */
  if (!ct || !cm || !prev || !next || !order || !listed) {
    free(ct); free(cm); free(prev); free(next); free(order); free(listed);
    return ORACLE_BAD_ARG;
  }
  const int64_t LIM = (int64_t)1 << 62;
  int64_t st = 0, sm = 0;
  for (int32_t g = 0; g < G; ++g) {
    if (t[g] < 0 || p[g] < 0 || a[g] < 0 || t[g] >= LIM - st || p[g] >= LIM - sm || a[g] >= LIM - sm - p[g]) {
      free(ct); free(cm); free(prev); free(next); free(order); free(listed);
      return t[g] < 0 || p[g] < 0 || a[g] < 0 ? ORACLE_BAD_ARG : ORACLE_OVERFLOW;
    }
    st += t[g];
    sm += p[g] + a[g];
    ct[g] = t[g];
    cm[g] = p[g] + a[g];
    prev[g] = g - 1;
    next[g] = g + 1 < G ? g + 1 : -1;
  }
  int32_t count = G;
  /* a group is named by its first input group; next/prev link the group heads along the chain */
  for (int32_t pass = 1; count > k && (max_passes <= 0 || pass <= max_passes); ++pass) {
    /* the groups as they stand, by ascending time, equal times by position: the heads are met in
     * chain order and the insertion sort keeps the order of equals */
    int32_t n = 0;
    for (int32_t g = 0; g >= 0; g = next[g]) {
      order[n++] = g;
      listed[g] = 1;
    }
    for (int32_t x = 1; x < n; ++x) {
      int32_t v = order[x], y = x - 1;
      while (y >= 0 && ct[order[y]] > ct[v]) { order[y + 1] = order[y]; --y; }
      order[y + 1] = v;
    }
    int32_t merged = 0;
    for (int32_t x = 0; x < n && count > k; ++x) {
      const int32_t v = order[x];
      if (!listed[v]) continue;
      const int32_t l = prev[v], r = next[v];
      int32_t w;
      if (l < 0 && r < 0) break; /* a single group */
      if (l < 0) w = r;
      else if (r < 0) w = l;
      else w = ct[r] < ct[l] ? r : l;
      if (cm[v] + cm[w] > M) continue; /* the union does not fit */
      const int32_t first = w == l ? l : v, second = w == l ? v : r; /* chain order */
      ct[first] += ct[second];
      cm[first] += cm[second];
      next[first] = next[second];
      if (next[second] >= 0) prev[next[second]] = first;
      listed[first] = listed[second] = 0; /* neither is the listed group any more */
      --count;
      ++merged;
    }
    if (!merged) break;
  }
  int32_t n = 0;
  for (int32_t g = 0; g >= 0; g = next[g]) end[n++] = next[g] >= 0 ? next[g] : G;
  *n_out = n;
  free(ct); free(cm); free(prev); free(next); free(order); free(listed);
  return n == count ? ORACLE_OK : ORACLE_BAD_ARG;
}

/* Estimated time of one synchronous-pipeline iteration with MB microbatches over n_stages
 * stages whose slowest takes opt (fill and drain of the schedule of Fig. 1): (MB + s - 1)*opt,
 * saturating at INT64_MAX.  Secondary output only; it does not enter the search. */
int64_t rannc_oracle_est_iter_ns(int64_t opt, int32_t n_stages, int32_t MB) {
  if (n_stages <= 0 || opt == ORACLE_INF) return ORACLE_INF;
  int64_t f = (int64_t)MB + n_stages - 1;
  if (opt != 0 && f > ORACLE_INF / opt) return ORACLE_INF;
  return f * opt;
}

int rannc_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
