/*
 * rannc_dp.h -- C ABI of the MI355X stage-level partition search.
 *
 * The search is the dynamic program of RaNNC's stage-level partitioning (Sec. III-C,
 * Algorithm 1 "form_stage_dp"): split a chain of N coarsened blocks into at most S
 * contiguous pipeline stages, give every stage a replica (data-parallel) device count so
 * that the counts sum to D, require every stage to fit device memory M, and minimise the
 * time of the slowest stage.
 *
 * Cost model (the additive stand-in of Sec. IV-D for the paper's profile() call): with
 * prefix sums T, P, A of the per-block inputs, the stage of blocks i+1..j at r replicas has
 *     time  h(i,j,r) = ceil((T[j]-T[i]) / r)
 *     memory m(i,j,r) = (P[j]-P[i]) + ceil((A[j]-A[i]) / r),       fits iff m <= M.
 * Recurrence (Sec. III-C):  V[s][j][d] = min over i<j, d'<d with V[s-1][i][d'] finite and
 * (i,j,d-d') fitting of max(V[s-1][i][d'], h(i,j,d-d')),  V[0][0][0] = 0, other V[0] infinite.
 * Result: opt = min over 1 <= s <= min(S,N,D) of V[s][N][D] (ties: fewest stages); the plan
 * follows, from (s*,N,D), the lexicographically smallest (i,d') attaining each cell -- the
 * candidate Algorithm 1's scan order with its strict "<" keeps.
 *
 * All times are int64 nanoseconds, all sizes int64 bytes; results are exact integers.
 *
 * Conventions
 *  - Every function returns RANNC_DP_OK (0) or a negative rannc_dp_status_t; nothing throws.
 *  - Pointers are marked HOST or DEVICE.  DEVICE pointers must be valid on the device that is
 *    current when the call is made.  The library never allocates or frees device memory: the
 *    caller passes a workspace at create time; the handle sub-allocates inside it.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).  solve and
 *    traceback only enqueue work on that stream and return; they never synchronise the device.
 *    Inputs may be released once the stream has passed the end of solve.
 *  - A handle serves one solve at a time: a later solve reuses the workspace, so calls on one
 *    handle must be issued in stream order from one host thread.
 *  - Infeasible is a result, not an error (Algorithm 1 returns INFEASIBLE as a value):
 *    opt = INT64_MAX, n_stages = 0, plan slots -1.
 */
#ifndef RANNC_DP_H_
#define RANNC_DP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported symbols of the shared library (everything else in it is hidden). */
#define RANNC_DP_API __attribute__((visibility("default")))

typedef enum {
  RANNC_DP_OK = 0,
  RANNC_DP_INVALID_ARG = -1,         /* null pointer, count < 1, negative capacity, bad offsets */
  RANNC_DP_LIMIT_EXCEEDED = -2,      /* a problem exceeds the limits the handle was created with */
  RANNC_DP_WORKSPACE_TOO_SMALL = -3, /* workspace cannot hold the tables of this batch */
  RANNC_DP_OVERFLOW = -4,            /* size computation overflowed */
  RANNC_DP_HIP_ERROR = -5,           /* a HIP runtime call failed (launch, copy, event) */
  RANNC_DP_BAD_STATE = -6,           /* traceback / read_table before a successful solve */
  RANNC_DP_NO_HOST_MEMORY = -7
} rannc_dp_status_t;

/* Per-problem status word written to d_status by solve (device-side input validation). */
#define RANNC_DP_PROBLEM_OK 0
#define RANNC_DP_PROBLEM_NEGATIVE_INPUT 1   /* a block time or size is negative */
#define RANNC_DP_PROBLEM_SUM_OVERFLOW 2     /* a prefix sum reaches 2^62, or a cut's bytes exceed (2^62-1)/1000 */
#define RANNC_DP_PROBLEM_TIME_TOO_LARGE 3   /* total time (forward plus backward, plus the longest send time
                                               of a cut at one replica) exceeds limits.max_total_time_ns */
/* A problem with a non-zero status is reported as infeasible. */

#define RANNC_DP_MAX_DEVICES 64   /* largest D the kernels are built for */

/* Level kernels (Sec. III-C recurrence, one stage count s per launch). */
#define RANNC_DP_ALGO_AUTO 0      /* the fastest applicable of the following */
#define RANNC_DP_ALGO_MERGE 1     /* sorted-merge form of the (min,max) convolution over d'; the stage
                                     times h(i,j,r) are read from the table that solve builds */
#define RANNC_DP_ALGO_SCAN 2      /* literal scan of every (i, d') candidate per cell (reads the table) */
#define RANNC_DP_ALGO_RECOMPUTE 3 /* sorted-merge form with h(i,j,r) recomputed from the prefix sums
                                     inside the level kernel: solve then builds only the fits-in-memory
                                     table, and the stage-time table is built when rannc_dp_read_table
                                     asks for it.  Applies to 32-bit handles (max_total_time_ns up to
                                     4294967294) and batches without a communication term; elsewhere
                                     this value behaves as RANNC_DP_ALGO_MERGE.  Same results.  (The
                                     one-launch kernel of small searches, see one_launch_small, also
                                     recomputes on 64-bit handles whose max_total_time_ns is at most
                                     2^40, under AUTO and RECOMPUTE.) */

/* Handle flag: run Algorithm 1 as printed, with separate forward and backward block times.  A
 * cell of the search then keeps, besides its value, the largest forward and the largest backward
 * stage time of the plan behind it; a candidate is worth
 *   max(fwd so far, fwd time of the new stage) + max(bwd so far, bwd time of the new stage),
 * and the first candidate in scan order (split point ascending, then devices of the earlier
 * stages ascending) with the smallest sum is kept.  Only that one pair is seen by the next level:
 * from three stages on this is the paper's heuristic, not the exact minimum of
 * (largest forward + largest backward).  Batches on such a handle must carry time_bwd_ns
 * (time_ns is then the forward time); opt is the sum.  The workspace holds two more value tables
 * and a second stage-time table. */
#define RANNC_DP_FLAG_SPLIT_OBJECTIVE 1

typedef struct rannc_dp rannc_dp_t; /* opaque; owns host memory, a few events and three streams (default
                                       priority), no device memory */

/* Capacity of a handle. */
typedef struct {
  int32_t max_problems;      /* Q of the largest batch, >= 1 */
  int32_t max_blocks;        /* largest N of any problem, >= 1 */
  int32_t max_devices;       /* largest D, 1..RANNC_DP_MAX_DEVICES */
  int32_t max_stages;        /* largest S of any problem (values above it are clamped by N, D) */
  int64_t max_total_time_ns; /* bound on the sum of a problem's block times.  Up to
                                4294967294 the tables hold 32-bit values (half the memory
                                traffic); above it 64-bit.  Results are the same int64.  A tight
                                bound helps: up to 2^40 (18 minutes) small searches on 64-bit
                                tables can take the kernel that recomputes the stage times. */
  int32_t algo;              /* RANNC_DP_ALGO_* */
  int32_t flags;             /* RANNC_DP_FLAG_* or 0 */
  /* Tuning; 0 everywhere = the library's own choices.  None of them changes a result. */
  int32_t rows_per_wave;     /* sorted-merge level kernel: predecessor rows a wave takes one after the
                                other before the workgroup folds (1, 2, 4, 8, 12 or 16; values between
                                round up); 0 = by the size of the launch.  Environment override: RANNC_DP_ROWS_PER_WAVE */
  int32_t one_launch_small;  /* searches of at most 128 blocks can run as ONE launch with one workgroup
                                per search: 0 = where it measured faster (few rows x levels,
                                classes of >= 256 searches with D <= 16 or N <= 64, or a class of
                                few searches that finishes within the time of the batch's longest
                                class anyway), 1 = never,
                                2 = whenever N <= 128.  Environment override: RANNC_DP_FUSED_SMALL
                                (0 = never, 1 = where faster, 2 = always) */
  int32_t single_stream;     /* 0 = the device-count classes of a batch run on streams of the handle,
                                1 = everything on the caller's stream.  Environment override:
                                RANNC_DP_STREAMS (0 = caller's stream only) */
  int32_t reserved;          /* must be 0 */
} rannc_dp_limits_t;

/* A batch of Q independent searches (Algorithm 2 of Sec. III-C issues many form_stage_dp
 * calls with different D, S and MB; one batch is one such set).  Structure of arrays. */
typedef struct {
  int32_t n_problems;            /* Q >= 1 */
  const int32_t *n_blocks;       /* HOST [Q]  N_q >= 1 */
  const int32_t *n_devices;      /* HOST [Q]  D_q >= 1 */
  const int32_t *max_stages;     /* HOST [Q]  S_q >= 1; effective bound is min(S_q,N_q,D_q) */
  const int32_t *n_microbatches; /* HOST [Q]  MB_q >= 1; only enters est_iter_ns */
  const int64_t *mem_capacity;   /* HOST [Q]  M_q >= 0 bytes */
  const int64_t *block_offset;   /* HOST [Q+1] problem q owns entries block_offset[q] ..
                                    block_offset[q+1]-1 of the arrays below;
                                    block_offset[q+1]-block_offset[q] == N_q, block_offset[0] >= 0 */
  const int64_t *time_ns;        /* DEVICE  fwd+bwd time of a block, one microbatch, one replica */
  const int64_t *param_bytes;    /* DEVICE  persistent per-replica bytes (weights, grads, optimizer) */
  const int64_t *act_bytes;      /* DEVICE  transient bytes of one microbatch at one replica */
  /* Optional communication term (Sec. III-C: a stage's execution time includes sending its
   * outputs to the following stage; Sec. III-B: estimated from the sizes of the values and the
   * bandwidth).  Both NULL: no term.  Otherwise a stage that ends after block j < N_q on r
   * replicas takes ceil(1000 * cut_bytes[j] / (r * bandwidth)) ns longer (each replica sends its
   * 1/r of the microbatch); the stage that ends at block N_q sends nothing. */
  const int64_t *bandwidth_bytes_per_us; /* HOST [Q]  >= 1, bytes per microsecond */
  const int64_t *cut_bytes;      /* DEVICE  indexed like time_ns: bytes of the values that cross the cut
                                    after the block, one microbatch; 0 .. (2^62-1)/1000 */
  const int64_t *time_bwd_ns;    /* DEVICE  backward time of a block; required on a handle with
                                    RANNC_DP_FLAG_SPLIT_OBJECTIVE (time_ns is then the forward time and
                                    the send time of a cut belongs to the forward pass), NULL otherwise */
} rannc_dp_batch_t;

/* Bytes of device workspace that any batch within `limits` fits in (worst case).
 * Returns 0 if limits is NULL or invalid. */
RANNC_DP_API size_t rannc_dp_workspace_bytes(const rannc_dp_limits_t *limits);

/* Exact bytes a given batch needs with these limits (only HOST members of batch are read).
 * Returns 0 on invalid input. */
RANNC_DP_API size_t rannc_dp_workspace_bytes_for(const rannc_dp_limits_t *limits, const rannc_dp_batch_t *batch);

/* Create a handle over a caller-owned DEVICE workspace (256-byte aligned).  The workspace
 * must stay valid until destroy.  A workspace smaller than rannc_dp_workspace_bytes(limits) is
 * accepted; solve then rejects batches that do not fit.  *out is NULL on failure.  The handle
 * allocates pinned host staging for the descriptors, events, and three streams on the current
 * device; it never allocates device memory. */
RANNC_DP_API int rannc_dp_create(const rannc_dp_limits_t *limits, void *d_workspace, size_t workspace_bytes,
                    rannc_dp_t **out);

/* Enqueue the whole search for a batch: prefix sums, stage-time / fits-in-memory tables
 * (the h and m of Sec. III-C over every (i, j, r)), one DP level per stage count
 * (the recurrence of Sec. III-C, loops of Algorithm 1) and the final choice of the stage count.
 *   d_opt        DEVICE int64[Q]  slowest-stage time of the best plan; INT64_MAX if infeasible
 *   d_n_stages   DEVICE int32[Q]  s*; 0 if infeasible
 *   d_est_iter_ns DEVICE int64[Q] or NULL: (MB + s* - 1) * opt, the fill-and-drain time of one
 *                synchronous pipeline iteration (Fig. 1), saturating at INT64_MAX
 *   d_status     DEVICE int32[Q] or NULL: RANNC_DP_PROBLEM_* per problem
 * Searches of different device-count classes (D <= 8, 16, 32, 64) of one batch may run on streams
 * of the handle; they start after the work already on hip_stream and hip_stream is made to wait
 * for them, so for the caller everything is ordered on hip_stream as if it ran there.
 * Host-side argument errors are returned before anything is enqueued. */
RANNC_DP_API int rannc_dp_solve(rannc_dp_t *h, const rannc_dp_batch_t *batch, void *hip_stream,
                   int64_t *d_opt, int32_t *d_n_stages, int64_t *d_est_iter_ns,
                   int32_t *d_status);

/* Enqueue plan recovery for the batch of the last solve (what Algorithm 1 returns: the stage
 * boundaries and replica counts behind the optimal table value): per problem, stage u (1-based)
 * ends after block d_stage_end[q*plan_stride + u-1] (so the last used slot holds N_q) and runs on
 * d_replicas[q*plan_stride + u-1] devices (they sum to D_q).  Slots from s* on are -1.
 * plan_stride must be >= min(S_q,N_q,D_q) for every problem of the batch. */
RANNC_DP_API int rannc_dp_traceback(rannc_dp_t *h, void *hip_stream, int32_t plan_stride,
                       int32_t *d_stage_end, int32_t *d_replicas);

/* As rannc_dp_traceback, but for problem q the plan of EXACTLY d_levels[q] stages is recovered
 * (Algorithm 1's own answer for a given S: the boundaries and replica counts behind V[S][|B|][D]) when
 * d_levels[q] > 0; all slots are -1 if no plan of that many stages exists.  d_levels[q] == 0 or
 * d_levels == NULL: the best stage count chosen by solve.  d_levels[q] < 0: no plan is recovered for
 * problem q (all its slots are -1; a caller that wants one plan out of a batch pays for one walk).
 * d_levels: DEVICE int32[Q]. */
RANNC_DP_API int rannc_dp_traceback_at(rannc_dp_t *h, void *hip_stream, const int32_t *d_levels,
                                       int32_t plan_stride, int32_t *d_stage_end, int32_t *d_replicas);

/* V[s][N][D] of the last solve for every exact stage count: d_values[q*stride + s-1], s = 1..stride
 * (DEVICE int64), INT64_MAX where no plan of exactly s stages exists or s > min(S_q,N_q,D_q).
 * stride must be >= min(S_q,N_q,D_q) for every problem. */
RANNC_DP_API int rannc_dp_level_values(rannc_dp_t *h, void *hip_stream, int32_t stride, int64_t *d_values);

/* Outer driver of the search: Algorithm 2 "form_stage(N, D_node, BS)" of Sec. III-C.  For node
 * counts n = 1, 2, 4, ... <= n_nodes (D = devices_per_node * n devices, replica factor
 * R = n_nodes / n), stage counts S ascending over (devices_per_node*(n-1), devices_per_node*n] and
 * microbatch counts MB = 1, 2, 4, ... <= floor(batch_size / R), form_stage_dp is asked for a plan
 * of exactly S stages; the first S with any feasible MB returns the best of its solutions.
 * All these searches run as ONE batch through rannc_dp_solve on the given handle; the loops then
 * run over the per-level values in a small kernel, the chosen plan is recovered on the device and
 * one copy brings the result to the host.  Readings where the paper is silent: a block's time
 * and transient bytes are linear in the b = floor(batch_size / R / MB) samples of a microbatch on
 * one pipeline replica (inputs are per sample), persistent bytes are not scaled; "best" is the
 * smallest (MB + S - 1) * V (one synchronous pipeline iteration, Fig. 1), the smallest MB among
 * equals.  This call is synchronous: it waits for the stream once, at its end.  Its first use on a handle
 * (and any later use with larger inputs) allocates pinned host memory, freed by destroy.
 *   h            handle whose limits cover rannc_dp_form_stage_problems(in) problems of n_blocks
 *                blocks, devices_per_node * n_max devices and as many stages
 *   d_scratch    DEVICE memory, 256-byte aligned, rannc_dp_form_stage_scratch_bytes(in) bytes
 *   out          HOST result; out->feasible == 0 means INFEASIBLE (not an error)
 *   stage_end, replicas  HOST int32[plan_stride]: the plan as in rannc_dp_traceback (replicas
 *                before the factor R: stage u runs on replicas[u] * R devices in total)
 * Errors: INVALID_ARG (bad sizes, negative inputs, backward times that do not match the handle's
 * RANNC_DP_FLAG_SPLIT_OBJECTIVE, devices_per_node * n_max > 64,
 * plan_stride < min(devices_per_node * n_max, n_blocks)), OVERFLOW (scaled inputs or their sums
 * exceed the handle's value width or 2^62), LIMIT_EXCEEDED (more searches, blocks, devices or
 * stages than the handle was created for; checked before anything is copied),
 * WORKSPACE_TOO_SMALL (scratch_bytes, or the handle's workspace for this batch). */
typedef struct {
  int32_t n_blocks;                   /* N >= 1 */
  int32_t n_nodes;                    /* >= 1; only n = 1, 2, 4, ... <= n_nodes are visited */
  int32_t devices_per_node;           /* D_node >= 1 */
  int32_t reserved;                   /* must be 0 */
  int64_t batch_size;                 /* BS >= 1 samples per iteration */
  int64_t mem_capacity;               /* M bytes */
  const int64_t *time_per_sample_ns;  /* HOST [N] fwd+bwd time of a block for one sample */
  const int64_t *act_bytes_per_sample;/* HOST [N] transient bytes of a block for one sample */
  const int64_t *param_bytes;         /* HOST [N] persistent per-replica bytes */
  const int64_t *cut_bytes_per_sample;/* HOST [N] or NULL: bytes crossing the cut after a block for one
                                         sample (communication term of rannc_dp_batch_t; grows
                                         with the samples of a microbatch like the times) */
  int64_t bandwidth_bytes_per_us;     /* >= 1 if cut_bytes_per_sample is given, else ignored */
  const int64_t *time_bwd_per_sample_ns; /* HOST [N]: required on a handle with
                                         RANNC_DP_FLAG_SPLIT_OBJECTIVE (every form_stage_dp call is then
                                         Algorithm 1 as printed, time_per_sample_ns the forward time,
                                         stage_time_ns the sum of the two maxima), NULL otherwise */
} rannc_dp_form_stage_in_t;

typedef struct {
  int32_t feasible;        /* 0: INFEASIBLE, every other field 0 and the plan -1 */
  int32_t n;               /* nodes per pipeline replica */
  int32_t devices;         /* D = devices_per_node * n */
  int32_t replica_factor;  /* R = n_nodes / n */
  int32_t n_stages;        /* S */
  int32_t n_microbatches;  /* MB */
  int64_t stage_time_ns;   /* V[S][N][D]: slowest stage, one microbatch */
  int64_t est_iter_ns;     /* (MB + S - 1) * stage_time_ns, saturating */
} rannc_dp_form_stage_out_t;

RANNC_DP_API int32_t rannc_dp_form_stage_problems(const rannc_dp_form_stage_in_t *in); /* 0 if invalid */
RANNC_DP_API size_t rannc_dp_form_stage_scratch_bytes(const rannc_dp_form_stage_in_t *in);
RANNC_DP_API int rannc_dp_form_stage(rannc_dp_t *h, const rannc_dp_form_stage_in_t *in, void *hip_stream,
                                     void *d_scratch, size_t scratch_bytes,
                                     rannc_dp_form_stage_out_t *out, int32_t *stage_end,
                                     int32_t *replicas, int32_t plan_stride);

/* Compaction step of the block-level phase (Sec. III-B: the step that hands k blocks to the
 * stage-level search), on a chain of G groups in topological order, each with a computation time,
 * persistent and transient bytes.  A walk: the groups as they stand are listed by ascending
 * computation time (equal times by position); a listed group that is still as listed (neither
 * absorbed nor grown since) picks the neighbour in the chain whose current computation time is
 * smaller (equal: the left one) and merges with it if the union fits the device memory (all
 * persistent + all transient bytes <= mem_capacity; the other neighbour is not tried); a union is
 * not listed again in the walk that formed it; everything stops as soon as k groups are left.
 * Sec. III-B repeats this "until |G| = k" and does not say what happens when the list runs out
 * first: with max_walks = 0 the groups are then listed again by their current times and walked
 * again, until k groups are left or a walk merges nothing (every chosen union then exceeds the
 * memory, so further walks could not differ); max_walks = n > 0 stops after n walks (1: a single
 * walk over the initial list, which at most about halves the number of groups).
 * Enqueued on the stream, no synchronisation, no handle.
 *   d_time_ns, d_param_bytes, d_act_bytes  DEVICE int64[G], >= 0, totals below 2^62
 *   d_workspace   DEVICE, 256-byte aligned, rannc_dp_compact_workspace_bytes(G) bytes
 *   d_n_blocks    DEVICE int32[1]: number n of resulting blocks (>= min(k, G)); 0 on bad inputs
 *   d_block_end   DEVICE int32[G]: block u covers the groups d_block_end[u-1]+1 .. d_block_end[u]
 *                 (1-based, d_block_end[n-1] = G); entries from n on are not written
 *   d_time_out, d_param_out, d_act_out  DEVICE int64[G]: summed time and bytes of the n blocks, in
 *                 the form rannc_dp_batch_t takes as block arrays
 *   d_status      DEVICE int32[1]: RANNC_DP_PROBLEM_OK / _NEGATIVE_INPUT / _SUM_OVERFLOW
 * G <= 65535.  Errors: INVALID_ARG (also max_walks < 0), WORKSPACE_TOO_SMALL, HIP_ERROR. */
RANNC_DP_API size_t rannc_dp_compact_workspace_bytes(int32_t n_groups); /* 0 if n_groups is out of range */
RANNC_DP_API int rannc_dp_compact(void *hip_stream, int32_t n_groups, int32_t k, int32_t max_walks,
                                  int64_t mem_capacity, const int64_t *d_time_ns, const int64_t *d_param_bytes,
                                  const int64_t *d_act_bytes, void *d_workspace, size_t workspace_bytes,
                                  int32_t *d_n_blocks, int32_t *d_block_end, int64_t *d_time_out,
                                  int64_t *d_param_out, int64_t *d_act_out, int32_t *d_status);

/* rannc_dp_compact for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernel, same
 * arguments and results, but its workspace is a fixed array inside the library's device image
 * (rannc_dp_compact_workspace_bytes(RANNC_DP_COMPACT_STATIC_MAX_GROUPS) = 786 432 bytes per device,
 * held until the process ends).  The call allocates nothing on host or device; its first use on a
 * device looks the array's address up once.  n_groups > RANNC_DP_COMPACT_STATIC_MAX_GROUPS returns
 * RANNC_DP_LIMIT_EXCEEDED.  All calls on one device share the array: two calls that may overlap on
 * the device (different streams, no ordering between them) race; calls on one stream, or ordered by
 * events, are safe.  The array keeps the previous call's contents; the kernel writes every word
 * before reading it, so nothing is cleared. */
#define RANNC_DP_COMPACT_STATIC_MAX_GROUPS 16384
RANNC_DP_API int rannc_dp_compact_static(void *hip_stream, int32_t n_groups, int32_t k, int32_t max_walks,
                                         int64_t mem_capacity, const int64_t *d_time_ns,
                                         const int64_t *d_param_bytes, const int64_t *d_act_bytes,
                                         int32_t *d_n_blocks, int32_t *d_block_end, int64_t *d_time_out,
                                         int64_t *d_param_out, int64_t *d_act_out, int32_t *d_status);

/* Export one table of one problem of the last solve in a layout-independent form, for parity
 * checks and inspection (not part of the timed path).  d_dst is DEVICE memory of `bytes`
 * bytes; with D = D_q, N = N_q, L = min(S_q,N_q,D_q):
 *   COST  int64[N(N+1)/2 * D]  entry (j,i,r), 1<=j<=N, 0<=i<j, 1<=r<=D at
 *                              ((j(j-1)/2 + i) * D + (r-1)); INT64_MAX where the stage does not fit
 *   FIT   uint8, same indexing; 1 = fits
 *   V     int64[(L+1)][(N+1)][(D+1)]; INT64_MAX = no plan
 *   ARG_I, ARG_D  int32, shape of V: the (i, d') chosen for the cell, -1 where V is infinite or s = 0
 * Returns RANNC_DP_INVALID_ARG if bytes is not exactly the table's size. */
#define RANNC_DP_TABLE_COST 0
#define RANNC_DP_TABLE_FIT 1
#define RANNC_DP_TABLE_V 2
#define RANNC_DP_TABLE_ARG_I 3
#define RANNC_DP_TABLE_ARG_D 4
/* split objective only: backward stage times (as COST), and per cell the largest forward /
 * backward stage time of the plan behind it (as V) */
#define RANNC_DP_TABLE_COST_BWD 5
#define RANNC_DP_TABLE_MAX_FWD 6
#define RANNC_DP_TABLE_MAX_BWD 7
RANNC_DP_API int rannc_dp_read_table(rannc_dp_t *h, int which, int32_t problem, void *d_dst, size_t bytes,
                        void *hip_stream);

/* Which level kernel the last solve ran for each device-count class (D <= 8, 16, 32, 64) of its batch. */
#define RANNC_DP_KERNEL_NONE 0            /* no search of that class in the batch */
#define RANNC_DP_KERNEL_MERGE_TABLE 1     /* sorted merge, stage times read from their table */
#define RANNC_DP_KERNEL_MERGE_RECOMPUTE 2 /* sorted merge, stage times recomputed */
#define RANNC_DP_KERNEL_ONE_LAUNCH 3      /* whole search in one launch, one workgroup per search */
#define RANNC_DP_KERNEL_SCAN 4            /* literal scan */
#define RANNC_DP_KERNEL_SPLIT 5           /* split objective, packed winners */
#define RANNC_DP_KERNEL_SPLIT_SCAN 6      /* split objective, literal scan */
#define RANNC_DP_KERNEL_ONE_LAUNCH_RECOMPUTE 7 /* one launch per search, stage times recomputed */
typedef struct {
  int32_t n_problems[4];
  int32_t level_kernel[4];  /* RANNC_DP_KERNEL_* */
} rannc_dp_solve_info_t;
/* RANNC_DP_BAD_STATE before the first successful solve. */
RANNC_DP_API int rannc_dp_solve_info(rannc_dp_t *h, rannc_dp_solve_info_t *out);

/* Waits for the handle's own streams, frees host state, events and streams; the workspace remains
 * the caller's.  NULL is allowed. */
RANNC_DP_API void rannc_dp_destroy(rannc_dp_t *h);

/* Static description of a status code; never NULL. */
RANNC_DP_API const char *rannc_dp_strerror(int status);

/* Kernel timing of the last solve, in milliseconds, measured with HIP events recorded on the
 * solve's stream around (0) the prefix-sum and table-build kernels, (1) all DP level kernels,
 * (2) the final selection.  Events are recorded only when enabled (non-zero) before solve;
 * get blocks until the last recorded event has completed.  out_ms has 3 entries. */
RANNC_DP_API int rannc_dp_set_timing(rannc_dp_t *h, int enabled);
RANNC_DP_API int rannc_dp_get_timing(rannc_dp_t *h, float *out_ms, int32_t *out_level_launches);

#ifdef __cplusplus
}
#endif
#endif /* RANNC_DP_H_ */
