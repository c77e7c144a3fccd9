/*
 * libkvsched -- batched evaluation of candidate schedules for LLM serving under a KV-cache
 * budget (offline, backlogged model of "LLM Serving Optimization with Variable Prefill and
 * Decode Lengths").  C ABI; every entry point runs hand-written HIP kernels for gfx950 on
 * one GPU.  There is no CPU fallback.
 *
 * Model (Section 2, "Batch Processing and Memory Constraint", with the timing of the
 * integer program Optimal-IP in Section 6): rounds are 0,1,2,...; request i has prompt
 * length s_i and decode length o_i; started at round p it holds s_i + j tokens of KV memory
 * at round p + j (j = 1..o_i) and completes at round c_i = p + o_i; the memory held by all
 * running requests may not exceed M at any round.  All n requests are present at round 0
 * (kvsched_online alone takes arrival rounds).
 *
 * Conventions common to all entry points
 *   - Every array argument is a DEVICE pointer owned by the caller (for instance the
 *     data_ptr() of a torch tensor on the context's device), contiguous, row-major.
 *     The library neither frees nor keeps them after the call's work has run.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are
 *     enqueued on it; outputs are valid once the caller has synchronised the stream.  A call
 *     blocks the host only for the short length scan described at kvsched_set_o_max().
 *   - Return value: KVSCHED_OK or a negative KVSCHED_E* code for errors the host can see
 *     (null pointers, sizes, unsupported ranges, HIP runtime failures).  Faults only the
 *     device can see (a length < 1, s_i + o_i > M, an order row that is not a permutation,
 *     a malformed move) set bits in a device status word, readable with
 *     kvsched_device_status(); the affected candidates get tel = -1.
 *   - int32 for lengths, ids, orders, rounds; int64 for M and total latencies.
 *   - A context is bound to one device and may be used by one host thread at a time; its calls
 *     share the context's scratch memory, so work of two calls on one context must not overlap on
 *     the GPU (same stream, or ordered by events).  Independent work takes a context each.
 */
#ifndef KVSCHED_H
#define KVSCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvsched_ctx kvsched_ctx;

#define KVSCHED_OK 0
#define KVSCHED_EINVAL (-1)  /* null pointer, non-positive size, bad enum value            */
#define KVSCHED_ERANGE (-2)  /* a size beyond what the kernels support (see each call)     */
#define KVSCHED_EHIP (-3)    /* a HIP runtime call failed                                  */
#define KVSCHED_ENOMEM (-4)  /* device scratch could not be allocated                      */

/* bits of the device status word */
#define KVSCHED_DEV_BAD_LENGTH 1 /* some s_i < 1, o_i < 1 or s_i + o_i > M (Theorem 1's premise) */
#define KVSCHED_DEV_BAD_ORDER 2  /* an order row is not a permutation of 0..n-1               */
#define KVSCHED_DEV_BAD_MOVE 4   /* a move has type outside {0,1} or a position outside [0,n) */
#define KVSCHED_DEV_O_MAX 8      /* a decode length exceeds the bound given to kvsched_set_o_max() */
#define KVSCHED_DEV_BAD_ARRIVAL 16 /* kvsched_online: an arrival round is negative or out of order   */
#define KVSCHED_DEV_BACKLOG 32     /* kvsched_online: more requests wait than the caller's backlog_cap   */
#define KVSCHED_DEV_BAD_STREAM 64  /* kvsched_online: a stream descriptor is malformed or out of range */
#define KVSCHED_DEV_ROUND_LIMIT 128 /* kvsched_simulate_predicted: a timeline passed 2^26 rounds          */

#define KVSCHED_MOVE_SWAP 0   /* exchange the entries at positions i and j                  */
#define KVSCHED_MOVE_INSERT 1 /* take the entry at position i out, put it back at position j */

#define KVSCHED_TIE_LARGER 0  /* equal F: the larger batch (Section 4: minimise (F, -|X|))   */
#define KVSCHED_TIE_SMALLER 1 /* equal F: the smaller batch (first minimum scanning k upward) */

/* Phase-1 batch feasibility */
#define KVSCHED_FEAS_SUM_OF_PEAKS 0 /* a batch is feasible if sum (s_i + o_i) <= M (Algorithms 2-4)  */
#define KVSCHED_FEAS_PROFILE 1      /* ... if, all started together, memory <= M at every completion
                                       time (the constraint of Algorithm 1's Phase 1)              */

/* largest supported decode length (slots of the per-timeline future-memory ring) */
#define KVSCHED_MAX_O 16384

/* Phase-1 batch solvers selectable in kvsched_phase1_G */
#define KVSCHED_SOLVER_SORTED_PREFIX 0 /* as kvsched_sortedF    */
#define KVSCHED_SOLVER_LOCAL_SWAP 1    /* as kvsched_local_swap */
#define KVSCHED_SOLVER_EXACT_DP 2      /* as kvsched_exact_dp   */

/* planners of kvsched_online: what a refresh of the cached priority order does with the backlog */
#define KVSCHED_PLANNER_ARRIVAL 0         /* arrival order (id): FCFS                                   */
#define KVSCHED_PLANNER_SHORTEST_DECODE 1 /* ascending (o_i, i): shortest decode first, MC-SF           */
#define KVSCHED_PLANNER_FOOTPRINT 2       /* ascending (s_i + o_i, o_i, i): the paper's fallback order  */
#define KVSCHED_PLANNER_SORTED_F 3        /* Sorted-F-Online: F-metric batches on a look-ahead window   */
#define KVSCHED_ONLINE_MAX_BACKLOG 4096   /* largest backlog_cap                                        */
#define KVSCHED_ONLINE_MAX_WINDOW 1024    /* largest look-ahead window                                  */
#define KVSCHED_ONLINE_MAX_O 8192         /* longest decode length kvsched_online accepts               */
#define KVSCHED_EXACT_MAX_N 4096    /* most requests kvsched_exact_dp accepts                      */

/* Create / destroy a context on HIP device `device_id`.  The context owns a few KB of device
 * and pinned host scratch plus buffers that grow with the largest n / K seen. */
int kvsched_create(kvsched_ctx **out, int device_id);
void kvsched_destroy(kvsched_ctx *ctx);

/* The context's scratch buffer grows when a call needs more than any call before it, and growing
 * means waiting for the device, freeing and allocating.  A caller that wants none of that inside
 * its loop reserves once, for the largest call it will make: kvsched_simulate with up to `rows`
 * rows, kvsched_best_neighbor / kvsched_horizon_step with up to `moves` moves, and the Phase-1
 * calls (kvsched_sortedF, kvsched_local_swap, kvsched_phase1_G with those solvers), all on up to
 * `n` positions (0 rows / moves: that call is not planned).  Calls within these sizes then never
 * allocate.  (kvsched_exact_dp sizes its tables from the data and kvsched_online from the number
 * of streams: not covered.)  ENOMEM if the device cannot provide the buffer. */
int kvsched_reserve(kvsched_ctx *ctx, int32_t rows, int32_t n, int32_t moves);

/* Static description of a return code. */
const char *kvsched_strerror(int status);

/* The kernels size their future-memory ring from the largest decode length.  By default
 * every call first scans o[] on the device and waits for that one number (the only host
 * synchronisation a call makes).  A caller that knows an upper bound on o_i can set it here
 * (1..KVSCHED_MAX_O) to make calls fully asynchronous; 0 restores the scan.  A length above
 * the bound is reported as KVSCHED_DEV_O_MAX and the affected candidates get tel = -1. */
int kvsched_set_o_max(kvsched_ctx *ctx, int32_t o_max_bound);

/* Optional kernel timing.  With `on` != 0 every later kvsched_simulate / kvsched_best_neighbor /
 * kvsched_horizon_step call records a pair of HIP events on the caller's stream around the launch
 * (two launches when rows are resumed in two) that runs its candidates' timelines;
 * kvsched_last_timeline_ms() waits for the second event and returns that duration in milliseconds
 * (EINVAL if timing is off or no call was made).  Outside the bracket: the one-wavefront launch
 * that places a prefix common to all candidates, and kvsched_horizon_step's timeline of the
 * chosen order. */
int kvsched_enable_timing(kvsched_ctx *ctx, int on);
int kvsched_last_timeline_ms(kvsched_ctx *ctx, float *ms_out);

/* Wait for `stream` and return (in *status_out) the device status word of the last call
 * made on this context: an OR of KVSCHED_DEV_* bits, 0 when the data was well-formed. */
int kvsched_device_status(kvsched_ctx *ctx, void *stream, int32_t *status_out);

/*
 * Phase 2 of Algorithm 1 ("Scheduling Execution") for C candidate priority orders at once.
 * Each row of `orders` is turned into a continuous-batching timeline: at every round the
 * pending requests are admitted in row order for as long as the memory check of Eq. (1)
 * (peak over all future rounds) holds, stopping at the first request that does not fit.
 *
 *   orders          [C][n] int32, each row a permutation of 0..n-1
 *   s, o            [n]    int32, 1 <= s_i, 1 <= o_i <= KVSCHED_MAX_O, s_i + o_i <= M
 *   M               KV budget, 1 <= M < 2^30
 *   tel_out         [C]    int64: total end-to-end latency sum_i c_i of each row (Section 2,
 *                   "Objective"), or -1 for a faulty row
 *   completion_out  [C][n] int32 or NULL: c_i, indexed by REQUEST ID (not by position)
 *   common_prefix   hint: the first common_prefix positions are identical in all rows
 *                   (0 = no hint).  Never changes results; a wrong hint is detected and
 *                   reported as KVSCHED_DEV_BAD_ORDER.
 * Rows that repeat row 0 on their leading positions (local-search neighbours of a base order
 * passed as row 0) need not be placed from the start: with enough rows and positions (see
 * kvsched_set_resume_min_rows) and no declared prefix, row 0's timeline state is saved every 64
 * positions and every row that shares at least 64 leading positions with row 0 starts from the
 * last such state it shares (see kvsched_set_resume_one_launch for how the states are handed
 * over).  Such a row may also stop before its end: if it differs from row 0 only at positions
 * i..j (the same requests in another order) and row 0 starts the requests of positions i-1..j in
 * one round (round 0 for i = 0), the row starts them in that round too and its timeline is row 0's
 * from position j+1 on (Algorithm 1, Phase 2: admission in order, Eq. (1) holds for every part of
 * a set it holds for); what row 0 places behind the next 64-position boundary is then taken from
 * row 0.  Results are the same; kvsched_simulate_resume_positions() and
 * kvsched_simulate_stop_positions() tell which positions each row placed itself.
 * ERANGE: n * (ring size) >= 2^31 (round counters are int32), M >= 2^30, o_max bound too large.
 */
int kvsched_simulate(kvsched_ctx *ctx, const int32_t *orders, int32_t C, int32_t n,
                     const int32_t *s, const int32_t *o, int64_t M, int64_t *tel_out,
                     int32_t *completion_out, int32_t common_prefix, void *stream);

/* Number of rows from which kvsched_simulate resumes rows from saved states of row 0.  Default
 * KVSCHED_RESUME_AUTO: when the plan and the wait for row 0 are likely to cost less than the
 * skipped positions save (at least 4096 rows, 385 positions and 8 million positions in all; 16384 rows
 * when the states are handed over between two launches); 0 = never; rows > 0 = whenever there are
 * that many rows (and more than 128 positions). */
#define KVSCHED_RESUME_AUTO (-1)
int kvsched_set_resume_min_rows(kvsched_ctx *ctx, int32_t rows);

/* How the resumed rows get row 0's saved states.  wait_polls > 0 (default 4096): all rows run in
 * one launch, row 0's wavefront reports each state once the whole device can read it, a row polls
 * for the state it needs about every 3 microseconds for as long as row 0 keeps reporting progress
 * (it gives up after wait_polls polls without any) and otherwise starts from the latest state that
 * is there (or from its first position).  wait_polls == 0: two launches, the quarter of the rows that
 * shares least with row 0 (at most 4096) beside row 0 in the first, the others in the second.  Results
 * are the same in every case.  EINVAL: wait_polls < 0. */
int kvsched_set_resume_one_launch(kvsched_ctx *ctx, int32_t wait_polls);

/*
 * Phase 2 under predicted decode lengths (Section 5, "Handling Prediction Uncertainty via Adaptive
 * Output Length Refinement"; appendix algorithm "Sorted-F + A_min") for C candidate orders at once.
 * The scheduler does not see o_i: it holds a running estimate e_i, started from est0_i (the lower
 * bound of the predicted interval for A_min, the upper bound for the conservative A_max, o_i itself
 * for exact predictions), and at every round t
 *   1. a running request that has produced a = t - p tokens leaves if a = o_i (c_i = t); otherwise
 *      it needs at least one more token: e_i <- max(e_i, a + 1);
 *   2. waiting requests are started in the row's sequence while memory, with every running request
 *      j assumed to hold s_j + (tq - p_j) at rounds tq = p_j + 1 .. p_j + e_j and nothing afterwards,
 *      stays <= M at every future round; the first that does not fit ends the round's admissions;
 *   3. while that projection exceeds M, the running request of least (e_i, i) is stopped: it loses
 *      what it has produced, keeps e_i, and waits again at its own place of the row.
 * With est0 = o this is kvsched_simulate.  (The paper's pseudo-code counts rounds from 1 and writes
 * the update as max(e_i, t - p_i); with rounds from 0 that is a + 1.)
 *
 *   orders          [C][n] int32 permutations, n <= 65535 and 16 n + 4 H <= 160 KB with H the power
 *                   of two >= every o_i and est0_i
 *   est0            [E][n] int32 by request id, 1 <= est0_i, s_i + est0_i <= M; E = 1 (one
 *                   prediction for all rows) or E = C (row c is run under prediction c)
 *   tel_out         [C] int64: sum of completion rounds, -1 for a faulty row
 *   completion_out  [C][n] int32 by request id, or NULL
 *   evictions_out   [C] int32 or NULL: times a request was stopped in row c
 * The largest estimate is read back from the device (one host synchronisation) unless
 * kvsched_set_o_max() gave a bound, which then covers estimates as well.
 */
int kvsched_simulate_predicted(kvsched_ctx *ctx, const int32_t *orders, int32_t C, int32_t n, const int32_t *s,
                               const int32_t *o, const int32_t *est0, int32_t E, int64_t M, int64_t *tel_out,
                               int32_t *completion_out, int32_t *evictions_out, void *stream);

/* For accounting of work: resume_pos_out[c] (device, [C] int32) = the position from which row c of
 * the LAST kvsched_simulate call on this context was placed (0 = from its first position; 64 b =
 * resumed from row 0's state after 64 b positions).  C must be that call's C; valid until the next
 * call on the context that is not kvsched_argmin / kvsched_device_status. */
int kvsched_simulate_resume_positions(kvsched_ctx *ctx, int32_t C, int32_t *resume_pos_out, void *stream);

/* Its counterpart: stop_pos_out[c] (device, [C] int32) = the position before which row c of that call
 * stopped placing, its timeline having become row 0's again (n = it placed its last position itself;
 * 0 = it placed nothing: the whole timeline is row 0's).  C and n must be that call's; same validity. */
int kvsched_simulate_stop_positions(kvsched_ctx *ctx, int32_t C, int32_t n, int32_t *stop_pos_out, void *stream);

/* The same for the moves of the LAST kvsched_best_neighbor / kvsched_horizon_step call on this context
 * (not kvsched_best_neighbor_static): stop_pos_out[m] (device, [K] int32) = the position before which the
 * timeline of move m stopped being placed because it had become the base order's again (n = placed to its
 * end; 0 = not placed at all: the move only reorders requests the base order starts in one round, or
 * changes nothing).  K and n must be that call's; same validity. */
int kvsched_neighbor_stop_positions(kvsched_ctx *ctx, int32_t K, int32_t n, int32_t *stop_pos_out, void *stream);

/*
 * Phase 1 of Algorithm 1 ("Batch Construction") with the batch chosen among the feasible
 * prefixes of the remaining requests sorted by (s_i + o_i, o_i, i): for every feasible prefix
 * length k, F(k) = sum_{first k} o_i / k^2 (Section 4); the batch is the prefix of least F (ties
 * per `tie_rule`), emitted in nondecreasing o_i (ties by id); repeat on what remains.  F is
 * compared in exact integers; reported as one IEEE double division.
 *
 *   feas_mode        KVSCHED_FEAS_SUM_OF_PEAKS: prefix k is feasible if sum_{first k}(s_i + o_i) <= M;
 *                    KVSCHED_FEAS_PROFILE: if, all k started together, the memory at every
 *                    completion time o_j, sum over {i: o_i >= o_j} of (s_i + o_j), is <= M
 *                    (the constraint of Algorithm 1's Phase 1).  Both are monotone in k.
 *   order_out        [n] int32: the Sorted-F priority order
 *   batch_end_out    [n] int32: batch_end_out[b] = number of requests in batches 0..b; only
 *                    the first *num_batches_out entries are written
 *   F_out            [n] double: F of batch b; same extent
 *   num_batches_out  [1] int32
 */
int kvsched_sortedF(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                    int32_t tie_rule, int32_t feas_mode, int32_t *order_out, int32_t *batch_end_out,
                    double *F_out, int32_t *num_batches_out, void *stream);

/*
 * Phase 1 of Algorithm 1 ("Batch Construction") with every batch chosen by Local Swap Search
 * (the appendix algorithm "Local Swap Search"): the remaining requests are sorted by
 * (s_i + o_i, o_i, i); the batch X starts as the greedy fill in that order (sum of s_i + o_i
 * <= M); then, repeatedly, members r_out and non-members r_in are scanned in the sorted order
 * and the first pair with sum(s+o) still <= M after the exchange and a smaller F is exchanged
 * (|X| is unchanged by an exchange, so F falls exactly when o_in < o_out); when a full scan
 * finds no such pair the batch is emitted in nondecreasing o_i (ties by id) and removed.
 *
 *   order_out, batch_end_out, F_out, num_batches_out   as for kvsched_sortedF
 *   swaps_out        [n] int32 or NULL: exchanges made while forming batch b; same extent
 */
int kvsched_local_swap(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                       int32_t *order_out, int32_t *batch_end_out, double *F_out,
                       int32_t *swaps_out, int32_t *num_batches_out, void *stream);

/*
 * Phase 1 of Algorithm 1 ("Batch Construction") with every batch the exact minimiser of
 * (F(X), -|X|) over the feasible subsets of the remaining requests, by Algorithm 2 ("Exact
 * Optimal Request Selection via Dynamic Programming"): dp[k][m] = least sum of o over sets of k
 * requests of load exactly m; requests are offered one by one, a state is replaced only by a
 * strictly smaller value and remembers the set that produced it; the state of least dp/k^2 is
 * chosen (equal F: `tie_rule`, then the smaller load), its set is emitted in nondecreasing o_i
 * (ties by id) and removed; repeat.
 *   feas_mode KVSCHED_FEAS_SUM_OF_PEAKS: load = sum (s_i + o_i) <= M, requests offered in input order
 *             (Algorithm 2 as printed);
 *   feas_mode KVSCHED_FEAS_PROFILE: the memory of X started together, sum over {i: o_i >= o_j} of
 *             (s_i + o_j), is <= M for every j in X (Algorithm 1, Phase 1); requests offered in
 *             order of decreasing o_i (ties by id), load = sum s_i.
 * Cost O(n^2 M) per batch; one host synchronisation per batch.
 *
 *   order_out, batch_end_out, F_out, num_batches_out   as for kvsched_sortedF
 * ERANGE: n > KVSCHED_EXACT_MAX_N, or tables beyond 16 GiB ((k_max + 1) (M + 1) (8 + n / 8) bytes,
 * k_max = the most requests that can share a batch).
 */
int kvsched_exact_dp(kvsched_ctx *ctx, int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                     int32_t feas_mode, int32_t tie_rule, int32_t *order_out, int32_t *batch_end_out,
                     double *F_out, int32_t *num_batches_out, void *stream);

/*
 * Phase 1 of Algorithm 1 under the generalised metric of Section 7 ("Robustness to prefill
 * weighting"), G(X) = sum (alpha s_i + o_i) / |X|^2 with alpha = alpha_num / alpha_den (alpha_num >= 0,
 * alpha_den >= 1; alpha = 0 is the F-metric and gives exactly what the three calls above give).  The
 * effective length alpha s_i + o_i takes the place of o_i in the metric only: batch feasibility, the
 * sort keys (s_i + o_i, o_i, i) and the emission of a batch in nondecreasing o_i keep the true
 * lengths.  Decisions are taken on the integers alpha_num s_i + alpha_den o_i, exactly.
 *
 *   solver      KVSCHED_SOLVER_SORTED_PREFIX / _LOCAL_SWAP (feas_mode must be SUM_OF_PEAKS; tie_rule
 *               unused; an exchange is taken when it lowers the sum of effective lengths) / _EXACT_DP
 *   G_out       [n] double: G of batch b = sum (alpha_num s_i + alpha_den o_i) / (alpha_den |X|^2)
 *   swaps_out   [n] int32 or NULL: exchanges per batch (local swap only)
 *   other arguments as for the solver's own call
 * ERANGE: max(alpha_num, alpha_den) > 65535; for Local Swap Search max(alpha_num, alpha_den) * M >= 2^31,
 * for the exact DP max(alpha_num, alpha_den) * 2 M >= 2^31 (effective lengths are held in int32).
 */
int kvsched_phase1_G(kvsched_ctx *ctx, int32_t solver, int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                     int32_t alpha_num, int32_t alpha_den, int32_t tie_rule, int32_t feas_mode, int32_t *order_out,
                     int32_t *batch_end_out, double *G_out, int32_t *swaps_out, int32_t *num_batches_out, void *stream);

/*
 * Local-search step on a priority order: every move is applied to `base_order` on the fly
 * (no [K][n] matrix is materialised), the resulting order is run through Phase 2 exactly
 * as in kvsched_simulate, and the move of least total latency is returned, the lowest move
 * index among equals.
 *
 *   base_order  [n]    int32 permutation
 *   moves       [K][3] int32 {type, i, j}: KVSCHED_MOVE_SWAP / KVSCHED_MOVE_INSERT on
 *               positions i, j in [0, n); i == j is the identity
 *   tel_out     [K]    int64 or NULL: latency of every neighbour (-1 for a malformed move)
 *   result_out  [3]    int64: {index of the best move or -1 if none is valid, its total
 *               latency, total latency of base_order itself}
 * Work that the neighbours share with the base order is done once: when no move touches a
 * position before p >= 64, those p positions are placed once and every timeline starts from
 * there; otherwise, with enough moves and positions (kvsched_set_resume_min_rows, with the moves
 * counted as rows), the base order's timeline saves its state every 64 positions and a move on
 * positions i, j starts from the last state before min(i, j) (handed over within the launch, see
 * kvsched_set_resume_one_launch).  And a move that only reorders requests which the base order
 * starts in one and the same round (see kvsched_simulate) gives the base order's timeline: behind
 * a common prefix the base order is placed once more through the last position any move touches and
 * such moves are not run at all; a timeline started from a saved state stops at the 64-position
 * boundary behind max(i, j) once the base order's timeline has got there.  Results are the same;
 * kvsched_neighbor_stop_positions() tells which moves were cut short.
 */
int kvsched_best_neighbor(kvsched_ctx *ctx, const int32_t *base_order, int32_t n,
                          const int32_t *moves, int32_t K, const int32_t *s, const int32_t *o,
                          int64_t M, int64_t *tel_out, int64_t *result_out, void *stream);

/*
 * kvsched_best_neighbor for callers that cannot allocate device memory while they run: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and
 * results; what differs:
 *   - its working memory (latencies of the K + 1 timelines, the plan and the saved states for
 *     resuming) is a fixed array of KVSCHED_STATIC_SCRATCH_MIB MiB in the library's device image (one
 *     copy on every GPU the library is used on, held until the process ends; its address on the
 *     context's device is looked up once, in kvsched_create).  The call allocates and frees nothing
 *     and never waits for the device;
 *   - o_max_bound (1..KVSCHED_MAX_O) is the caller's bound on the decode lengths, as for
 *     kvsched_set_o_max (a longer one is reported as KVSCHED_DEV_O_MAX, tel = -1), in place of the
 *     length scan's read-back;
 *   - ERANGE when the working memory needed, about 24 (K + 1) + 4 n + (768 + 256 R) floor((n - 1) / 64) +
 *     64 KiB bytes with R = 9 / 33 / 65 / 129 / 225 for o_max_bound up to 512 / 2048 / 4096 / 8192 /
 *     14336, exceeds the array (K = 65536 moves with o_max_bound <= 4096 fit up to n = 16384
 *     positions), or the context's device number is 64 or more.
 * Every call on a GPU uses that GPU's one array, whatever the context: two such calls whose work
 * overlaps on one GPU race (order them on one stream or by events).  Nothing in the array needs to
 * be zero at entry; it keeps the last call's contents.
 */
#define KVSCHED_STATIC_SCRATCH_MIB 8
int kvsched_best_neighbor_static(kvsched_ctx *ctx, const int32_t *base_order, int32_t n, const int32_t *moves,
                                 int32_t K, const int32_t *s, const int32_t *o, int64_t M, int32_t o_max_bound,
                                 int64_t *tel_out, int64_t *result_out, void *stream);

/*
 * One re-planning step of receding-horizon scheduling (Section 6, "Heuristics under Online
 * Arrival": plan on a look-ahead window of the pending order, admit what the live memory
 * profile allows, plan again), in its offline form with every request present at round 0:
 *   1. kvsched_best_neighbor over `moves` (the caller draws them inside its look-ahead window
 *      and includes an identity move, so the result is never worse than `order` itself);
 *   2. the best move is applied to `order` IN PLACE;
 *   3. the new order is run through Phase 2 (one timeline, completion rounds);
 *   4. T = the round by which min(n, completed_in + complete_every) requests have completed
 *      (that order statistic of the completion rounds); every position started by round T is
 *      committed -- start rounds are nondecreasing along the order, so they form a prefix that
 *      later moves beyond it can no longer influence.
 *
 *   order           [n]    int32 permutation, updated in place
 *   moves, K, tel_out      as for kvsched_best_neighbor
 *   completed_in    requests completed at the previous step's T (0 at the start)
 *   complete_every  >= 1: completions to wait for before re-planning
 *   completion_out  [n]    int32 or NULL: completion rounds of the new order, by request id
 *   result_out      [6]    int64: {best move, its total latency, latency of the order before
 *                   the move, committed positions, requests completed by T, T}
 *
 * Between steps the context keeps the timeline state behind the positions that no move of the last
 * step touched (with copies of that part of the order and of s and o, in a buffer of its own of
 * about 16 n bytes + 60 KB): the next step places only what lies between there and its own moves.
 * The copies are compared with `order`, s and o on the device at every step; when the caller has
 * changed any of them (or n, M, or moved the window back) the step starts from position 0 as if
 * nothing had been kept.  Results never depend on it.
 */
int kvsched_horizon_step(kvsched_ctx *ctx, int32_t *order, int32_t n, const int32_t *moves, int32_t K,
                         const int32_t *s, const int32_t *o, int64_t M, int64_t completed_in,
                         int32_t complete_every, int64_t *tel_out, int32_t *completion_out,
                         int64_t *result_out, void *stream);

/*
 * Scheduling under online arrivals (Section 6, "Heuristics under Online Arrival"; the policies of
 * Section 7, "Experiment under Online Poisson Arrivals") for B independent request streams at once.
 * Request i of a stream becomes known at round a_i.  Iteration t = 0, 1, 2, ... of a stream:
 *   1. requests with a_i <= t join the backlog (arrived, not started) and the END of the cached
 *      priority list, in arrival order;
 *   2. if the backlog is not empty and a refresh is due, the planner re-orders the whole backlog
 *      into a new cached list.  Due: the entries placed by the last refresh are used up (also:
 *      never planned), or `period` iterations have passed since it, or refresh_den > 0 and
 *      (entries that arrived since and still wait) * refresh_den >= refresh_num * (backlog size at
 *      the last refresh) -- the paper uses period 10 and 1/2;
 *   3. list entries are admitted from the front while the memory check of Eq. (1) holds beside the
 *      running requests, stopping at the first that does not fit (as kvsched_simulate does).
 * Planner KVSCHED_PLANNER_SORTED_F sorts the backlog by (s_i + o_i, o_i, i), re-orders the first
 * min(window, backlog) entries by Phase 1 of Algorithm 1 with Local Swap Search batches over those
 * entries alone (as kvsched_local_swap, budget M) and leaves the rest behind them in that
 * fallback order (the paper: window 300).  The other planners sort the backlog by their key.
 *
 *   streams         [B][8] int32: {first request, number of requests, planner, period >= 1,
 *                   window in [0, KVSCHED_ONLINE_MAX_WINDOW], refresh_num >= 0, refresh_den >= 0,
 *                   first output slot}.  Streams may share requests (same arrivals under several
 *                   policies); their output ranges must not overlap.
 *   a, s, o         [N] int32: arrival round (>= 0, nondecreasing within a stream), prompt and
 *                   decode length (o_i <= KVSCHED_ONLINE_MAX_O, s_i + o_i <= M)
 *   backlog_cap     1..KVSCHED_ONLINE_MAX_BACKLOG: the most requests of one stream that may wait at
 *                   the same time; a stream that exceeds it is faulted (KVSCHED_DEV_BACKLOG).  The
 *                   per-stream state lives in LDS and is sized from this bound and the longest
 *                   decode length (size classes 512 / 1024 / 4096 waiting requests): the smaller
 *                   the bound, the more streams run side by side.
 *   completion_out  [out_len] int32: completion round c_i of request k of stream b at
 *                   [first output slot of b + k]
 *   stats_out       [B][4] int64: {sum of c_i - a_i, refreshes, last completion round, largest
 *                   backlog}; all -1 for a stream that hit a device-visible fault
 *                   (KVSCHED_DEV_BAD_LENGTH / _O_MAX / _BAD_ARRIVAL / _BACKLOG / _BAD_STREAM).
 * ERANGE: a decode length above KVSCHED_ONLINE_MAX_O (from the length scan or kvsched_set_o_max).
 */
int kvsched_online(kvsched_ctx *ctx, int32_t B, const int32_t *streams, int32_t N, const int32_t *a,
                   const int32_t *s, const int32_t *o, int64_t M, int32_t backlog_cap, int32_t *completion_out,
                   int32_t out_len, int64_t *stats_out, void *stream);

/*
 * Candidate scoring step for explicit order rows (Section 2, "Objective": the score of a
 * candidate is its total end-to-end latency): index of the least non-negative entry of
 * tel[0..C), the lowest index among equals.  Deterministic (fixed reduction order).
 *
 *   tel         [C] int64 as written by kvsched_simulate (-1 marks a faulty row, skipped)
 *   result_out  [2] int64: {index of the best row or -1 if none is valid, its total latency}
 */
int kvsched_argmin(kvsched_ctx *ctx, const int64_t *tel, int32_t C, int64_t *result_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KVSCHED_H */
