// Internal declarations shared by the translation units of libkvsched.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kvsched.h"

// Device-side scratch words owned by a context (int32 each).
enum {
    KVS_W_STATUS = 0,  // OR of KVSCHED_DEV_* bits for the call in flight
    KVS_W_OMAX = 1,    // largest decode length found by the length scan
    KVS_W_MINPOS = 2,  // smallest position any move touches (best_neighbor)
    KVS_W_REMAIN = 3,  // exact DP: requests not yet in a batch
    KVS_W_KMAX = 4,    // exact DP: bound on the size of the next batch
    KVS_W_BESTK = 5,   // exact DP: best state of the batch in hand
    KVS_W_BESTM = 6,
    KVS_W_ESTMAX = 7,  // largest initial estimate (kvsched_simulate_predicted)
    KVS_W_MAXPOS = 8,  // largest position any move touches (best_neighbor), -1: none
    KVS_W_COUNT = 16
};

struct kvsched_ctx {
    int device;
    int32_t o_max_bound;   // 0 = scan o[] on every call
    int32_t *d_words;      // [KVS_W_COUNT] device
    int32_t *h_words;      // [KVS_W_COUNT] pinned host mirror
    void *d_scratch;       // grows on demand
    size_t scratch_bytes;
    void *static_scratch;  // this device's address of the library's fixed working array (never freed)
    void *d_tables;        // exact DP: tables and records, grows on demand
    size_t tables_bytes;
    int timing;            // record events around the timeline kernel
    int timed;             // a pair of events has been recorded
    int32_t resume_rows;   // rows of the last kvsched_simulate call if it resumed rows from snapshots, else 0
    int32_t resume_first;  // ... and how many of them (in sorted order) ran from the start
    size_t rejoin_offset;  // ... and where in the scratch buffer the blocks at which rows stopped early are (0: nowhere)
    size_t neighbor_stop_offset;  // the same for the moves of the last kvsched_best_neighbor / kvsched_horizon_step call
    int32_t neighbor_moves;       // ... and how many moves that call had
    int32_t resume_min_rows;  // kvsched_simulate resumes rows from row 0's snapshots from this many rows on
    int32_t resume_wait_polls;  // ... in one launch, a row waiting at most so many polls for its snapshot; 0: in two launches
    hipEvent_t ev0, ev1;
    // kvsched_horizon_step: the state behind the positions no move touched at the last step, with what it was
    // computed from (copies of the order's prefix and of the lengths, compared on the device before use)
    void *d_horizon;          // state | order copy [n] | s copy [n] | o copy [n] | completion rounds by position [n] | flag
    size_t horizon_bytes;
    int32_t hz_n, hz_len, hz_o_bound;  // hz_len = 0: nothing kept
    int64_t hz_M;
};

// How a candidate's order is presented to the timeline kernel.
struct OrderSource {
    const int32_t *orders;  // [C][n] explicit rows, or NULL
    const int32_t *base;    // [n] base order when moves are applied on the fly
    const int32_t *moves;   // [K][3]; candidate K (one past the last move) is the base itself
};

struct SimParams {
    OrderSource src;
    int32_t C;  // number of timelines to run
    int32_t n;
    const int32_t *s;
    const int32_t *o;
    int32_t M;
    int64_t *tel_out;         // [C]
    int32_t *completion_out;  // [C][n] or NULL
    int32_t completion_by_position;  // 1: row entry k = completion of position k (a later pass permutes)
    int32_t *d_words;
    int32_t o_bound;          // lengths above this are reported, not simulated
    // Register kernel only: simulate positions [k_begin, k_end) (k_end == 0: up to n), starting
    // from / leaving behind a saved timeline state of KVS_STATE_HEAD_WORDS + 64 NR int32 words:
    // {b64, t, 62 unused, the 64 lanes' partial sums of completion rounds as int64, then the
    // NR x 64 profile registers}.  t = -1 marks a state nothing may resume from.
    int32_t k_begin = 0;
    int32_t k_end = 0;
    const int32_t *state_in = nullptr;
    int32_t *state_out = nullptr;
    // ... unless *resume_ok == 0 (when set): then from position 0 and an empty timeline after all
    const int32_t *resume_ok = nullptr;
    // Register kernel, explicit rows only: resuming rows from snapshots of row 0.  When cand_list is
    // set, wave w of the launch runs candidate cand_list[w].  Snapshot j (j >= 1) is the timeline
    // state of row 0 after 64 j positions, at snapshots + (j - 1) * snap_stride.  The wave that runs
    // candidate snap_cand (row 0) writes snapshots 1..snap_blocks (word 1 of a snapshot, the round t, is set to -1 by
    // the host beforehand: a snapshot that is never taken poisons whoever resumes from it); a
    // candidate c with resume_block[c] = b > 0 starts from snapshot b at position 64 b.
    // With snap_flags (the progress word in KVS_PROGRESS_WORDS words, zero at launch) both happen in ONE launch: the wave of
    // candidate snap_cand stores there the number of snapshots it has published so far (or ~that number
    // when it stops early), a candidate with b > 0 waits until the word reaches b, as long as the word
    // keeps moving, then takes the latest snapshot that is there and writes the block it really started
    // from back to resume_block[c].
    const int32_t *cand_list = nullptr;
    int32_t *resume_block = nullptr;
    int32_t *snapshots = nullptr;
    int32_t snap_stride = 0;
    int32_t snap_blocks = 0;
    int32_t *snap_flags = nullptr;
    int32_t snap_wait_polls = 0;  // polls (about 3 us each) a candidate waits for its snapshot at most
    int32_t snap_cand = 0;        // the candidate whose wave writes the snapshots (row 0; the base order among moves)
    // Explicit rows resumed from row 0 may also stop early: a row that differs from row 0 at positions
    // diff_first[c] .. diff_last[c] only, and whose timeline is row 0's again behind them, stops at the
    // 64-position boundary b behind diff_last[c] (b <= rejoin_blocks, the boundaries row 0 saves a state at) and
    // writes b to rejoin_block[c] (INT_MAX: placed everything itself; 0: placed nothing); its tel_out is then
    // relative to row 0's and its completion rounds from position 64 b on are row 0's.  The test needs row 0's
    // start rounds by position, which the wave of row 0 stores in start0.
    // With moves the stretch is the move's own (positions min(i, j) .. max(i, j)) and diff_first / diff_last stay
    // unset; the candidate whose timeline the others rejoin is snap_cand, the base order.
    const int32_t *diff_first = nullptr;
    const int32_t *diff_last = nullptr;
    int32_t *rejoin_block = nullptr;
    int32_t *start0 = nullptr;  // (a launch of one timeline that takes no snapshots stores its start rounds here too)
    int32_t rejoin_blocks = 0;
    // Candidates with skip[c] != INT_MAX are not run at all: they are known to stop at block skip[c] (the
    // encoding of rejoin_block; in practice 0, nothing to place); their tel_out is set to 0.
    const int32_t *skip = nullptr;
};
constexpr int KVS_STATE_HEAD_WORDS = 192;
// the progress word of the snapshot hand-over: this many copies, this far apart (SimParams::snap_flags)
constexpr int KVS_PROGRESS_COPIES = 64;
constexpr int KVS_PROGRESS_STRIDE_WORDS = 16;
constexpr int KVS_PROGRESS_WORDS = KVS_PROGRESS_COPIES * KVS_PROGRESS_STRIDE_WORDS;
constexpr size_t KVS_STATE_MAX_WORDS = KVS_STATE_HEAD_WORDS + 225 * 64;

// simulate.hip
int kvs_launch_scan_lengths(const int32_t *s, const int32_t *o, int32_t n, int32_t M, int32_t o_bound,
                            int32_t *d_words, hipStream_t st);
int kvs_launch_simulate(const SimParams &p, int32_t ring_slots, hipStream_t st);
// timeline_reg.hip (decode lengths up to KVS_REG_MAX_O)
constexpr int32_t KVS_REG_MAX_O = 14336;  // 224 rows of 64 rounds, and one more row for the window's offset
int kvs_launch_simulate_reg(const SimParams &p, hipStream_t st);
int32_t kvs_reg_state_words(int32_t o_bound);  // words of one snapshot for this decode bound

int kvs_launch_check_orders(const int32_t *orders, int32_t C, int32_t n, int64_t *tel_out, int32_t *d_words,
                            hipStream_t st);
// horizon.hip: ok = (order[0 .. old_len) and the lengths equal their copies); the copies are then brought up to
// date (order[0 .. new_len), s, o)
int kvs_launch_horizon_verify(const int32_t *order, const int32_t *s, const int32_t *o, int32_t n, int32_t old_len,
                              int32_t new_len, int32_t *order_copy, int32_t *s_copy, int32_t *o_copy, int32_t *ok,
                              hipStream_t st);
// completion_by_id[order[k]] = by_position[k], k < len
int kvs_launch_scatter_prefix(const int32_t *order, const int32_t *by_position, int32_t len, int32_t n,
                              int32_t *completion_by_id, hipStream_t st);
int kvs_launch_check_moves(const int32_t *moves, int32_t K, int32_t n, int64_t *tel_out, int32_t *d_words,
                           hipStream_t st);
int kvs_launch_argmin(const int64_t *tel, int32_t K, int64_t *result_out, int32_t with_base, hipStream_t st);

// exactdp.hip
size_t kvs_exact_dp_list_bytes(int32_t n);
size_t kvs_exact_dp_table_bytes(int32_t r, int32_t kmax, int32_t M);
int kvs_launch_exact_dp_prepare(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t feas_mode,
                                void *lists, int32_t *d_words, int32_t *num_batches_out, hipStream_t st);
// ga, gb: the metric's numerator sums ga s_i + gb o_i (0, 1: the F-metric; else G with alpha = ga / gb)
int kvs_launch_exact_dp_batch(int32_t n, int32_t r, int32_t kmax, const int32_t *s, const int32_t *o, int32_t M,
                              int32_t ga, int32_t gb, int32_t feas_mode, int32_t tie_rule, int32_t nb, void *lists, void *tables,
                              int32_t *batch_end_out, double *F_out, int32_t *d_words, hipStream_t st);
int kvs_exact_dp_small_lg(int32_t n, int32_t kmax_bound, int32_t M);
size_t kvs_exact_dp_small_record_bytes(int32_t n, int32_t kmax_bound, int lg);
int kvs_launch_exact_dp_small(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t ga, int32_t gb,
                              int32_t feas_mode,
                              int32_t tie_rule, int lg, void *lists, void *records, int32_t *order_out,
                              int32_t *batch_end_out, double *F_out, int32_t *num_batches_out, int32_t *d_words,
                              hipStream_t st);
int kvs_launch_exact_dp_emit(int32_t n, int32_t nb, void *lists, int32_t *order_out, int32_t *num_batches_out,
                             hipStream_t st);

// localswap.hip
size_t kvs_local_swap_scratch_bytes(int32_t n);
int kvs_launch_local_swap(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t ga, int32_t gb,
                          int32_t *order_out,
                          int32_t *batch_end_out, double *F_out, int32_t *swaps_out, int32_t *num_batches_out,
                          void *scratch, int32_t *d_words, hipStream_t st);

// sortedf.hip
size_t kvs_sortedF_scratch_bytes(int32_t n);
int kvs_launch_sortedF(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t ga, int32_t gb,
                       int32_t tie_rule, int32_t feas_mode,
                       int32_t *order_out, int32_t *batch_end_out, double *F_out, int32_t *num_batches_out,
                       void *scratch, int32_t *d_words, hipStream_t st);

// permute.hip: rows of completion rounds from position order to request-id order, in place; rows
// that are no permutation get tel = -1 and KVSCHED_DEV_BAD_ORDER (what kvs_launch_check_orders does)
constexpr int32_t KVS_PERMUTE_MAX_N = 15872;  // one row and its bitmap must fit in 64 KB of LDS
// resume_block / row0 (or NULL): row c placed only the positions from 64 resume_block[c] on; the
// completion rounds before them are row0[k], row 0's in position order
int kvs_launch_permute_rows(const int32_t *orders, int32_t C, int32_t n, int32_t *completion, int64_t *tel_out,
                            int32_t *d_words, const int32_t *resume_block, const int32_t *row0,
                            const int32_t *rejoin_block, hipStream_t st);

// horizon.hip
int kvs_launch_apply_best_move(const int32_t *order, int32_t n, const int32_t *moves, const int64_t *result,
                               int32_t *order_out, hipStream_t st);
int kvs_launch_horizon_advance(const int32_t *order, const int32_t *completion, const int32_t *o, int32_t n,
                               int64_t completed_in, int32_t complete_every, int64_t *result_out, hipStream_t st);

// online.hip
int kvs_launch_online(int32_t B, const int32_t *streams, int32_t N, const int32_t *a, const int32_t *s,
                      const int32_t *o, int32_t M, int32_t backlog_cap, int32_t ring_slots, int32_t *completion_out,
                      int32_t out_len, int64_t *stats_out, int32_t *order_scratch, int32_t *d_words, hipStream_t st);

// predicted.hip
constexpr size_t KVS_PREDICTED_MAX_LDS = 160 * 1024;  // LDS of one workgroup on gfx950
int kvs_launch_scan_estimates(const int32_t *est, size_t count, int32_t *d_words, hipStream_t st);
size_t kvs_predicted_lds_bytes(int32_t n, int32_t H);
int kvs_launch_predicted(const int32_t *orders, int32_t C, int32_t n, const int32_t *s, const int32_t *o,
                         const int32_t *est0, int32_t E, int32_t M, int32_t H, int32_t round_limit, int64_t *tel_out,
                         int32_t *completion_out, int32_t *evictions_out, int32_t *retry /*[C] scratch*/,
                         uint16_t *est_stopped /*[C][n] scratch*/, int32_t *d_words, hipStream_t st);

// prefix.hip
int kvs_launch_moves_min_position(const int32_t *moves, int32_t K, int32_t n, int32_t *d_words, hipStream_t st);
int kvs_launch_check_prefix(const int32_t *orders, int32_t C, int32_t n, int32_t cp, int64_t *tel_out,
                            int32_t *d_words, hipStream_t st);
int kvs_launch_broadcast_prefix(const int32_t *prefix, int32_t cp, int32_t C, int32_t n, int32_t *completion,
                                hipStream_t st);
// rows resumed from snapshots of row 0 (see SimParams)
int kvs_launch_shared_blocks(const int32_t *orders, int32_t C, int32_t n, int32_t *blocks, int32_t *diff_first,
                             int32_t *diff_last, hipStream_t st);
// tel[c] += tel[base] for the candidates that stopped early (rejoin[c] != INT_MAX), c != base
int kvs_launch_rejoin_finish(const int32_t *rejoin, int32_t C, int32_t base, int64_t *tel, hipStream_t st);
int kvs_launch_stop_positions(const int32_t *rejoin, int32_t C, int32_t n, int32_t *stop_pos_out, hipStream_t st);
// Moves behind a common prefix of `first` positions whose timeline is the base order's: the move only reorders
// requests that the base order starts in one round (start rounds of positions first .. first + count - 1 in
// window_start, that of position first - 1 in word 1 of the prefix's state).  rejoin[m] = 0 for those (and for
// moves that change nothing), INT_MAX for the others and for the base order itself (entry K).
int kvs_launch_mark_noop_moves(const int32_t *moves, int32_t K, int32_t n, int32_t first, int32_t count,
                               const int32_t *window_start, const int32_t *prefix_state, int32_t *rejoin,
                               hipStream_t st);
// flags / nflags: words to clear on the way (the snapshot flags of the launch that follows), or NULL
int kvs_launch_sort_by_blocks(const int32_t *blocks, int32_t C, int32_t first_row, int32_t *tmp, int32_t *sorted,
                              int32_t *flags, int32_t nflags, hipStream_t st);
int kvs_launch_move_blocks(const int32_t *moves, int32_t K, int32_t n, int32_t *blocks, hipStream_t st);
int kvs_launch_copy_row0_prefix(const int32_t *orders, int32_t C, int32_t n, const int32_t *sorted, int32_t first,
                                const int32_t *blocks, int32_t by_position, int32_t *completion, hipStream_t st);
int kvs_launch_mark_snapshots_unusable(int32_t *snapshots, int32_t count, int32_t stride, hipStream_t st);
int kvs_launch_resume_plan(const int32_t *sorted, int32_t C, int32_t first, const int32_t *blocks,
                           int32_t *resume_pos_out, hipStream_t st);
