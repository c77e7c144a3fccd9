// Support kernels for resuming candidate timelines from a shared prefix: every candidate whose
// order agrees with the others on the first cp positions has, after those positions, exactly
// the same timeline state (admission is in order, Algorithm 1's Phase 2), so the prefix is run
// once and its state handed to all of them.
#include "kvsched_internal.h"
#include "phase1_util.h"

#include <limits.h>

namespace {

// Smallest position touched by any well-formed move that changes the order.
__global__ __launch_bounds__(256) void moves_min_position_kernel(const int32_t *moves, int32_t K, int32_t n,
                                                                 int32_t *words)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    int pos = INT_MAX;
    if (m < K) {
        const int ty = moves[3 * (size_t)m], i = moves[3 * (size_t)m + 1], j = moves[3 * (size_t)m + 2];
        const bool ok = (ty == KVSCHED_MOVE_SWAP || ty == KVSCHED_MOVE_INSERT) && i >= 0 && j >= 0 && i < n && j < n;
        if (ok && i != j) pos = min(i, j);
        if (!ok) pos = 0;  // malformed moves are clamped by the timeline kernel: no shared prefix
    }
    int top = -1;
    if (m < K) top = min(max(max(moves[3 * (size_t)m + 1], moves[3 * (size_t)m + 2]), 0), n - 1);  // (as the timeline kernel clamps)
    for (int d = 32; d > 0; d >>= 1) {
        pos = min(pos, __shfl_down(pos, d));
        top = max(top, __shfl_down(top, d));
    }
    if ((threadIdx.x & 63) == 0 && pos != INT_MAX) atomicMin(&words[KVS_W_MINPOS], pos);
    if ((threadIdx.x & 63) == 0 && top >= 0) atomicMax(&words[KVS_W_MAXPOS], top);
}

__global__ __launch_bounds__(256) void mark_noop_moves_kernel(const int32_t *moves, int32_t K, int32_t n, int32_t first,
                                                              int32_t count, const int32_t *window_start,
                                                              const int32_t *prefix_state, int32_t *rejoin)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m > K) return;
    int r = INT_MAX;
    if (m < K) {
        const int i0 = min(max(moves[3 * (size_t)m + 1], 0), n - 1), j0 = min(max(moves[3 * (size_t)m + 2], 0), n - 1);
        const int i = min(i0, j0), j = max(i0, j0);
        if (i == j) {
            r = 0;  // the base order itself
        } else if (i >= first && j < first + count) {
            const int before = i > first ? window_start[i - 1 - first] : (first > 0 ? prefix_state[1] : 0);
            if (window_start[j - first] == before && (i > 0 || before == 0)) r = 0;
        }
    }
    rejoin[m] = r;
}

// Rows that differ from row 0 inside the declared common prefix are faulty.
__global__ __launch_bounds__(256) void check_prefix_kernel(const int32_t *orders, int32_t C, int32_t n, int32_t cp,
                                                           int64_t *tel_out, int32_t *words)
{
    const int row = blockIdx.x;
    const int32_t *a = orders;
    const int32_t *b = orders + (size_t)row * (size_t)n;
    int bad = 0;
    for (int k = threadIdx.x; k < cp; k += blockDim.x) bad |= a[k] != b[k];
    if (__syncthreads_or(bad) && threadIdx.x == 0) {
        tel_out[row] = -1;
        atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_ORDER);
    }
}

// completion[c][k] = prefix[k] for k < cp (completion rounds in position order).
__global__ __launch_bounds__(256) void broadcast_prefix_kernel(const int32_t *prefix, int32_t cp, int32_t n,
                                                               int32_t *completion)
{
    int32_t *dst = completion + (size_t)blockIdx.x * (size_t)n;
    for (int k = threadIdx.x; k < cp; k += blockDim.x) dst[k] = prefix[k];
}

// Rows that agree with row 0 on their leading positions can start from a snapshot of row 0's
// timeline.  blocks[c] = number of leading 64-position blocks on which row c equals row 0, at
// most (n - 1) / 64 so that something is left to place; 0 for row 0 itself, which is the row
// that takes the snapshots.  One wavefront per row, reading stops at the first difference.
// With diff_first / diff_last the first and the last position at which the row differs from row 0
// are found as well (the row is read from its end down to the last difference); both are -1 when
// the row equals row 0 or the first difference was not looked for (it lies in the last block).
__global__ __launch_bounds__(256) void shared_blocks_kernel(const int32_t *orders, int32_t C, int32_t n, int32_t *blocks,
                                                            int32_t *diff_first, int32_t *diff_last)
{
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= C) return;
    const int32_t *a = orders;
    const int32_t *b = orders + (size_t)c * (size_t)n;
    const int cap = (n - 1) >> 6;
    int nb = 0, first = -1, last = -1;
    if (c > 0) {
        // four blocks a turn: the loads of a turn are in flight together, the turns are a dependent chain
        while (nb < cap && first < 0) {
            unsigned long long d[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k = 64 * (nb + u) + lane;  // < n where nb + u < cap: blocks below cap are complete
                d[u] = __builtin_amdgcn_ballot_w64(nb + u < cap && a[k] != b[k]);
            }
            int same = min(4, cap - nb);
#pragma unroll
            for (int u = 3; u >= 0; --u)
                if (d[u] != 0) same = u;
            if (same < 4 && nb + same < cap) first = 64 * (nb + same) + (__ffsll((long long)d[same & 3]) - 1);
            nb += same;
        }
    }
    if (lane == 0) blocks[c] = nb;
    if (!diff_first) return;
    if (first >= 0) {
        // from the end down (block by block: what is read beyond the last difference is read for nothing,
        // and this kernel is bound by what it reads); ends at block nb at the latest
        for (int top = (n - 1) >> 6; top >= nb; --top) {
            const int kk = 64 * top + lane;
            const unsigned long long e = __builtin_amdgcn_ballot_w64(kk < n && a[kk] != b[kk]);
            if (e != 0) {
                last = 64 * top + (63 - __clzll((long long)e));
                break;
            }
        }
    }
    if (lane == 0) {
        diff_first[c] = first;
        diff_last[c] = last;
    }
}

// Rows that stopped where their timeline had become row 0's again (rejoin[c] != INT_MAX) hold their
// sum of completion rounds relative to row 0's (the base order's, among moves): add that (or pass on that it
// could not be scheduled).
__global__ __launch_bounds__(256) void rejoin_finish_kernel(const int32_t *rejoin, int32_t C, int32_t base, int64_t *tel)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C || c == base || rejoin[c] == INT_MAX) return;
    const long long t0 = tel[base];
    tel[c] = t0 < 0 ? -1 : tel[c] + t0;
}

// stop_pos_out[c] = position at which row c stopped placing (n: it placed its last position itself).
__global__ __launch_bounds__(256) void stop_positions_kernel(const int32_t *rejoin, int32_t C, int32_t n, int32_t *stop_pos_out)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    stop_pos_out[c] = (rejoin && rejoin[c] != INT_MAX) ? 64 * rejoin[c] : n;
}

// The same count for the neighbours of a base order given as moves: a swap or an insertion of
// positions i, j leaves the positions before min(i, j) as they are; a move that changes nothing
// shares all of them (up to the cap), a malformed one is taken to share nothing.  blocks[K] = 0 stands
// for the base order itself, the timeline that takes the snapshots.
__global__ __launch_bounds__(256) void move_blocks_kernel(const int32_t *moves, int32_t K, int32_t n, int32_t *blocks)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m > K) return;
    int nb = 0;
    if (m < K) {
        const int ty = moves[3 * (size_t)m], i = moves[3 * (size_t)m + 1], j = moves[3 * (size_t)m + 2];
        const bool ok = (ty == KVSCHED_MOVE_SWAP || ty == KVSCHED_MOVE_INSERT) && i >= 0 && j >= 0 && i < n && j < n;
        const int cap = (n - 1) >> 6;
        if (ok) nb = i == j ? cap : min(min(i, j) >> 6, cap);
    }
    blocks[m] = nb;
}

// Row indices in ascending order of blocks[], row first_row (whose count is 0) first.  One workgroup.  Up to 2047 blocks (any
// order of up to 131072 positions) it is a counting sort in LDS: count, scan, scatter through one
// cursor per value; rows of equal value come in no particular order (the order only decides which
// rows are dispatched first).  Beyond that, stable 8-bit radix passes.
constexpr int KVS_COUNT_SORT_KEYS = 2048;

// Also clears the `nflags` snapshot flags of the launch that follows (saves a launch of its own).
__global__ __launch_bounds__(1024) void sort_by_blocks_kernel(const int32_t *blocks, int32_t C, int32_t first_row,
                                                              int32_t *tmp, int32_t *sorted, int32_t *flags,
                                                              int32_t nflags)
{
    for (int i = threadIdx.x; i < nflags; i += 1024) flags[i] = 0;
    __shared__ RadixLds<1024> L;
    __shared__ int sh_max[16];
    __shared__ int cnt[KVS_COUNT_SORT_KEYS];
    __shared__ int wave_total[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int mx = 0;
    for (int i = tid; i < C; i += 1024) mx = max(mx, blocks[i]);
    for (int d = 32; d > 0; d >>= 1) mx = max(mx, __shfl_xor(mx, d));
    if (lane == 0) sh_max[wave] = mx;
    cnt[tid] = 0;
    cnt[tid + 1024] = 0;
    __syncthreads();
    for (int w = 0; w < 16; ++w) mx = max(mx, sh_max[w]);
    if (mx < KVS_COUNT_SORT_KEYS) {
        for (int i = tid; i < C; i += 1024) atomicAdd(&cnt[blocks[i]], 1);
        __syncthreads();
        // exclusive scan of the 2048 counts, two consecutive ones per thread
        const int c0 = cnt[2 * tid], c1 = cnt[2 * tid + 1];
        int incl = c0 + c1;
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_total[wave] = incl;
        __syncthreads();
        int off = 0;
        for (int w = 0; w < wave; ++w) off += wave_total[w];
        const int start = off + incl - (c0 + c1);
        cnt[2 * tid] = start + (tid == 0 ? 1 : 0);  // (slot 0 is first_row's: its value is 0, the lowest)
        cnt[2 * tid + 1] = start + c0;
        __syncthreads();
        for (int i = tid; i < C; i += 1024) {
            if (i == first_row) sorted[0] = i;
            else sorted[atomicAdd(&cnt[blocks[i]], 1)] = i;
        }
        return;
    }
    auto key = [blocks](int id) { return blocks[id]; };
    // one 8-bit pass per byte of the largest count; the ids start in whichever buffer makes the
    // last pass land in `sorted`
    const int passes = (bits_of(mx) + 7) / 8;
    int *src = (passes & 1) ? tmp : sorted, *dst = (passes & 1) ? sorted : tmp;
    // (stable passes keep the starting order among equal counts: first_row goes in first)
    for (int i = threadIdx.x; i < C; i += 1024) src[i] = i == 0 ? first_row : (i <= first_row ? i - 1 : i);
    __threadfence_block();
    __syncthreads();
    for (int pass = 0; pass < passes; ++pass) {
        radix_pass<1024>(src, dst, C, 8 * pass, key, L);
        __threadfence_block();
        __syncthreads();
        int *sw = src; src = dst; dst = sw;
    }
}

// Completion rounds of the positions a resumed row did not place itself: those of row 0.
// Wave w handles row sorted[first + w].
__global__ __launch_bounds__(256) void copy_row0_prefix_kernel(const int32_t *orders, int32_t C, int32_t n,
                                                               const int32_t *sorted, int32_t first,
                                                               const int32_t *blocks, int32_t by_position,
                                                               int32_t *completion)
{
    const int lane = threadIdx.x & 63;
    const int w = first + blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= C) return;
    const int c = sorted[w];
    const int cp = 64 * blocks[c];
    const int32_t *row = orders + (size_t)c * (size_t)n;
    int32_t *dst = completion + (size_t)c * (size_t)n;
    for (int k = lane; k < cp; k += 64) {
        const int idx = by_position ? k : min(max(row[k], 0), n - 1);
        dst[idx] = completion[idx];
    }
}

// Word 1 of a snapshot is its round t; -1 there makes every timeline that resumes from it report
// tel = -1.  All snapshots start like that; row 0's wave overwrites those it takes.
__global__ __launch_bounds__(256) void mark_snapshots_unusable_kernel(int32_t *snapshots, int32_t count, int32_t stride)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < count) snapshots[(size_t)j * (size_t)stride + 1] = -1;
}

// resume_pos_out[c] = position from which row c was simulated (0: from the start).
__global__ __launch_bounds__(256) void resume_plan_kernel(const int32_t *sorted, int32_t C, int32_t first,
                                                          const int32_t *blocks, int32_t *resume_pos_out)
{
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= C) return;
    const int c = sorted[w];
    resume_pos_out[c] = w >= first ? 64 * blocks[c] : 0;
}

}  // namespace

int kvs_launch_shared_blocks(const int32_t *orders, int32_t C, int32_t n, int32_t *blocks, int32_t *diff_first,
                             int32_t *diff_last, hipStream_t st)
{
    hipLaunchKernelGGL(shared_blocks_kernel, dim3((unsigned)((C + 3) / 4)), dim3(256), 0, st, orders, C, n, blocks,
                       diff_first, diff_first ? diff_last : nullptr);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_rejoin_finish(const int32_t *rejoin, int32_t C, int32_t base, int64_t *tel, hipStream_t st)
{
    hipLaunchKernelGGL(rejoin_finish_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, rejoin, C, base, tel);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_mark_noop_moves(const int32_t *moves, int32_t K, int32_t n, int32_t first, int32_t count,
                               const int32_t *window_start, const int32_t *prefix_state, int32_t *rejoin,
                               hipStream_t st)
{
    hipLaunchKernelGGL(mark_noop_moves_kernel, dim3((unsigned)(K / 256 + 1)), dim3(256), 0, st, moves, K, n, first, count,
                       window_start, prefix_state, rejoin);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_stop_positions(const int32_t *rejoin, int32_t C, int32_t n, int32_t *stop_pos_out, hipStream_t st)
{
    hipLaunchKernelGGL(stop_positions_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, rejoin, C, n,
                       stop_pos_out);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_move_blocks(const int32_t *moves, int32_t K, int32_t n, int32_t *blocks, hipStream_t st)
{
    hipLaunchKernelGGL(move_blocks_kernel, dim3((unsigned)(K / 256 + 1)), dim3(256), 0, st, moves, K, n, blocks);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_sort_by_blocks(const int32_t *blocks, int32_t C, int32_t first_row, int32_t *tmp, int32_t *sorted,
                              int32_t *flags, int32_t nflags, hipStream_t st)
{
    hipLaunchKernelGGL(sort_by_blocks_kernel, dim3(1), dim3(1024), 0, st, blocks, C, first_row, tmp, sorted, flags,
                       flags ? nflags : 0);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_copy_row0_prefix(const int32_t *orders, int32_t C, int32_t n, const int32_t *sorted, int32_t first,
                                const int32_t *blocks, int32_t by_position, int32_t *completion, hipStream_t st)
{
    if (first >= C) return KVSCHED_OK;
    hipLaunchKernelGGL(copy_row0_prefix_kernel, dim3((unsigned)((C - first + 3) / 4)), dim3(256), 0, st, orders, C, n,
                       sorted, first, blocks, by_position, completion);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_mark_snapshots_unusable(int32_t *snapshots, int32_t count, int32_t stride, hipStream_t st)
{
    if (count < 1) return KVSCHED_OK;
    hipLaunchKernelGGL(mark_snapshots_unusable_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                       snapshots, count, stride);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_resume_plan(const int32_t *sorted, int32_t C, int32_t first, const int32_t *blocks,
                           int32_t *resume_pos_out, hipStream_t st)
{
    hipLaunchKernelGGL(resume_plan_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, sorted, C, first, blocks,
                       resume_pos_out);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_moves_min_position(const int32_t *moves, int32_t K, int32_t n, int32_t *d_words, hipStream_t st)
{
    hipLaunchKernelGGL(moves_min_position_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, moves, K, n,
                       d_words);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_check_prefix(const int32_t *orders, int32_t C, int32_t n, int32_t cp, int64_t *tel_out,
                            int32_t *d_words, hipStream_t st)
{
    hipLaunchKernelGGL(check_prefix_kernel, dim3((unsigned)C), dim3(256), 0, st, orders, C, n, cp, tel_out, d_words);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_broadcast_prefix(const int32_t *prefix, int32_t cp, int32_t C, int32_t n, int32_t *completion,
                                hipStream_t st)
{
    hipLaunchKernelGGL(broadcast_prefix_kernel, dim3((unsigned)C), dim3(256), 0, st, prefix, cp, n, completion);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
