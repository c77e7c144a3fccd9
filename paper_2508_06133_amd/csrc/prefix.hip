// Support kernels for resuming candidate timelines from a shared prefix: every candidate whose
// order agrees with the others on the first cp positions has, after those positions, exactly
// the same timeline state (admission is in order, Algorithm 1's Phase 2), so the prefix is run
// once and its state handed to all of them.
#include "kvsched_internal.h"

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
    for (int d = 32; d > 0; d >>= 1) pos = min(pos, __shfl_down(pos, d));
    if ((threadIdx.x & 63) == 0 && pos != INT_MAX) atomicMin(&words[KVS_W_MINPOS], pos);
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

}  // namespace

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
