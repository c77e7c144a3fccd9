// Kernels of the receding-horizon step (an offline adaptation of the paper's Sorted-F-Online,
// Section 6 "Heuristics under Online Arrival": plan on a look-ahead window of the pending
// order, commit what the timeline admits, plan again).  All requests are present at round 0;
// the committed part of the order is the prefix of positions already admitted.
#include "kvsched_internal.h"

namespace {

// order_out = order with move moves[result[0]] applied (result[0] < 0: unchanged).
__global__ __launch_bounds__(256) void apply_best_move_kernel(const int32_t *order, int32_t n, const int32_t *moves,
                                                              const int64_t *result, int32_t *order_out)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n) return;
    const long long best = result[0];
    int pos = k;
    if (best >= 0) {
        const int ty = moves[3 * best];
        const int i = min(max(moves[3 * best + 1], 0), n - 1);
        const int j = min(max(moves[3 * best + 2], 0), n - 1);
        if (ty == KVSCHED_MOVE_SWAP) {
            pos = (k == i) ? j : ((k == j) ? i : k);
        } else if (i < j) {
            if (k >= i && k <= j) pos = (k == j) ? i : k + 1;
        } else {
            if (k >= j && k <= i) pos = (k == j) ? i : k - 1;
        }
    }
    order_out[k] = order[pos];
}

// One block.  T = round by which min(n, completed_in + complete_every) requests have
// completed (the k-th smallest completion round); result = {positions admitted by T (they form
// a prefix of the order, start rounds being nondecreasing along it), requests completed by
// T, T}.
__global__ __launch_bounds__(1024) void horizon_advance_kernel(const int32_t *order, const int32_t *completion,
                                                              const int32_t *o, int32_t n, long long completed_in,
                                                              int32_t complete_every, int64_t *result_out)
{
    __shared__ int sh_cnt;
    __shared__ int sh_max;
    const int tid = threadIdx.x;
    if (tid == 0) sh_max = 0;
    __syncthreads();
    int mx = 0;
    for (int i = tid; i < n; i += blockDim.x) mx = max(mx, completion[i]);
    atomicMax(&sh_max, mx);
    __syncthreads();
    long long kk = completed_in + complete_every;
    if (kk > n) kk = n;
    if (kk < 1) kk = 1;
    const int k = (int)kk;
    int lo = 0, hi = sh_max;  // smallest T in [lo, hi] with #{c <= T} >= k
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (tid == 0) sh_cnt = 0;
        __syncthreads();
        int c = 0;
        for (int i = tid; i < n; i += blockDim.x) c += completion[i] <= mid;
        atomicAdd(&sh_cnt, c);
        __syncthreads();
        const int total = sh_cnt;
        __syncthreads();
        if (total >= k) hi = mid; else lo = mid + 1;
    }
    const int T = lo;
    if (tid == 0) sh_cnt = 0;
    __syncthreads();
    int done = 0, admitted = 0;
    for (int i = tid; i < n; i += blockDim.x) {
        done += completion[i] <= T;
        const int r = order[i];
        admitted += (completion[r] - o[r]) <= T;
    }
    atomicAdd(&sh_cnt, done);
    __syncthreads();
    const int done_all = sh_cnt;
    __syncthreads();
    if (tid == 0) sh_cnt = 0;
    __syncthreads();
    atomicAdd(&sh_cnt, admitted);
    __syncthreads();
    if (tid == 0) {
        result_out[0] = sh_cnt;
        result_out[1] = done_all;
        result_out[2] = T;
    }
}


// One workgroup.  ok[0] = 1 iff the first old_len entries of the order and all lengths equal their copies;
// afterwards the copies hold order[0 .. new_len), s and o.
__global__ __launch_bounds__(1024) void horizon_verify_kernel(const int32_t *order, const int32_t *s, const int32_t *o,
                                                              int32_t n, int32_t old_len, int32_t new_len,
                                                              int32_t *order_copy, int32_t *s_copy, int32_t *o_copy,
                                                              int32_t *ok)
{
    int same = 1;
    for (int i = threadIdx.x; i < n; i += 1024) {
        const int sv = s[i], ov = o[i];
        same &= (sv == s_copy[i]) & (ov == o_copy[i]);
        s_copy[i] = sv;
        o_copy[i] = ov;
    }
    for (int k = threadIdx.x; k < new_len; k += 1024) {
        const int id = order[k];
        if (k < old_len) same &= id == order_copy[k];
        order_copy[k] = id;
    }
    const int all = __syncthreads_and(same);
    if (threadIdx.x == 0) ok[0] = all ? 1 : 0;
}

__global__ void scatter_prefix_kernel(const int32_t *order, const int32_t *by_position, int32_t len, int32_t n,
                                      int32_t *completion_by_id)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < len) {
        const int id = order[k];
        if (id >= 0 && id < n) completion_by_id[id] = by_position[k];
    }
}

}  // namespace

int kvs_launch_apply_best_move(const int32_t *order, int32_t n, const int32_t *moves, const int64_t *result,
                               int32_t *order_out, hipStream_t st)
{
    hipLaunchKernelGGL(apply_best_move_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, order, n, moves,
                       result, order_out);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_horizon_advance(const int32_t *order, const int32_t *completion, const int32_t *o, int32_t n,
                               int64_t completed_in, int32_t complete_every, int64_t *result_out, hipStream_t st)
{
    hipLaunchKernelGGL(horizon_advance_kernel, dim3(1), dim3(1024), 0, st, order, completion, o, n,
                       (long long)completed_in, complete_every, result_out);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_horizon_verify(const int32_t *order, const int32_t *s, const int32_t *o, int32_t n, int32_t old_len,
                              int32_t new_len, int32_t *order_copy, int32_t *s_copy, int32_t *o_copy, int32_t *ok,
                              hipStream_t st)
{
    hipLaunchKernelGGL(horizon_verify_kernel, dim3(1), dim3(1024), 0, st, order, s, o, n, old_len, new_len, order_copy,
                       s_copy, o_copy, ok);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_scatter_prefix(const int32_t *order, const int32_t *by_position, int32_t len, int32_t n,
                              int32_t *completion_by_id, hipStream_t st)
{
    if (len < 1) return KVSCHED_OK;
    hipLaunchKernelGGL(scatter_prefix_kernel, dim3((unsigned)((len + 255) / 256)), dim3(256), 0, st, order, by_position,
                       len, n, completion_by_id);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
