// Completion rounds from position order to request-id order.
//
// The timeline kernels produce the completion round of every position of a candidate order;
// callers want it per request id (c_i of Section 2, "Objective").  Storing by id from the
// timeline kernel means 4-byte stores scattered over an 8 KB row while thousands of rows are
// in flight: measured HBM write traffic was 9x the payload.  Instead the timeline kernel stores
// by position (256 contiguous bytes per 64 positions) and this kernel permutes each row in
// place: one workgroup per row, the row staged in LDS, read and written coalesced.
#include "kvsched_internal.h"

namespace {

__global__ __launch_bounds__(256) void permute_rows_kernel(const int32_t *orders, int32_t n, int32_t *completion)
{
    extern __shared__ int row_by_id[];
    const int32_t *order = orders + (size_t)blockIdx.x * (size_t)n;
    int32_t *comp = completion + (size_t)blockIdx.x * (size_t)n;
    for (int k = threadIdx.x; k < n; k += blockDim.x) {
        const int r = min(max(order[k], 0), n - 1);  // rows that are no permutation are reported elsewhere
        row_by_id[r] = comp[k];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) comp[i] = row_by_id[i];
}

}  // namespace

int kvs_launch_permute_rows(const int32_t *orders, int32_t C, int32_t n, int32_t *completion, hipStream_t st)
{
    if (n > KVS_PERMUTE_MAX_N) return KVSCHED_ERANGE;
    hipLaunchKernelGGL(permute_rows_kernel, dim3((unsigned)C), dim3(256), sizeof(int32_t) * (size_t)n, st, orders, n,
                       completion);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
