// Completion rounds from position order to request-id order.
//
// The timeline kernels produce the completion round of every position of a candidate order;
// callers want it per request id (c_i of Section 2, "Objective").  Storing by id from the
// timeline kernel means 4-byte stores scattered over an 8 KB row while thousands of rows are
// in flight: measured HBM write traffic was 9x the payload.  Instead the timeline kernel stores
// by position (256 contiguous bytes per 64 positions) and this kernel permutes each row in
// place: one workgroup per row, the row staged in LDS, read and written coalesced.  The same pass
// over the order row checks that it is a permutation of 0..n-1 (a bitmap of n bits beside the row).
// A row that was resumed from row 0's timeline after 64 b positions did not place those itself: their
// completion rounds are row 0's, taken from a copy of row 0's row in position order.  Likewise a row
// that stopped at position 64 b' because its timeline had become row 0's again: from there on every
// request completes when it does in row 0 (the positions are then those of row 0's order: behind the
// last difference the two orders are the same, and a row that placed nothing holds the same requests
// as row 0 wherever they differ).
#include "kvsched_internal.h"

#include <limits.h>

namespace {

__global__ __launch_bounds__(256) void permute_rows_kernel(const int32_t *orders, int32_t n, int32_t *completion,
                                                           int64_t *tel_out, int32_t *words,
                                                           const int32_t *resume_block, const int32_t *row0,
                                                           const int32_t *rejoin_block)
{
    extern __shared__ int row_by_id[];
    unsigned int *seen = (unsigned int *)(row_by_id + n);  // one bit per request id
    const int32_t *order = orders + (size_t)blockIdx.x * (size_t)n;
    int32_t *comp = completion + (size_t)blockIdx.x * (size_t)n;
    for (int i = threadIdx.x; i < ((n + 31) >> 5); i += blockDim.x) seen[i] = 0;
    const int shared = resume_block ? min(64 * resume_block[blockIdx.x], n) : 0;  // positions placed by row 0 only
    int tail = n;  // ... and from here on
    if (rejoin_block && rejoin_block[blockIdx.x] != INT_MAX) tail = min(64 * rejoin_block[blockIdx.x], n);
    __syncthreads();
    int bad = 0;
    for (int k = threadIdx.x; k < n; k += blockDim.x) {
        const int raw = order[k];
        const int r = min(max(raw, 0), n - 1);
        const unsigned int bit = 1u << (r & 31);
        if (raw != r || (atomicOr(&seen[r >> 5], bit) & bit)) bad = 1;  // out of range, or met before
        if (k < tail) row_by_id[r] = k < shared ? row0[k] : comp[k];
    }
    for (int k = tail + threadIdx.x; k < n; k += blockDim.x) row_by_id[min(max(orders[k], 0), n - 1)] = row0[k];
    if (__syncthreads_or(bad) && threadIdx.x == 0) {  // the row is no permutation: its results are void
        tel_out[blockIdx.x] = -1;
        atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_ORDER);
    }
    for (int i = threadIdx.x; i < n; i += blockDim.x) comp[i] = row_by_id[i];
}

}  // namespace

int kvs_launch_permute_rows(const int32_t *orders, int32_t C, int32_t n, int32_t *completion, int64_t *tel_out,
                            int32_t *d_words, const int32_t *resume_block, const int32_t *row0,
                            const int32_t *rejoin_block, hipStream_t st)
{
    if (n > KVS_PERMUTE_MAX_N) return KVSCHED_ERANGE;
    const size_t lds = sizeof(int32_t) * ((size_t)n + (((size_t)n + 31) >> 5));
    hipLaunchKernelGGL(permute_rows_kernel, dim3((unsigned)C), dim3(256), lds, st, orders, n, completion, tel_out,
                       d_words, resume_block, row0, rejoin_block);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
