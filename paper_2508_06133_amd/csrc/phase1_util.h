// Block-level building blocks of the Phase 1 kernels (one workgroup of T threads builds the
// whole order): a stable 8-bit LSD radix pass over request ids.
#pragma once

#include "kvsched_internal.h"

namespace {

template <int T>
struct RadixLds {
    int hist[256];
    int wcount[T / 64][256];  // per tile: lanes of wave w holding digit d
    int woff[T / 64][256];    // per tile: output offset of wave w's first lane with digit d
};

__device__ __forceinline__ unsigned long long lanemask_lt()
{
    return (1ull << (threadIdx.x & 63)) - 1ull;
}

// One stable counting pass on an 8-bit digit of key(id).  in/out: [n] ids.
template <int T, class KeyFn>
__device__ void radix_pass(const int *in, int *out, int n, int shift, KeyFn key, RadixLds<T> &L)
{
    constexpr int TPB = T, NWAVES = T / 64;
    const int tid = threadIdx.x, wave = tid >> 6;
    for (int i = tid; i < 256; i += TPB) L.hist[i] = 0;
    for (int i = tid; i < NWAVES * 256; i += TPB) (&L.wcount[0][0])[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += TPB) atomicAdd(&L.hist[(key(in[i]) >> shift) & 255], 1);
    __syncthreads();
    if (wave == 0) {  // exclusive scan of the 256 digit counts -> running output base per digit
        const int lane = tid;
        const int c0 = L.hist[4 * lane], c1 = L.hist[4 * lane + 1], c2 = L.hist[4 * lane + 2],
                  c3 = L.hist[4 * lane + 3];
        int incl = c0 + c1 + c2 + c3;  // each lane owns four digits
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        const int base = incl - (c0 + c1 + c2 + c3);
        L.hist[4 * lane] = base;
        L.hist[4 * lane + 1] = base + c0;
        L.hist[4 * lane + 2] = base + c0 + c1;
        L.hist[4 * lane + 3] = base + c0 + c1 + c2;
    }
    __syncthreads();
    for (int tile = 0; tile < n; tile += TPB) {
        const int i = tile + tid;
        const bool valid = i < n;
        const int id = valid ? in[i] : 0;
        const int d = valid ? ((key(id) >> shift) & 255) : 256;
        // lanes of this wave holding the same digit
        unsigned long long peers = ~0ull;
#pragma unroll
        for (int b = 0; b < 9; ++b) {
            const unsigned long long bal = __builtin_amdgcn_ballot_w64((d >> b) & 1);
            peers &= ((d >> b) & 1) ? bal : ~bal;
        }
        const int rank = __popcll(peers & lanemask_lt());
        if (valid && rank == 0) L.wcount[wave][d] = __popcll(peers);
        __syncthreads();
        for (int dd = tid; dd < 256; dd += TPB) {  // per digit: offsets of the waves in order, advance the running base
            int off = L.hist[dd];
            for (int w = 0; w < NWAVES; ++w) {
                const int c = L.wcount[w][dd];
                L.wcount[w][dd] = 0;  // ready for the next tile
                L.woff[w][dd] = off;
                off += c;
            }
            L.hist[dd] = off;
        }
        __syncthreads();
        if (valid) out[L.woff[wave][d] + rank] = id;
        __syncthreads();
    }
}

// The same pass done by ONE wavefront (no barriers: LDS operations of a wavefront take effect in
// program order): 64 ids a turn, in order, each lane ranked among the lanes of its turn that hold the
// same digit; hist[] holds 256 running output positions.
template <class KeyFn>
__device__ void radix_pass_wave(const int *in, int *out, int n, int shift, KeyFn key, int *hist)
{
    const int lane = threadIdx.x & 63;
    for (int i = lane; i < 256; i += 64) hist[i] = 0;
    for (int i = lane; i < n; i += 64) atomicAdd(&hist[(key(in[i]) >> shift) & 255], 1);
    {
        const int c0 = hist[4 * lane], c1 = hist[4 * lane + 1], c2 = hist[4 * lane + 2], c3 = hist[4 * lane + 3];
        int incl = c0 + c1 + c2 + c3;  // each lane owns four digits
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        const int base = incl - (c0 + c1 + c2 + c3);
        hist[4 * lane] = base;
        hist[4 * lane + 1] = base + c0;
        hist[4 * lane + 2] = base + c0 + c1;
        hist[4 * lane + 3] = base + c0 + c1 + c2;
    }
    for (int i0 = 0; i0 < n; i0 += 64) {
        const int i = i0 + lane;
        const bool valid = i < n;
        const int id = valid ? in[i] : 0;
        const int d = valid ? ((key(id) >> shift) & 255) : 256;
        unsigned long long peers = ~0ull;
#pragma unroll
        for (int b = 0; b < 9; ++b) {
            const unsigned long long bal = __builtin_amdgcn_ballot_w64((d >> b) & 1);
            peers &= ((d >> b) & 1) ? bal : ~bal;
        }
        const int rank = __popcll(peers & lanemask_lt());
        const int cnt = __popcll(peers);
        const int base = valid ? hist[d] : 0;
        if (valid) out[base + rank] = id;
        if (valid && rank == cnt - 1) hist[d] = base + cnt;  // one lane per digit moves its position on
    }
}

__device__ __forceinline__ int bits_of(long long v)
{
    return v <= 0 ? 1 : 64 - __clzll(v);
}

}  // namespace
