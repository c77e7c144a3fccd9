// Phase 1 of Algorithm 1 ("Batch Construction") with every batch chosen by Local Swap Search
// (the appendix algorithm of that name): fill greedily in ascending s+o, then repeat the first
// improving single exchange (r_out in X, r_in not in X) that keeps sum(s+o) <= M, scanning
// members and non-members in the sorted order (s+o, o, id).
//
// An exchange keeps |X|, so it lowers F = sum o / |X|^2 exactly when o_in < o_out.  With the
// remaining requests in sorted order (w = s+o ascending) and slack = M - mem, r_in fits against
// r_out iff w_in <= w_out + slack, i.e. iff r_in lies before ub(out) = first place with
// w > w_out + slack.  Hence, with pm[j] = least o among the non-members before place j,
//     r_out has an improving partner   <=>   pm[ub(out)] < o_out,
// the pair the double scan meets first is the first such member, and its partner is the first
// non-member with o < o_out (it lies before ub(out) because one such non-member does).
// One step = one exclusive prefix-minimum scan, one binary search per member, two block-wide
// minimum reductions; the whole construction runs in one workgroup, the working set in LDS once
// at most LS_CAP requests remain.
#include "phase1_util.h"

namespace {

constexpr int LS_CAP = 8192;             // remaining requests held in LDS
constexpr int LS_INF = 0x7fffffff;
constexpr unsigned LS_MEMBER = 0x80000000u;  // membership flag kept in the sign bit of the o entry
constexpr int LS_NONE = 0x7fffffff;

struct SwapLds {
    int wave_min[NWAVES];
    int first_out[2];  // alternating slots: least place of a member that has a partner
    int first_in[2];   //                    least place of its partner
    unsigned long long acc_mem, acc_S;
    long long scan_w[NWAVES];
    int scan_c[NWAVES];
};

struct WorkLds {
    int w[LS_CAP];
    int o[LS_CAP];
    int pm[LS_CAP + 1];
};

union PhaseLds {
    RadixLds radix;
    WorkLds work;
};

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_else(int keep, int v)
{
    return __builtin_amdgcn_update_dpp(keep, v, CTRL, ROW_MASK, 0xf, false);
}

// inclusive prefix minimum over the 64 lanes (all lanes active)
__device__ __forceinline__ int wave_scan_min(int v)
{
    v = min(v, dpp_else<0x111, 0xf>(LS_INF, v));  // row_shr:1
    v = min(v, dpp_else<0x112, 0xf>(LS_INF, v));  // row_shr:2
    v = min(v, dpp_else<0x114, 0xf>(LS_INF, v));  // row_shr:4
    v = min(v, dpp_else<0x118, 0xf>(LS_INF, v));  // row_shr:8
    v = min(v, dpp_else<0x142, 0xa>(LS_INF, v));  // row_bcast15 into rows 1 and 3
    v = min(v, dpp_else<0x143, 0xc>(LS_INF, v));  // row_bcast31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ int wave_min_i32(int v)
{
    v = min(v, dpp_else<0xB1, 0xf>(v, v));   // quad_perm [1,0,3,2]
    v = min(v, dpp_else<0x4E, 0xf>(v, v));   // quad_perm [2,3,0,1]
    v = min(v, dpp_else<0x141, 0xf>(v, v));  // row_half_mirror
    v = min(v, dpp_else<0x140, 0xf>(v, v));  // row_mirror
    const int a = __builtin_amdgcn_readlane(v, 0);
    const int b = __builtin_amdgcn_readlane(v, 16);
    const int c = __builtin_amdgcn_readlane(v, 32);
    const int d = __builtin_amdgcn_readlane(v, 48);
    return min(min(a, b), min(c, d));
}

// first place in [lo, hi) whose w exceeds lim (hi if none); W ascending
__device__ __forceinline__ int upper_bound_w(const int *W, int lo, int hi, int lim)
{
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (W[mid] <= lim) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Greedy fill over W[0..m): the longest prefix with sum of w <= M.  Marks it in O, returns its
// length K; mem and S receive its sums.  (Sizes ascend, so nothing after the first request that
// does not fit can fit either: the fill of the algorithm is this prefix.)
__device__ int greedy_fill(const int *W, int *O, int m, int M, long long &mem, long long &S, SwapLds &L)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { L.acc_mem = 0; L.acc_S = 0; }
    __syncthreads();
    long long carry = 0;
    int K = 0;
    for (int tile = 0; tile < m; tile += TPB) {
        const int i = tile + tid;
        long long w = i < m ? (long long)W[i] : 0;
        const long long own = w;
        for (int d = 1; d < 64; d <<= 1) {
            const long long u = __shfl_up(w, d);
            if (lane >= d) w += u;
        }
        if (lane == 63) L.scan_w[wave] = w;
        __syncthreads();
        long long off = carry, total = carry;
        for (int v = 0; v < NWAVES; ++v) {
            const long long x = L.scan_w[v];
            if (v < wave) off += x;
            total += x;
        }
        const bool fit = i < m && w + off <= (long long)M;
        if (fit) {
            atomicAdd(&L.acc_mem, (unsigned long long)own);
            atomicAdd(&L.acc_S, (unsigned long long)O[i]);
            O[i] = (int)((unsigned)O[i] | LS_MEMBER);
        }
        const int c = __syncthreads_count(fit);
        K += c;
        carry = total;
        if (c < TPB) break;  // uniform: c is the same in every thread
    }
    __syncthreads();
    mem = (long long)L.acc_mem;
    S = (long long)L.acc_S;
    return K;
}

// The exchanges of one batch.  W, O, PM: m sorted entries (LDS or global memory), members flagged
// in O's sign bit, initially the first K.  Returns the number of exchanges; hi_out = a bound such
// that every member lies before it.
__device__ int swap_loop(const int *W, int *O, int *PM, int m, int K, int M, long long &mem, long long &S,
                         int &hi_out, SwapLds &L)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 2) { L.first_out[tid] = LS_NONE; L.first_in[tid] = LS_NONE; }
    __syncthreads();
    int hi = K, swaps = 0;
    for (int it = 0;; ++it) {
        const int slot = it & 1;
        const int slack = (int)((long long)M - mem);
        // no member is larger than W[hi-1]; places from U on fit against no member
        const int U = upper_bound_w(W, hi, m, W[hi - 1] + slack);

        // ---- pm[j] = least o among non-members before place j, j = 0..U
        int carry = LS_INF;
        for (int tile = 0; tile <= U; tile += TPB) {
            const int i = tile + tid;
            int v = LS_INF;
            if (i < U) {
                const int ov = O[i];
                if (ov >= 0) v = ov;
            }
            const int incl = wave_scan_min(v);
            if (lane == 63) L.wave_min[wave] = incl;
            int excl = __shfl_up(incl, 1);
            if (lane == 0) excl = LS_INF;
            __syncthreads();
            int off = carry, total = carry;
            for (int u = 0; u < NWAVES; ++u) {
                const int x = L.wave_min[u];
                if (u < wave) off = min(off, x);
                total = min(total, x);
            }
            if (i <= U) PM[i] = min(off, excl);
            carry = total;
            __syncthreads();
        }

        // ---- first member with an improving partner that fits
        int cand = LS_NONE;
        for (int tile = 0; tile < hi; tile += TPB) {
            const int a = tile + tid;
            if (a < hi) {
                const int ov = O[a];
                if (ov < 0) {
                    const int ub = upper_bound_w(W, a + 1, U, W[a] + slack);
                    if (PM[ub] < (int)((unsigned)ov & ~LS_MEMBER)) cand = min(cand, a);
                }
            }
        }
        cand = wave_min_i32(cand);
        if (lane == 0 && cand != LS_NONE) atomicMin(&L.first_out[slot], cand);
        __syncthreads();
        const int a_star = L.first_out[slot];
        if (a_star == LS_NONE) break;  // uniform

        // ---- its first partner: the first non-member with smaller o
        const int o_a = (int)((unsigned)O[a_star] & ~LS_MEMBER);
        int cb = LS_NONE;
        for (int tile = 0; tile < U; tile += TPB) {
            const int b = tile + tid;
            if (b < U) {
                const int ov = O[b];
                if (ov >= 0 && ov < o_a) cb = min(cb, b);
            }
        }
        cb = wave_min_i32(cb);
        if (lane == 0 && cb != LS_NONE) atomicMin(&L.first_in[slot], cb);
        __syncthreads();
        const int b_star = L.first_in[slot];
        if (b_star == LS_NONE) break;  // cannot happen: pm said a partner exists; never spin

        // ---- exchange; every thread keeps the running sums, the owners rewrite the flags
        const int o_b = (int)((unsigned)O[b_star] & ~LS_MEMBER);
        mem += (long long)W[b_star] - (long long)W[a_star];
        S += (long long)o_b - (long long)o_a;
        hi = max(hi, b_star + 1);
        ++swaps;
        if ((a_star & (TPB - 1)) == tid) O[a_star] = o_a;
        if ((b_star & (TPB - 1)) == tid) O[b_star] = (int)((unsigned)o_b | LS_MEMBER);
        if (tid == 0) {  // the other slot was last read two barriers ago; ready it for the next step
            L.first_out[slot ^ 1] = LS_NONE;
            L.first_in[slot ^ 1] = LS_NONE;
        }
    }
    hi_out = hi;
    return swaps;
}

__global__ __launch_bounds__(TPB) void local_swap_kernel(int32_t n, const int32_t *s, const int32_t *o, int32_t M,
                                                         int32_t *order_out, int32_t *batch_end_out, double *F_out,
                                                         int32_t *swaps_out, int32_t *num_batches_out, int *gw, int *go,
                                                         int *gid, int *alt_o, int *buf0, int *buf1, int *by_o,
                                                         int *batch_of, int32_t *words)
{
    __shared__ PhaseLds P;
    __shared__ SwapLds L;
    __shared__ int sh[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- well-formedness and key widths
    int omax = 0, wmax = 0, bad = 0;
    for (int i = tid; i < n; i += TPB) {
        const int sv = s[i], ov = o[i];
        if (sv < 1 || ov < 1 || (long long)sv + ov > (long long)M) bad = 1;
        omax = max(omax, ov);
        wmax = max(wmax, (sv < 1 || ov < 1) ? 0 : (int)min((long long)sv + ov, (long long)M));
    }
    if (tid < 4) sh[tid] = 0;
    __syncthreads();
    if (bad) atomicOr(&sh[2], 1);
    atomicMax(&sh[0], omax);
    atomicMax(&sh[1], wmax);
    __syncthreads();
    omax = sh[0];
    wmax = sh[1];
    if (sh[2] != 0) {  // a request that can never run: report, emit no batches
        if (tid == 0) {
            atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            *num_batches_out = 0;
        }
        return;
    }

    // ---- key sorts: ids by (o, id), kept for the emission order, then on by s+o
    for (int i = tid; i < n; i += TPB) buf0[i] = i;
    __syncthreads();
    int *cur = buf0, *alt = buf1;
    auto key_o = [o](int id) { return o[id]; };
    auto key_w = [s, o](int id) { return s[id] + o[id]; };
    for (int shift = 0; shift < bits_of(omax); shift += 8) {
        radix_pass(cur, alt, n, shift, key_o, P.radix);
        int *t = cur; cur = alt; alt = t;
    }
    for (int i = tid; i < n; i += TPB) by_o[i] = cur[i];
    __syncthreads();
    for (int shift = 0; shift < bits_of(wmax); shift += 8) {
        radix_pass(cur, alt, n, shift, key_w, P.radix);
        int *t = cur; cur = alt; alt = t;
    }
    for (int i = tid; i < n; i += TPB) {
        const int id = cur[i];
        gid[i] = id;
        go[i] = o[id];
        gw[i] = s[id] + o[id];
    }
    __threadfence_block();
    __syncthreads();
    int *alt_w = buf0, *alt_id = buf1;  // the sort buffers are free until the last step

    // ---- batches
    int a = 0, nb = 0;
    while (a < n) {
        const int m = n - a;
        const bool in_lds = m <= LS_CAP;
        int *W, *O, *PM;
        if (in_lds) {
            for (int i = tid; i < m; i += TPB) {
                P.work.w[i] = gw[a + i];
                P.work.o[i] = go[a + i];
            }
            __syncthreads();
        }
        long long mem = 0, S = 0;
        int K, hi = 0, swaps = 0;
        if (in_lds) {
            K = greedy_fill(P.work.w, P.work.o, m, M, mem, S, L);
            if (K >= 1) swaps = swap_loop(P.work.w, P.work.o, P.work.pm, m, K, M, mem, S, hi, L);
            W = P.work.w; O = P.work.o; PM = P.work.pm;
        } else {
            K = greedy_fill(gw + a, go + a, m, M, mem, S, L);
            if (K >= 1) swaps = swap_loop(gw + a, go + a, alt_o, m, K, M, mem, S, hi, L);
            W = gw + a; O = go + a; PM = alt_o;
        }
        (void)PM;
        if (K < 1) {  // cannot happen for well-formed input; never spin
            if (tid == 0) atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            break;
        }
        __syncthreads();
        if (tid == 0) {
            batch_end_out[nb] = a + K;
            F_out[nb] = (double)S / ((double)K * (double)K);
            if (swaps_out) swaps_out[nb] = swaps;
        }
        // members get the batch number; non-members of [0, hi) close up behind the K removed
        // places (stable), through the spare arrays
        int carry = 0;
        for (int tile = 0; tile < hi; tile += TPB) {
            const int i = tile + tid;
            int keep = 0, ov = 0;
            if (i < hi) {
                ov = O[i];
                if (ov < 0) batch_of[gid[a + i]] = nb;
                else keep = 1;
            }
            int c = keep;
            for (int d = 1; d < 64; d <<= 1) {
                const int u = __shfl_up(c, d);
                if (lane >= d) c += u;
            }
            if (lane == 63) L.scan_c[wave] = c;
            __syncthreads();
            int off = carry, total = carry;
            for (int u = 0; u < NWAVES; ++u) {
                const int x = L.scan_c[u];
                if (u < wave) off += x;
                total += x;
            }
            if (keep) {
                const int dst = K + off + c - 1;
                alt_w[dst] = W[i];
                alt_o[dst] = ov;
                alt_id[dst] = gid[a + i];
            }
            carry = total;
            __syncthreads();
        }
        __threadfence_block();
        __syncthreads();
        for (int i = K + tid; i < hi; i += TPB) {
            gw[a + i] = alt_w[i];
            go[a + i] = alt_o[i];
            gid[a + i] = alt_id[i];
        }
        __threadfence_block();
        __syncthreads();
        a += K;
        ++nb;
    }
    if (tid == 0) *num_batches_out = nb;
    __threadfence_block();
    __syncthreads();

    // ---- order the (o, id)-sorted ids by batch number (stable): each batch in nondecreasing o
    int *src = by_o, *dst = buf0, *other = buf1;
    auto key_b = [batch_of](int id) { return batch_of[id]; };
    bool first = true;
    for (int shift = 0; shift < bits_of(nb - 1); shift += 8) {
        radix_pass(src, dst, n, shift, key_b, P.radix);
        if (first) { src = dst; dst = other; first = false; }
        else { int *t = src; src = dst; dst = t; }
    }
    for (int i = tid; i < n; i += TPB) order_out[i] = src[i];
}

}  // namespace

size_t kvs_local_swap_scratch_bytes(int32_t n)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    return np * 8 * sizeof(int) + 256;
}

int kvs_launch_local_swap(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t *order_out,
                          int32_t *batch_end_out, double *F_out, int32_t *swaps_out, int32_t *num_batches_out,
                          void *scratch, int32_t *d_words, hipStream_t st)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    int *gw = (int *)scratch;
    int *go = gw + np;
    int *gid = go + np;
    int *alt_o = gid + np;
    int *buf0 = alt_o + np;
    int *buf1 = buf0 + np;
    int *by_o = buf1 + np;
    int *batch_of = by_o + np;
    hipLaunchKernelGGL(local_swap_kernel, dim3(1), dim3(TPB), 0, st, n, s, o, M, order_out, batch_end_out, F_out,
                       swaps_out, num_batches_out, gw, go, gid, alt_o, buf0, buf1, by_o, batch_of, d_words);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
