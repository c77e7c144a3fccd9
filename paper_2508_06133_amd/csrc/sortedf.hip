// Sorted-F order construction: Phase 1 of Algorithm 1 ("Batch Construction") with the batch
// taken among the feasible prefixes of the remaining requests sorted by (s+o, o, id), scored
// by the F-metric of Section 4, F(X) = sum o_i / |X|^2, or by the generalised metric of Section 7
// ("Robustness to prefill weighting"), G(X) = sum (alpha s_i + o_i) / |X|^2 with alpha = ga / gb: the
// effective length ga s_i + gb o_i replaces o_i in the metric's numerator, nowhere else.
//
// Since every batch is a prefix of what remains, the remaining requests stay sorted: one key
// sort serves all batches, and batch b is the segment [a_b, a_b + k*) of the sorted array.
// One workgroup does the whole construction:
//   1. stable LSD radix sort of the ids by o            -> requests in (o, id) order
//   2. continue the same sort on s+o                    -> requests in (s+o, o, id) order
//   3. prefix sums W (of s+o) and S (of o) over that order
//   4. per batch: feasible extent K by a two-level search on W (sum of peaks <= M), extended by a
//      bisection on the simultaneous-start memory profile when that is the feasibility asked for;
//      argmin over k <= K of S_k / k^2 compared in exact 128-bit integers, tie rule applied;
//      F reported as one fp64 division
//   5. stable sort of the (o, id)-ordered ids by batch number -> each batch in nondecreasing o
// The working arrays and a copy of the lengths (56 bytes per request) live in LDS when they fit
// beside the sort's tables (n up to about 2200), else in the caller's scratch buffer in HBM: the construction is a chain of short
// dependent steps by one workgroup, so its time is the latency of those arrays; in particular a
// barrier waits until every store before it has been acknowledged, which for HBM takes microseconds.
#include "phase1_util.h"

namespace {

constexpr int TPB = 1024;
constexpr int NWAVES = TPB / 64;

struct Lds {
    RadixLds<TPB> radix;
    int hist[2];
    long long scan_a[NWAVES];
    long long scan_b[NWAVES];
    long long carry_a, carry_b;
    long long red_S[NWAVES];
    int red_k[NWAVES];
    long long best_S;
    int best_k;
    int flag;
    int fit[2];
};

// sign of Sa/ka^2 - Sb/kb^2 in exact integers (Sa, Sb < 2^63; ka, kb < 2^31)
__device__ __forceinline__ int cmp_F(long long Sa, int ka, long long Sb, int kb)
{
    const unsigned long long qa = (unsigned long long)ka * (unsigned long long)ka;
    const unsigned long long qb = (unsigned long long)kb * (unsigned long long)kb;
    const unsigned long long l_hi = __umul64hi((unsigned long long)Sa, qb), l_lo = (unsigned long long)Sa * qb;
    const unsigned long long r_hi = __umul64hi((unsigned long long)Sb, qa), r_lo = (unsigned long long)Sb * qa;
    if (l_hi != r_hi) return l_hi < r_hi ? -1 : 1;
    if (l_lo != r_lo) return l_lo < r_lo ? -1 : 1;
    return 0;
}

// is prefix (Sa, ka) a better batch than (Sb, kb)?  kb == 0 means "none yet".
__device__ __forceinline__ bool better(long long Sa, int ka, long long Sb, int kb, int tie_rule)
{
    if (ka == 0) return false;
    if (kb == 0) return true;
    const int c = cmp_F(Sa, ka, Sb, kb);
    if (c != 0) return c < 0;
    return tie_rule == KVSCHED_TIE_LARGER ? ka > kb : ka < kb;
}

// The same question when every S < 2^32 and every k < 2^16: both cross products fit in 64 bits.
__device__ __forceinline__ bool better_small(unsigned Sa, int ka, unsigned Sb, int kb, int tie_rule)
{
    const unsigned long long l = (unsigned long long)Sa * (unsigned)(kb * kb);
    const unsigned long long r = (unsigned long long)Sb * (unsigned)(ka * ka);
    const bool wins = l != r ? l < r : (tie_rule == KVSCHED_TIE_LARGER ? ka > kb : ka < kb);
    return ka != 0 && (kb == 0 || wins);
}

template <int CTRL>
__device__ __forceinline__ void take_better_small(unsigned &bS, int &bk, int tie_rule)
{
    const unsigned oS = (unsigned)__builtin_amdgcn_update_dpp((int)bS, (int)bS, CTRL, 0xf, 0xf, false);
    const int ok = __builtin_amdgcn_update_dpp(bk, bk, CTRL, 0xf, 0xf, false);
    if (better_small(oS, ok, bS, bk, tie_rule)) { bS = oS; bk = ok; }
}

// Best (S, k) of a 16-lane row into all its lanes: lane exchanges 1, 2 apart, then the two
// mirrorings (quads, halves).  "Better" is a strict total order on distinct k, so any tree works.
__device__ __forceinline__ void row_best_small(unsigned &bS, int &bk, int tie_rule)
{
    take_better_small<0xB1>(bS, bk, tie_rule);   // quad_perm [1,0,3,2]
    take_better_small<0x4E>(bS, bk, tie_rule);   // quad_perm [2,3,0,1]
    take_better_small<0x141>(bS, bk, tie_rule);  // row_half_mirror
    take_better_small<0x140>(bS, bk, tie_rule);  // row_mirror
}

// Largest k in [0, rem] with g(k) <= M, for g increasing in k (k = 1..rem).  Every thread
// receives it.  While a thread's share of the probes is short (rem <= 4 TPB) each thread counts
// the fitting probes of its own run of consecutive k and the one thread whose run holds the
// boundary publishes the answer: one barrier.  `slot` alternates between back-to-back calls.
template <class G>
__device__ int count_fitting(int rem, G g, int32_t M, Lds &L, int slot)
{
    const int tid = threadIdx.x;
    const int stride = (rem + TPB - 1) / TPB;
    if (stride <= 4) {
        const int k0 = tid * stride;  // this thread probes k0+1 .. k0+stride, and k0+stride+1 to see the boundary
        bool fit[5];
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int k = k0 + 1 + j;
            fit[j] = j <= stride && k <= rem && g((long long)k) <= (long long)M;
        }
        int c = 0;
        bool beyond = false;  // does the first probe after this thread's run fit?
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            if (j < stride) c += fit[j] ? 1 : 0;
            if (j == stride) beyond = fit[j];
        }
        // a prefix of all probes fits: the boundary lies in the run that fits at least partly and
        // is not followed by a fitting probe; if nothing fits at all, thread 0 reports 0
        if ((c > 0 && !beyond) || (tid == 0 && c == 0)) L.fit[slot] = k0 + c;
        __syncthreads();
        return L.fit[slot];
    }
    const long long k1 = (long long)(tid + 1) * stride;  // coarse probes, a prefix of them fits
    const bool ok1 = k1 <= rem && g(k1) <= (long long)M;
    int K = __syncthreads_count(ok1) * stride;
    const long long k2 = (long long)K + tid + 1;  // fine probes inside the next stride
    const bool ok2 = tid < stride && k2 <= rem && g(k2) <= (long long)M;
    K += __syncthreads_count(ok2);
    return K;
}

// Do the k requests at places [a, a + k) of the (s+o, o, id) order, started together, stay within
// M at every completion time?  Memory at time o_j = sum over {i: o_i >= o_j} of (s_i + o_j)
// (Section 4).  The ids are visited in decreasing o through a list in ascending o that holds every
// member (all requests in (o, id) order, or the candidates of the batch sorted by o); running sums
// of s and of the count over the members seen so far give the memory at each member's completion
// (among equal o the last one visited sees the whole group, the earlier ones a part of it, which
// cannot exceed it).  Every thread receives the answer.
__device__ bool profile_fits(int n, int a, int k, const int32_t *s, const int32_t *o, const int *by_o,
                             const int *pos_w, int32_t M, Lds &L)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    long long carry_s = 0;
    int carry_c = 0, viol = 0;
    for (int tile = 0; tile < n; tile += TPB) {
        const int idx = n - 1 - (tile + tid);
        int id = 0, c = 0;
        long long sv = 0;
        if (idx >= 0) {
            id = by_o[idx];
            const int p = pos_w[id];
            if (p >= a && p < a + k) { c = 1; sv = s[id]; }
        }
        const int member = c;
        for (int d = 1; d < 64; d <<= 1) {
            const long long us = __shfl_up(sv, d);
            const int uc = __shfl_up(c, d);
            if (lane >= d) { sv += us; c += uc; }
        }
        if (lane == 63) { L.scan_a[wave] = sv; L.scan_b[wave] = c; }
        __syncthreads();
        long long off_s = carry_s, tot_s = carry_s;
        long long off_c = carry_c, tot_c = carry_c;
        for (int v = 0; v < NWAVES; ++v) {
            const long long xs = L.scan_a[v], xc = L.scan_b[v];
            if (v < wave) { off_s += xs; off_c += xc; }
            tot_s += xs;
            tot_c += xc;
        }
        if (member && (sv + off_s) + (c + off_c) * (long long)o[id] > (long long)M) viol = 1;
        carry_s = tot_s;
        carry_c = (int)tot_c;
        __syncthreads();
        if (carry_c >= k) break;  // uniform: every member has been seen
    }
    return __syncthreads_or(viol) == 0;
}

// PROFILE: feas_mode is KVSCHED_FEAS_PROFILE (its code stays out of the other instantiation)
template <bool IN_LDS, bool PROFILE>
__global__ __launch_bounds__(TPB) void sortedF_kernel(int32_t n, const int32_t *s_in, const int32_t *o_in, int32_t M,
                                                      int32_t ga, int32_t gb, int32_t tie_rule, int32_t feas_mode,
                                                      int32_t *order_out, int32_t *batch_end_out, double *F_out,
                                                      int32_t *num_batches_out, int *buf0, int *buf1, int *by_o,
                                                      long long *cumW, long long *cumS, long long *cumG,
                                                      int *batch_of, int *pos_w, int32_t *words)
{
    __shared__ Lds L;
    extern __shared__ long long lds_arrays[];
    // In this instantiation every working array below is carved from LDS and nothing else, so that
    // the accesses compile to LDS instructions (a pointer that may be either costs HBM-like latency).
    const int32_t *s = s_in, *o = o_in;
    int *ends = batch_end_out;  // batch ends: collected in LDS and copied out at the end, or written in place
    int *s_lds = nullptr, *o_lds = nullptr;  // the lengths too: every later read of them is a gather by request id
    if constexpr (IN_LDS) {
        const size_t np = ((size_t)n + 64) & ~(size_t)63;
        const bool alias = cumG == cumS;
        cumW = lds_arrays;
        cumS = cumW + np;
        cumG = alias ? cumS : cumS + np;
        buf0 = (int *)(lds_arrays + 3 * np);
        buf1 = buf0 + np;
        by_o = buf1 + np;
        batch_of = by_o + np;
        pos_w = batch_of + np;
        ends = pos_w + np;
        s_lds = ends + np;
        o_lds = s_lds + np;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- well-formedness and key widths
    int omax = 0, wmax = 0, bad = 0;
    for (int i = tid; i < n; i += TPB) {
        const int sv = s_in[i], ov = o_in[i];
        if constexpr (IN_LDS) {
            s_lds[i] = sv;
            o_lds[i] = ov;
        }
        if (sv < 1 || ov < 1 || (long long)sv + ov > (long long)M) bad = 1;
        omax = max(omax, ov);
        wmax = max(wmax, (sv < 1 || ov < 1) ? 0 : (int)min((long long)sv + ov, (long long)M));
    }
    if (tid == 0) L.flag = 0;
    __syncthreads();
    if (bad) atomicOr(&L.flag, 1);
    if (tid < 2) L.hist[tid] = 0;
    __syncthreads();
    atomicMax(&L.hist[0], omax);
    atomicMax(&L.hist[1], wmax);
    __syncthreads();
    omax = L.hist[0];
    wmax = L.hist[1];
    const bool any_bad = L.flag != 0;
    __syncthreads();
    if (any_bad) {  // a request that can never run: report, emit no batches
        if (tid == 0) {
            atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            *num_batches_out = 0;
        }
        return;
    }

    if constexpr (IN_LDS) {
        s = s_lds;
        o = o_lds;
    }

    // ---- 1/2: key sorts (ids start in id order, every pass is stable)
    for (int i = tid; i < n; i += TPB) buf0[i] = i;
    __syncthreads();
    int *cur = buf0, *alt = buf1;
    auto key_o = [o](int id) { return o[id]; };
    auto key_w = [s, o](int id) { return s[id] + o[id]; };
    for (int shift = 0; shift < bits_of(omax); shift += 8) {
        radix_pass(cur, alt, n, shift, key_o, L.radix);
        int *t = cur; cur = alt; alt = t;
    }
    for (int i = tid; i < n; i += TPB) by_o[i] = cur[i];
    __syncthreads();
    for (int shift = 0; shift < bits_of(wmax); shift += 8) {
        radix_pass(cur, alt, n, shift, key_w, L.radix);
        int *t = cur; cur = alt; alt = t;
    }
    const int *sorted = cur;  // (s+o, o, id) ascending
    if (PROFILE) {
        for (int i = tid; i < n; i += TPB) pos_w[sorted[i]] = i;
    }

    // ---- 3: inclusive prefix sums over the sorted order; cumW[0] = cumS[0] = 0
    if (tid == 0) {
        L.carry_a = 0;
        L.carry_b = 0;
        cumW[0] = 0;
        cumS[0] = 0;
        cumG[0] = 0;  // (cumG is cumS itself under the F-metric)
    }
    __syncthreads();
    for (int tile = 0; tile < n; tile += TPB) {
        const int i = tile + tid;
        long long w = 0, q = 0;
        if (i < n) {
            const int id = sorted[i];
            q = o[id];
            w = (long long)s[id] + q;
        }
        for (int d = 1; d < 64; d <<= 1) {
            const long long uw = __shfl_up(w, d), uq = __shfl_up(q, d);
            if (lane >= d) { w += uw; q += uq; }
        }
        if (lane == 63) { L.scan_a[wave] = w; L.scan_b[wave] = q; }
        __syncthreads();
        long long offw = L.carry_a, offq = L.carry_b;
        for (int v = 0; v < wave; ++v) { offw += L.scan_a[v]; offq += L.scan_b[v]; }
        if (i < n) { cumW[i + 1] = w + offw; cumS[i + 1] = q + offq; }
        __syncthreads();
        if (tid == TPB - 1) { L.carry_a = w + offw; L.carry_b = q + offq; }
        __syncthreads();
    }
    if (cumG != cumS) {  // sum of the effective lengths = ga (W - S) + gb S
        __threadfence_block();
        __syncthreads();
        for (int i = tid; i <= n; i += TPB) cumG[i] = (long long)ga * (cumW[i] - cumS[i]) + (long long)gb * cumS[i];
    }
    __threadfence_block();
    __syncthreads();

    // ---- 4 and 5 by one wavefront when everything sits in LDS and feasibility is the sum of peaks:
    // the steps that follow are short and dependent; sixteen wavefronts meeting at barriers after
    // each of them take 2.5 us a batch, one wavefront on its own 2 us (and the final sort 8 us instead of 4).
    if constexpr (IN_LDS && !PROFILE) {
        if (wave != 0) return;
        const bool small1 = n < 65536 && cumG[n] < (1ll << 32);
        int a1 = 0, nb1 = 0;
        while (a1 < n) {
            const long long W0 = cumW[a1], G0 = cumG[a1];
            // feasible extent K: 64 probes a turn narrow [lo, lo + span] (fit(lo) holds; fit is monotone)
            int lo = 0, span = n - a1;
            while (span > 0) {
                const int step = (span + 63) >> 6;
                const int k = lo + (lane + 1) * step;
                const bool ok = k <= lo + span && cumW[a1 + k] - W0 <= (long long)M;
                const int c = __popcll(__builtin_amdgcn_ballot_w64(ok));  // a prefix of the probes fits
                const int hi = lo + span;
                lo += c * step;
                span = min(hi, lo + step - 1) - lo;
            }
            const int K = lo;
            if (K < 1) {  // cannot happen for well-formed input; never spin
                if (lane == 0) atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
                break;
            }
            int bk = 0;
            if (small1) {
                unsigned bs = 0;
                for (int k = lane + 1; k <= K; k += 64) {
                    const unsigned Sk = (unsigned)(cumG[a1 + k] - G0);
                    if (better_small(Sk, k, bs, bk, tie_rule)) { bs = Sk; bk = k; }
                }
                row_best_small(bs, bk, tie_rule);
                for (int d = 16; d <= 32; d <<= 1) {
                    const unsigned oS = (unsigned)__shfl_xor((int)bs, d);
                    const int ok = __shfl_xor(bk, d);
                    if (better_small(oS, ok, bs, bk, tie_rule)) { bs = oS; bk = ok; }
                }
            } else {
                long long bS = 0;
                for (int k = lane + 1; k <= K; k += 64) {
                    const long long Sk = cumG[a1 + k] - G0;
                    if (better(Sk, k, bS, bk, tie_rule)) { bS = Sk; bk = k; }
                }
                for (int d = 1; d < 64; d <<= 1) {  // (exchanges both ways: every lane ends with the winner)
                    const long long oS = __shfl_xor(bS, d);
                    const int ok = __shfl_xor(bk, d);
                    if (better(oS, ok, bS, bk, tie_rule)) { bS = oS; bk = ok; }
                }
            }
            const int kstar = __builtin_amdgcn_readfirstlane(bk);
            if (lane == 0) ends[nb1] = a1 + kstar;
            for (int i = lane; i < kstar; i += 64) batch_of[sorted[a1 + i]] = nb1;
            a1 += kstar;
            ++nb1;
        }
        if (lane == 0) *num_batches_out = nb1;
        for (int b = lane; b < nb1; b += 64) {
            const int lo = b == 0 ? 0 : ends[b - 1], hi = ends[b];
            batch_end_out[b] = hi;
            const double k = (double)(hi - lo);
            F_out[b] = (double)(cumG[hi] - cumG[lo]) / ((double)gb * k * k);
        }
        // the (o, id)-sorted ids by batch number (stable): `sorted` and the other sort buffer are free now
        const int *src1 = by_o;
        int *dst1 = alt, *oth1 = cur;
        auto key_b1 = [batch_of](int id) { return batch_of[id]; };
        for (int shift = 0; shift < bits_of(nb1 - 1); shift += 8) {
            radix_pass_wave(src1, dst1, n, shift, key_b1, L.radix.hist);
            src1 = dst1;
            dst1 = oth1;
            oth1 = (int *)src1;
        }
        for (int i = lane; i < n; i += 64) order_out[i] = src1[i];
        return;
    }

    // ---- 4: batches
    const bool small = n < 65536 && cumG[n] < (1ll << 32);
    int a = 0, nb = 0;
    while (a < n) {
        const int rem = n - a;
        const long long W0 = cumW[a], S0 = cumS[a], G0 = cumG[a];
        // feasible extent K: the longest prefix within the budget (feasibility is monotone in k)
        int K = count_fitting(rem, [&](long long k) { return cumW[a + k] - W0; }, M, L, 0);  // sum of peaks <= M
        if (PROFILE && K >= 1 && K < rem) {
            // Started together, the prefix must stay within M at every completion time.  The sum of
            // peaks bounds that memory from above (so K is feasible), and the memory at the earliest
            // completion is at least sum (s_i + 1) (so nothing beyond hi is); bisect in between.
            int lo = K;
            int hi = count_fitting(rem, [&](long long k) { return (cumW[a + k] - W0) - (cumS[a + k] - S0) + k; }, M, L, 1);
            const int *list = by_o;  // ascending o, holds every member of any prefix probed
            int len = n;
            if (!IN_LDS && lo < hi) {
                // Many requests: a probe through all of them costs more than the batch is worth, and hi
                // (nothing beyond it fits even at the earliest completion) can lie far above the answer
                // when decode lengths are long.  So the candidates of this batch are sorted by o once
                // (stable passes, two spare arrays) and serve every probe; and only the first `cap` of
                // them, doubled while all of them fit.
                int cap = min(hi, lo + max(lo, TPB));
                for (;;) {
                    const int *src = sorted + a;
                    int *dst = alt, *oth = pos_w + (((size_t)n + 64) & ~(size_t)63);
                    for (int shift = 0; shift < bits_of(omax); shift += 8) {
                        radix_pass(src, dst, cap, shift, key_o, L.radix);
                        src = dst;
                        dst = oth;
                        oth = (int *)src;
                    }
                    list = src;
                    len = cap;
                    if (cap < hi) {
                        if (profile_fits(len, a, cap, s, o, list, pos_w, M, L)) {
                            lo = cap;
                            cap = min(hi, 2 * cap);
                            continue;
                        }
                        hi = cap - 1;
                    }
                    break;
                }
            }
            while (lo < hi) {
                const int mid = lo + (hi - lo + 1) / 2;
                if (profile_fits(len, a, mid, s, o, list, pos_w, M, L)) lo = mid;
                else hi = mid - 1;
            }
            K = lo;
        }
        if (K < 1) {  // cannot happen for well-formed input; never spin
            if (tid == 0) atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            break;
        }
        long long bS = 0;
        int bk = 0;
        if (small) {  // every numerator below 2^32, every size below 2^16: 64-bit cross products, lane exchanges
            unsigned bs = 0;
            for (int k = tid + 1; k <= K; k += TPB) {
                const unsigned Sk = (unsigned)(cumG[a + k] - G0);
                if (better_small(Sk, k, bs, bk, tie_rule)) { bs = Sk; bk = k; }
            }
            if (wave * 64 < K) {  // (a wave without candidates leaves the arithmetic units to the others)
                row_best_small(bs, bk, tie_rule);
                for (int d = 16; d <= 32; d <<= 1) {
                    const unsigned oS = (unsigned)__shfl_xor((int)bs, d);
                    const int ok = __shfl_xor(bk, d);
                    if (better_small(oS, ok, bs, bk, tie_rule)) { bs = oS; bk = ok; }
                }
            }
            if (lane == 0) { L.red_S[wave] = bs; L.red_k[wave] = bk; }
            __syncthreads();
            if (wave == 0) {  // the waves' winners in the first row of lanes
                static_assert(NWAVES == 16, "one 16-lane row holds the waves' winners");
                bs = (unsigned)L.red_S[lane & 15];
                bk = L.red_k[lane & 15];
                row_best_small(bs, bk, tie_rule);
                if (lane == 0) {
                    L.best_k = bk;
                    ends[nb] = a + bk;
                }
            }
        } else {
            for (int k = tid + 1; k <= K; k += TPB) {
                const long long Sk = cumG[a + k] - G0;
                if (better(Sk, k, bS, bk, tie_rule)) { bS = Sk; bk = k; }
            }
            if (wave * 64 < K) {
                for (int d = 32; d > 0; d >>= 1) {
                    const long long oS = __shfl_down(bS, d);
                    const int ok = __shfl_down(bk, d);
                    if (better(oS, ok, bS, bk, tie_rule)) { bS = oS; bk = ok; }
                }
            }
            if (lane == 0) { L.red_S[wave] = bS; L.red_k[wave] = bk; }
            __syncthreads();
            if (wave == 0) {  // the waves' winners, one per lane
                bS = lane < NWAVES ? L.red_S[lane] : 0;
                bk = lane < NWAVES ? L.red_k[lane] : 0;
                for (int d = NWAVES / 2; d > 0; d >>= 1) {
                    const long long oS = __shfl_down(bS, d);
                    const int ok = __shfl_down(bk, d);
                    if (better(oS, ok, bS, bk, tie_rule)) { bS = oS; bk = ok; }
                }
                if (lane == 0) {
                    L.best_k = bk;
                    ends[nb] = a + bk;
                }
            }
        }
        __syncthreads();
        // (no barrier closes the iteration: the next one passes a barrier before it writes what is read here)
        const int kstar = L.best_k;
        for (int i = tid; i < kstar; i += TPB) batch_of[sorted[a + i]] = nb;
        a += kstar;
        ++nb;
    }
    __threadfence_block();
    __syncthreads();
    // metric values of the batches: one fp64 division each
    for (int b = tid; b < nb; b += TPB) {
        const int lo = b == 0 ? 0 : ends[b - 1], hi = ends[b];
        if constexpr (IN_LDS) batch_end_out[b] = hi;
        const double k = (double)(hi - lo);
        F_out[b] = (double)(cumG[hi] - cumG[lo]) / ((double)gb * k * k);
    }
    if (tid == 0) *num_batches_out = nb;
    __threadfence_block();
    __syncthreads();

    // ---- 5: order the (o, id)-sorted ids by batch number (stable)
    int *src = by_o;
    int *dst = (cur == buf0) ? buf1 : buf0;  // `sorted` is no longer needed after step 4, but keep it intact
    int *other = (int *)cur;
    auto key_b = [batch_of](int id) { return batch_of[id]; };
    bool first = true;
    for (int shift = 0; shift < bits_of(nb - 1); shift += 8) {
        radix_pass(src, dst, n, shift, key_b, L.radix);
        if (first) { src = dst; dst = other; first = false; }
        else { int *t = src; src = dst; dst = t; }
    }
    for (int i = tid; i < n; i += TPB) order_out[i] = src[i];
}

}  // namespace

size_t kvs_sortedF_scratch_bytes(int32_t n)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    return np * (8 * sizeof(int) + 3 * sizeof(long long)) + 256;
}

int kvs_launch_sortedF(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t ga, int32_t gb,
                       int32_t tie_rule, int32_t feas_mode, int32_t *order_out, int32_t *batch_end_out, double *F_out, int32_t *num_batches_out,
                       void *scratch, int32_t *d_words, hipStream_t st)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    long long *cumW = (long long *)scratch;
    long long *cumS = cumW + np;
    long long *cumG = (ga == 0 && gb == 1) ? cumS : cumS + np;
    int *buf0 = (int *)(cumS + 2 * np);
    int *buf1 = buf0 + np;
    int *by_o = buf1 + np;
    int *batch_of = by_o + np;
    int *pos_w = batch_of + np;
    const size_t arrays = kvs_sortedF_scratch_bytes(n);
    const int profile = feas_mode == KVSCHED_FEAS_PROFILE ? 1 : 0;
    constexpr size_t kLdsPerWorkgroup = 160 * 1024;
    if (arrays + sizeof(Lds) <= kLdsPerWorkgroup) {
        // more than 64 KB of LDS in all: the kernel's limit on the dynamic part is raised first, as far as needed
        static size_t granted[2] = {64 * 1024 - sizeof(Lds), 64 * 1024 - sizeof(Lds)};
        if (arrays > granted[profile]) {
            const void *fn = profile ? (const void *)sortedF_kernel<true, true> : (const void *)sortedF_kernel<true, false>;
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)arrays) != hipSuccess)
                return KVSCHED_EHIP;
            granted[profile] = arrays;
        }
        if (profile)
            hipLaunchKernelGGL((sortedF_kernel<true, true>), dim3(1), dim3(TPB), arrays, st, n, s, o, M, ga, gb, tie_rule,
                               feas_mode, order_out, batch_end_out, F_out, num_batches_out, buf0, buf1, by_o, cumW,
                               cumS, cumG, batch_of, pos_w, d_words);
        else
            hipLaunchKernelGGL((sortedF_kernel<true, false>), dim3(1), dim3(TPB), arrays, st, n, s, o, M, ga, gb, tie_rule,
                               feas_mode, order_out, batch_end_out, F_out, num_batches_out, buf0, buf1, by_o, cumW,
                               cumS, cumG, batch_of, pos_w, d_words);
    } else if (profile) {
        hipLaunchKernelGGL((sortedF_kernel<false, true>), dim3(1), dim3(TPB), 0, st, n, s, o, M, ga, gb, tie_rule,
                           feas_mode, order_out, batch_end_out, F_out, num_batches_out, buf0, buf1, by_o, cumW, cumS,
                           cumG, batch_of, pos_w, d_words);
    } else {
        hipLaunchKernelGGL((sortedF_kernel<false, false>), dim3(1), dim3(TPB), 0, st, n, s, o, M, ga, gb, tie_rule,
                           feas_mode, order_out, batch_end_out, F_out, num_batches_out, buf0, buf1, by_o, cumW, cumS,
                           cumG, batch_of, pos_w, d_words);
    }
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
