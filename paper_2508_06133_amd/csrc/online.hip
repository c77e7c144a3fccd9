// Scheduling under online arrivals (Section 6, "Heuristics under Online Arrival"; Section 7,
// "Experiment under Online Poisson Arrivals"): many independent request streams at once, one
// workgroup of 256 threads per stream, the whole policy on the device.
//
// Per stream, iteration t = 0, 1, 2, ...:
//   1. requests with a_i <= t join the backlog and the end of the cached priority list;
//   2. when a refresh is due the planner re-orders the whole backlog into a new cached list;
//   3. list entries are admitted from the front while Eq. (1) holds beside the running requests,
//      stopping at the first that does not fit.
//
// State of a stream, all in LDS:
//   * the backlog as an array of 64-bit keys sorted in the planner's order; a key packs
//     (s+o, o, id) so that sorting, the fallback order and the lengths needed at admission all
//     come from the one word.  Arrivals are merged in (rank among the newcomers + binary search
//     in the backlog), admitted requests are struck out by a compaction; the two copies of the
//     array alternate;
//   * the cached list: a circular buffer of the same keys;
//   * the running requests' future memory P(tau) for the next H rounds in a ring of H slots
//     (H = power of two > longest decode length); an admission attempt checks its o rounds with
//     all threads and one barrier;
//   * the look-ahead window of the Sorted-F-Online planner lives in whichever backlog copy is
//     idle: Phase 1 of Algorithm 1 with Local Swap Search batches on at most 1024 requests,
//     4 sorted places per thread (greedy fill = longest prefix by a block scan; an exchange step
//     = exclusive prefix minimum of o over non-members + one binary search per member).
#include "kvsched_internal.h"

#include <limits.h>

namespace {

typedef unsigned long long u64;

constexpr int OT = 256;       // threads per stream
constexpr int ONW = OT / 64;  // wavefronts per stream
constexpr int OMAXQ = KVSCHED_ONLINE_MAX_BACKLOG;
constexpr int OMAXW = KVSCHED_ONLINE_MAX_WINDOW;
constexpr int OMAXH = KVSCHED_ONLINE_MAX_O + 1;
constexpr int OMAXCOUNT = 1 << 20;  // ids are 20-bit fields of the keys
static_assert((OMAXQ & (OMAXQ - 1)) == 0 && (OMAXH & (OMAXH - 1)) == 0, "ring sizes are powers of two");
static_assert(7 * OMAXW + 8 <= 2 * OMAXQ, "the planner's scratch must fit in one backlog copy");

struct OnlineLds {
    u64 qa[OMAXQ];
    u64 qb[OMAXQ];
    u64 list[OMAXQ];
    int ring[OMAXH];
    u64 newk[OT];   // keys of the arrivals being merged, in arrival order
    u64 newks[OT];  // the same keys sorted
    unsigned dead[OMAXQ / 32];
    long long part64[ONW];
    int part[ONW];
    int flag[3];
};

// (s+o, o, id) <-> key.  Fields: s+o < 2^30, o < 2^14, id < 2^20.
struct Codec {
    int planner;
    __device__ __forceinline__ u64 make(int w, int o, int id) const
    {
        if (planner == KVSCHED_PLANNER_ARRIVAL) return ((u64)id << 44) | ((u64)w << 14) | (u64)o;
        if (planner == KVSCHED_PLANNER_SHORTEST_DECODE) return ((u64)o << 50) | ((u64)id << 30) | (u64)w;
        return ((u64)w << 34) | ((u64)o << 20) | (u64)id;
    }
    __device__ __forceinline__ void split(u64 k, int &w, int &o, int &id) const
    {
        if (planner == KVSCHED_PLANNER_ARRIVAL) {
            id = (int)(k >> 44);
            w = (int)((k >> 14) & 0x3fffffffu);
            o = (int)(k & 0x3fffu);
        } else if (planner == KVSCHED_PLANNER_SHORTEST_DECODE) {
            o = (int)(k >> 50);
            id = (int)((k >> 30) & 0xfffffu);
            w = (int)(k & 0x3fffffffu);
        } else {
            w = (int)(k >> 34);
            o = (int)((k >> 20) & 0x3fffu);
            id = (int)(k & 0xfffffu);
        }
    }
};

// ---------------------------------------------------------------- block-wide primitives
// Every thread of the workgroup calls them; each ends with a barrier so that the partial
// arrays can be used again at once.

__device__ __forceinline__ int block_sum(int v, OnlineLds &L)
{
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    if ((threadIdx.x & 63) == 0) L.part[threadIdx.x >> 6] = v;
    __syncthreads();
    int tot = 0;
    for (int u = 0; u < ONW; ++u) tot += L.part[u];
    __syncthreads();
    return tot;
}

__device__ __forceinline__ int block_min(int v, OnlineLds &L)
{
    for (int d = 32; d >= 1; d >>= 1) v = min(v, __shfl_xor(v, d));
    if ((threadIdx.x & 63) == 0) L.part[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = INT_MAX;
    for (int u = 0; u < ONW; ++u) r = min(r, L.part[u]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ int block_or(int v, OnlineLds &L)
{
    for (int d = 32; d >= 1; d >>= 1) v |= __shfl_xor(v, d);
    if ((threadIdx.x & 63) == 0) L.part[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = 0;
    for (int u = 0; u < ONW; ++u) r |= L.part[u];
    __syncthreads();
    return r;
}

// exclusive prefix sum over the threads; *total = sum over all
__device__ __forceinline__ int block_excl_add(int v, int *total, OnlineLds &L)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
    for (int d = 1; d < 64; d <<= 1) {
        const int u = __shfl_up(inc, d);
        if (lane >= d) inc += u;
    }
    if (lane == 63) L.part[wave] = inc;
    __syncthreads();
    int off = 0, tot = 0;
    for (int u = 0; u < ONW; ++u) {
        const int x = L.part[u];
        if (u < wave) off += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return off + inc - v;
}

__device__ __forceinline__ long long block_excl_add64(long long v, OnlineLds &L)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    long long inc = v;
    for (int d = 1; d < 64; d <<= 1) {
        const long long u = __shfl_up(inc, d);
        if (lane >= d) inc += u;
    }
    if (lane == 63) L.part64[wave] = inc;
    __syncthreads();
    long long off = 0;
    for (int u = 0; u < wave; ++u) off += L.part64[u];
    __syncthreads();
    return off + inc - v;
}

// exclusive prefix minimum over the threads (INT_MAX for thread 0)
__device__ __forceinline__ int block_excl_min(int v, OnlineLds &L)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
    for (int d = 1; d < 64; d <<= 1) {
        const int u = __shfl_up(inc, d);
        if (lane >= d) inc = min(inc, u);
    }
    if (lane == 63) L.part[wave] = inc;
    int ex = __shfl_up(inc, 1);
    if (lane == 0) ex = INT_MAX;
    __syncthreads();
    for (int u = 0; u < wave; ++u) ex = min(ex, L.part[u]);
    __syncthreads();
    return ex;
}

// number of entries of the ascending array a[0..n) that are < key
__device__ __forceinline__ int lower_bound_u64(const u64 *a, int n, u64 key)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// first index of the ascending array a[0..n) whose entry is > lim
__device__ __forceinline__ int upper_bound_i32(const int *a, int n, int lim)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] <= lim) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// ------------------------------------------------- Sorted-F-Online's look-ahead window
//
// src[0..wn) are backlog keys in (s+o, o, id) order.  Phase 1 of Algorithm 1 with every batch
// chosen by Local Swap Search over these wn requests alone (budget M): greedy fill in that
// order, then the first improving exchange (members and non-members scanned in the sorted
// order; |X| is fixed, so F falls exactly when o_in < o_out) until none is left; the batch is
// emitted by (o, id) and removed.  Writes the wn keys to list[0..wn) in priority order.
// `wsc` is 7 * OMAXW + 8 ints of scratch.
__device__ void plan_window(const u64 *src, int wn, int M, int *wsc, u64 *list, OnlineLds &L)
{
    const int tid = threadIdx.x;
    int *ww = wsc, *wo = wsc + OMAXW, *wid = wsc + 2 * OMAXW;
    int *aw = wsc + 3 * OMAXW, *ao = wsc + 4 * OMAXW, *aid = wsc + 5 * OMAXW;
    int *pm = wsc + 6 * OMAXW;  // OMAXW + 1 entries
    u64 *bkey = (u64 *)aw;      // the batch's keys; aw and ao are idle while it is in use
    constexpr u64 LOW34 = (1ull << 34) - 1;  // (o, id) of a key

    for (int i = tid; i < wn; i += OT) {
        const u64 k = src[i];
        ww[i] = (int)(k >> 34);
        wo[i] = (int)((k >> 20) & 0x3fffu);
        wid[i] = (int)(k & 0xfffffu);
    }
    __syncthreads();

    int m = wn, outpos = 0;
    const int base = 4 * tid;  // this thread's four sorted places
    while (m > 0) {
        int w4[4], o4[4];
        bool v4[4], mem4[4];
        long long loc = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v4[e] = base + e < m;
            w4[e] = v4[e] ? ww[base + e] : 0;
            o4[e] = v4[e] ? wo[base + e] : INT_MAX;
            loc += w4[e];
        }
        // greedy fill: sizes ascend, so "add while it fits" is the longest prefix within M
        long long run = block_excl_add64(loc, L);
        int cnt = 0, wsum = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            run += w4[e];
            mem4[e] = v4[e] && run <= (long long)M;
            if (mem4[e]) { ++cnt; wsum += w4[e]; }
        }
        const int K = block_sum(cnt, L);
        int memsum = block_sum(wsum, L);

        for (;;) {  // one exchange per turn; every exchange lowers the batch's sum of o
            const int slack = M - memsum;
            int ex4[4], lm = INT_MAX;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ex4[e] = lm;
                if (v4[e] && !mem4[e]) lm = min(lm, o4[e]);
            }
            const int pre = block_excl_min(lm, L);
            const int all = block_min(lm, L);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (v4[e]) pm[base + e] = min(pre, ex4[e]);  // least o among non-members before this place
            if (tid == 0) pm[m] = all;
            __syncthreads();
            // a member has a partner iff some non-member that still fits has a smaller o; those
            // that fit are the places before the first size above w + slack
            int cand = INT_MAX;
#pragma unroll
            for (int e = 3; e >= 0; --e) {
                if (mem4[e]) {
                    const int ub = upper_bound_i32(ww, m, w4[e] + slack);
                    if (pm[ub] < o4[e]) cand = base + e;
                }
            }
            const int astar = block_min(cand, L);
            if (astar == INT_MAX) break;
            const int oa = wo[astar];
            int cb = INT_MAX;
#pragma unroll
            for (int e = 3; e >= 0; --e)
                if (v4[e] && !mem4[e] && o4[e] < oa) cb = base + e;
            const int bstar = block_min(cb, L);
            if (bstar == INT_MAX) break;  // cannot happen: pm[] promised a partner before the bound
            memsum += ww[bstar] - ww[astar];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (base + e == astar) mem4[e] = false;
                if (base + e == bstar) mem4[e] = true;
            }
        }

        // the batch in nondecreasing o, ties by id: rank of each member among the members
        int cntm = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) cntm += mem4[e] ? 1 : 0;
        int tot = 0;
        int offm = block_excl_add(cntm, &tot, L);
        u64 mine[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            mine[e] = 0;
            if (mem4[e]) {
                mine[e] = ((u64)w4[e] << 34) | ((u64)o4[e] << 20) | (u64)wid[base + e];
                bkey[offm++] = mine[e];
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (mem4[e]) {
                const u64 me = mine[e] & LOW34;
                int r = 0;
                for (int j = 0; j < K; ++j) r += ((bkey[j] & LOW34) < me) ? 1 : 0;
                list[outpos + r] = mine[e];
            }
        }
        __syncthreads();
        // what remains closes up, still sorted
        int cntn = 0, idk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            idk[e] = v4[e] ? wid[base + e] : 0;
            cntn += (v4[e] && !mem4[e]) ? 1 : 0;
        }
        int offn = block_excl_add(cntn, &tot, L);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (v4[e] && !mem4[e]) {
                aw[offn] = w4[e];
                ao[offn] = o4[e];
                aid[offn] = idk[e];
                ++offn;
            }
        }
        __syncthreads();
        for (int i = tid; i < m - K; i += OT) {
            ww[i] = aw[i];
            wo[i] = ao[i];
            wid[i] = aid[i];
        }
        __syncthreads();
        outpos += K;
        m -= K;
    }
}

// ------------------------------------------------------------------------ the stream kernel

struct OnlineParams {
    int32_t B;
    const int32_t *streams;  // [B][8]
    int32_t N;
    const int32_t *a, *s, *o;
    int32_t M;
    int32_t H;  // ring slots: power of two > longest decode length
    int32_t out_len;
    int32_t *completion_out;
    int64_t *stats_out;  // [B][4]
    int32_t *d_words;
};

__global__ __launch_bounds__(OT) void online_kernel(OnlineParams p)
{
    __shared__ OnlineLds L;
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int32_t *d = p.streams + 8 * (size_t)b;
    const int begin = d[0], count = d[1], planner = d[2], period = d[3], window = d[4];
    const int rnum = d[5], rden = d[6], outb = d[7];
    int64_t *stats = p.stats_out + 4 * (size_t)b;
    const bool bad_desc = begin < 0 || count < 0 || count > OMAXCOUNT || (long long)begin + count > p.N ||
                          planner < 0 || planner > KVSCHED_PLANNER_SORTED_F || period < 1 || window < 0 ||
                          window > OMAXW || rnum < 0 || rden < 0 || outb < 0 ||
                          (long long)outb + count > p.out_len;
    if (bad_desc) {
        if (tid == 0) {
            atomicOr(&p.d_words[KVS_W_STATUS], KVSCHED_DEV_BAD_STREAM);
            stats[0] = stats[1] = stats[2] = stats[3] = -1;
        }
        return;
    }
    if (count == 0) {
        if (tid == 0) stats[0] = stats[1] = stats[2] = stats[3] = 0;
        return;
    }
    const int H = p.H, HM = H - 1, M = p.M;
    const int32_t *a = p.a + begin, *s = p.s + begin, *o = p.o + begin;
    int32_t *cout = p.completion_out + outb;
    Codec codec{planner};

    for (int i = tid; i < H; i += OT) L.ring[i] = 0;
    for (int i = tid; i < OMAXQ / 32; i += OT) L.dead[i] = 0;
    if (tid < 3) L.flag[tid] = 0;
    __syncthreads();

    u64 *cur = L.qa, *oth = L.qb;
    int t = 0;
    int q = 0;                 // backlog size = entries of the cached list
    int head = 0;              // list entries are list[(head + i) & (OMAXQ - 1)], i < q
    int planned_left = 0;      // leading list entries that were placed by the last refresh
    int known = 0, started = 0;
    int t_plan = 0, backlog_at_plan = 0;
    long long refreshes = 0, sum_c = 0, sum_a = 0;  // sum_a: this thread's share
    int last_c = 0, max_backlog = 0;
    int next_a = a[0];
    int fault = 0;
    unsigned attempt = 0;
    // No admission for H iterations in a row with a backlog is impossible (every running request
    // has left by then and a single request always fits), idle stretches are skipped in one step:
    // the budget below is never reached by well-formed input and bounds the loop otherwise.
    long long budget = (long long)count * (H + 2) + 16;

    while (started < count) {
        if (--budget < 0) { fault = KVSCHED_DEV_BAD_STREAM; break; }
        if (q == 0 && next_a > t) {  // nothing waits: jump to the next arrival, retiring the rounds passed
            const int span = min(next_a - t, H);
            for (int i = tid; i < span; i += OT) L.ring[(t + i) & HM] = 0;
            t = next_a;
            __syncthreads();
        }
        // ---- 1. arrivals, up to 256 at a time
        while (known < count && next_a <= t) {
            const int idx = known + tid;
            const int aj = idx < count ? a[idx] : INT_MAX;
            const bool in = aj <= t;
            int sj = 1, oj = 1, bad = 0;
            if (in) {
                sj = s[idx];
                oj = o[idx];
                if (sj < 1 || oj < 1 || (long long)sj + oj > (long long)M) bad |= KVSCHED_DEV_BAD_LENGTH;
                if (oj >= H) bad |= KVSCHED_DEV_O_MAX;
                if (aj < 0 || (idx > 0 && a[idx - 1] > aj)) bad |= KVSCHED_DEV_BAD_ARRIVAL;
            }
            const int kc = block_sum(in ? 1 : 0, L);
            fault = block_or(bad, L);
            if (q + kc > OMAXQ) fault |= KVSCHED_DEV_BACKLOG;
            if (fault) break;
            // merge: a newcomer lands at (entries of the backlog before it) + (newcomers before it)
            const u64 key = in ? codec.make(sj + oj, oj, idx) : ~0ull;
            L.newk[tid] = key;
            __syncthreads();
            if (in) {
                int rank = 0;
                for (int i = 0; i < kc; ++i) rank += (L.newk[i] < key) ? 1 : 0;
                const int lb = lower_bound_u64(cur, q, key);
                oth[lb + rank] = key;
                L.newks[rank] = key;
                L.list[(head + q + tid) & (OMAXQ - 1)] = key;  // arrival order
                sum_a += aj;
            }
            __syncthreads();
            for (int i = tid; i < q; i += OT) {
                const u64 k = cur[i];
                oth[i + lower_bound_u64(L.newks, kc, k)] = k;
            }
            __syncthreads();
            u64 *sw = cur; cur = oth; oth = sw;
            q += kc;
            known += kc;
            next_a = known < count ? a[known] : INT_MAX;
        }
        if (fault) break;
        max_backlog = max(max_backlog, q);

        // ---- 2. refresh of the cached order
        if (q > 0) {
            const long long newly = q - planned_left;
            const bool due = planned_left == 0 || t - t_plan >= period ||
                             (rden > 0 && newly * rden >= (long long)rnum * backlog_at_plan);
            if (due) {
                int wn = 0;
                if (planner == KVSCHED_PLANNER_SORTED_F && window > 0) {
                    wn = min(window, q);
                    plan_window(cur, wn, M, (int *)oth, L.list, L);
                }
                for (int i = wn + tid; i < q; i += OT) L.list[i] = cur[i];
                head = 0;
                planned_left = q;
                t_plan = t;
                backlog_at_plan = q;
                ++refreshes;
                __syncthreads();
            }
        }

        // ---- 3. admission of the longest feasible prefix of the list
        if (tid == 0) L.ring[t & HM] = 0;  // round t is behind every check from now on
        int adm = 0;
        while (adm < q) {
            const u64 key = L.list[(head + adm) & (OMAXQ - 1)];
            int w, oo, id;
            codec.split(key, w, oo, id);
            const int sr = w - oo;
            const unsigned slot = attempt % 3u;
            if (tid == 0) L.flag[(attempt + 1u) % 3u] = 0;
            bool viol = false;
            for (int j = tid + 1; j <= oo; j += OT) viol |= L.ring[(t + j) & HM] + sr + j > M;
            if (viol) L.flag[slot] = 1;
            __syncthreads();
            ++attempt;
            if (L.flag[slot]) break;
            for (int j = tid + 1; j <= oo; j += OT) L.ring[(t + j) & HM] += sr + j;
            if (tid == 0) cout[id] = t + oo;
            sum_c += t + oo;
            last_c = max(last_c, t + oo);
            ++adm;
        }
        // ---- the admitted requests leave the backlog
        if (adm > 0) {
            if (adm < q) {
                for (int j = tid; j < adm; j += OT) {
                    const int pos = lower_bound_u64(cur, q, L.list[(head + j) & (OMAXQ - 1)]);
                    atomicOr(&L.dead[pos >> 5], 1u << (pos & 31));
                }
                __syncthreads();
                const int per = (q + OT - 1) / OT;
                const int lo = min(q, tid * per), hi = min(q, lo + per);
                int alive = 0;
                for (int i = lo; i < hi; ++i) alive += ((L.dead[i >> 5] >> (i & 31)) & 1u) ? 0 : 1;
                int tot = 0;
                int off = block_excl_add(alive, &tot, L);
                for (int i = lo; i < hi; ++i)
                    if (!((L.dead[i >> 5] >> (i & 31)) & 1u)) oth[off++] = cur[i];
                __syncthreads();
                for (int i = tid; i < (q + 31) / 32; i += OT) L.dead[i] = 0;
                u64 *sw = cur; cur = oth; oth = sw;
            }
            head = (head + adm) & (OMAXQ - 1);
            q -= adm;
            started += adm;
            planned_left = max(planned_left - adm, 0);
            __syncthreads();
        }
        ++t;
    }

    // sum of a_i over the stream: every thread holds a share
    for (int dlt = 32; dlt >= 1; dlt >>= 1) sum_a += __shfl_xor(sum_a, dlt);
    __syncthreads();
    if ((tid & 63) == 0) L.part64[tid >> 6] = sum_a;
    __syncthreads();
    if (tid == 0) {
        if (fault) {
            atomicOr(&p.d_words[KVS_W_STATUS], fault);
            stats[0] = stats[1] = stats[2] = stats[3] = -1;
        } else {
            long long sa = 0;
            for (int u = 0; u < ONW; ++u) sa += L.part64[u];
            stats[0] = sum_c - sa;
            stats[1] = refreshes;
            stats[2] = last_c;
            stats[3] = max_backlog;
        }
    }
}

}  // namespace

int kvs_launch_online(int32_t B, const int32_t *streams, int32_t N, const int32_t *a, const int32_t *s,
                      const int32_t *o, int32_t M, int32_t ring_slots, int32_t *completion_out, int32_t out_len,
                      int64_t *stats_out, int32_t *d_words, hipStream_t st)
{
    if (ring_slots < 2 || ring_slots > OMAXH || (ring_slots & (ring_slots - 1))) return KVSCHED_ERANGE;
    OnlineParams p;
    p.B = B;
    p.streams = streams;
    p.N = N;
    p.a = a;
    p.s = s;
    p.o = o;
    p.M = M;
    p.H = ring_slots;
    p.out_len = out_len;
    p.completion_out = completion_out;
    p.stats_out = stats_out;
    p.d_words = d_words;
    hipLaunchKernelGGL(online_kernel, dim3((unsigned)B), dim3(OT), 0, st, p);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
