// Scheduling under online arrivals (Section 6, "Heuristics under Online Arrival"; Section 7,
// "Experiment under Online Poisson Arrivals"): many independent request streams at once, ONE
// 64-lane WAVEFRONT PER STREAM, the whole policy on the device.
//
// Per stream, iteration t = 0, 1, 2, ...:
//   1. requests with a_i <= t join the backlog and the end of the cached priority list;
//   2. when a refresh is due the planner re-orders the whole backlog into a new cached list;
//   3. list entries are admitted from the front while Eq. (1) holds beside the running requests,
//      stopping at the first that does not fit.
// Iterations that cannot change anything are not executed one by one: with an empty backlog the
// stream moves to the next arrival, and when the head of the list does not fit, to the earliest of
// the first round at which it might, the next arrival and the next refresh that could change the
// list (refreshes of an unchanged backlog reproduce the list and are only counted).
//
// A stream is a chain of small dependent steps (a refresh of the paper's setting is some
// twenty batches and a hundred exchanges on fifty requests), so nothing is gained by putting
// more lanes on one stream; the chip is filled by running thousands of streams side by side.
// One wavefront per stream needs no workgroup barrier anywhere: every decision is a ballot or a
// wave reduction, and the LDS a stream needs (24 KB in the smallest size class) lets six
// streams share a compute unit.
//
// State of a stream, all in LDS:
//   * the backlog as an array of 64-bit keys sorted in the planner's order; a key packs
//     (s+o, o, id) so that sorting, the fallback order and the lengths needed at admission all
//     come from the one word.  Arrivals are merged in (rank among the newcomers + binary search
//     in the backlog), admitted requests are struck out by a compaction; two copies alternate;
//   * the cached list: a circular buffer of the same keys;
//   * the running requests' future memory P(tau) for the next H rounds in a ring of H slots
//     (H = power of two >= longest decode length; the slot of round t is cleared at iteration t
//     before anything is admitted, so it can stand for round t + H); an attempt checks its o rounds 64 at
//     a time and ends in one ballot;
//   * the look-ahead window of the Sorted-F-Online planner: Phase 1 of Algorithm 1 with Local
//     Swap Search batches, sorted place 64 r + lane in row r of the lane's registers (greedy fill
//     = longest prefix by a saturating wave scan; an exchange step = exclusive prefix minimum of
//     o over non-members, one binary search per member of the first rows, two ballots).
#include "kvsched_internal.h"
#include "phase1_util.h"

#include <limits.h>

namespace {

typedef unsigned long long u64;

constexpr int OMAXW = KVSCHED_ONLINE_MAX_WINDOW;
constexpr int OMAXCOUNT = 1 << 20;  // ids are 20-bit fields of the keys

template <int QCAP, int HCAP>
struct StreamLds {
    static constexpr int WCAP = QCAP < OMAXW ? QCAP : OMAXW;
    u64 qa[QCAP];
    u64 qb[QCAP];
    u64 list[QCAP];
    u64 wk[WCAP];  // the planner's window, compacted after every batch
    int ring[HCAP];
    unsigned dead[QCAP / 32];
};

// (s+o, o, id) <-> key.  Fields: s+o < 2^30 (30 bits), o <= 2^13 (14 bits), id < 2^20; the planner's
// sort order decides which field is most significant.
struct Codec {
    int w_shift, o_shift, id_shift;
    __device__ explicit Codec(int planner)
    {
        if (planner == KVSCHED_PLANNER_ARRIVAL) { id_shift = 44; w_shift = 14; o_shift = 0; }        // (id)
        else if (planner == KVSCHED_PLANNER_SHORTEST_DECODE) { o_shift = 50; id_shift = 30; w_shift = 0; }  // (o, id)
        else { w_shift = 34; o_shift = 20; id_shift = 0; }                                           // (s+o, o, id)
    }
    __device__ __forceinline__ u64 make(int w, int o, int id) const
    {
        return ((u64)w << w_shift) | ((u64)o << o_shift) | ((u64)id << id_shift);
    }
    __device__ __forceinline__ int size(u64 k) const { return (int)((k >> w_shift) & 0x3fffffffu); }
    __device__ __forceinline__ int decode(u64 k) const { return (int)((k >> o_shift) & 0x3fffu); }
    __device__ __forceinline__ int id(u64 k) const { return (int)((k >> id_shift) & 0xfffffu); }
};

// ------------------------------------------------------------------ wavefront primitives
// All 64 lanes are active wherever these are called (control flow is uniform per stream).

__device__ __forceinline__ void wave_sync()
{
    // LDS traffic of one wavefront is served in order; this keeps the compiler from moving
    // accesses across a point where lanes read what other lanes wrote
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

__device__ __forceinline__ u64 lanes_below()
{
    return (1ull << lane_id()) - 1ull;
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ u64 uni64(u64 v)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
    return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 lane_u64(u64 v, int lane)  // lane is uniform
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

// DPP moves: lanes whose source lies outside the pattern (or whose row is masked off) get `idle`.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp(int idle, int v)
{
    return __builtin_amdgcn_update_dpp(idle, v, CTRL, ROW_MASK, 0xf, false);
}
constexpr int DPP_QUAD_1032 = 0xB1, DPP_QUAD_2301 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118;
constexpr int DPP_BCAST15 = 0x142, DPP_BCAST31 = 0x143;  // last lane of a row -> the next row(s)
constexpr int DPP_WAVE_SHR1 = 0x138;                      // every lane from the lane below, across rows

// After these four steps every lane of a 16-lane row holds the row's total.
#define KVS_ROW_BUTTERFLY(v, OP)                      \
    v = OP(v, dpp<DPP_QUAD_1032>(v, v));              \
    v = OP(v, dpp<DPP_QUAD_2301>(v, v));              \
    v = OP(v, dpp<DPP_HALF_MIRROR>(v, v));            \
    v = OP(v, dpp<DPP_MIRROR>(v, v));

__device__ __forceinline__ int op_add(int a, int b) { return a + b; }
__device__ __forceinline__ int op_max(int a, int b) { return max(a, b); }

__device__ __forceinline__ int wave_sum(int v)
{
    KVS_ROW_BUTTERFLY(v, op_add)
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

__device__ __forceinline__ long long wave_sum64(long long v)
{
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    return (long long)uni64((u64)v);
}

__device__ __forceinline__ int wave_max(int v)
{
    KVS_ROW_BUTTERFLY(v, op_max)
    return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// Inclusive prefix scans over the 64 lanes: within rows by shifts of 1, 2, 4, 8, then the last
// lane of row 0 / 2 into rows 1 / 3 and the last lane of row 1 into rows 2 and 3.

// sums of non-negative values, saturating at cap (cap <= 2^30)
__device__ __forceinline__ unsigned wave_incl_add_sat(unsigned v, unsigned cap)
{
    v = min(v + (unsigned)dpp<DPP_ROW_SHR1>(0, (int)v), cap);
    v = min(v + (unsigned)dpp<DPP_ROW_SHR2>(0, (int)v), cap);
    v = min(v + (unsigned)dpp<DPP_ROW_SHR4>(0, (int)v), cap);
    v = min(v + (unsigned)dpp<DPP_ROW_SHR8>(0, (int)v), cap);
    v = min(v + (unsigned)dpp<DPP_BCAST15, 0xa>(0, (int)v), cap);
    v = min(v + (unsigned)dpp<DPP_BCAST31, 0xc>(0, (int)v), cap);
    return v;
}

// inclusive prefix minimum
__device__ __forceinline__ int wave_incl_min(int v)
{
    v = min(v, dpp<DPP_ROW_SHR1>(INT_MAX, v));
    v = min(v, dpp<DPP_ROW_SHR2>(INT_MAX, v));
    v = min(v, dpp<DPP_ROW_SHR4>(INT_MAX, v));
    v = min(v, dpp<DPP_ROW_SHR8>(INT_MAX, v));
    v = min(v, dpp<DPP_BCAST15, 0xa>(INT_MAX, v));
    v = min(v, dpp<DPP_BCAST31, 0xc>(INT_MAX, v));
    return v;
}

__device__ __forceinline__ int first_lane(u64 ballot) { return __ffsll((long long)ballot) - 1; }

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

// first index of wk[0..n) (keys ascending in s+o) whose s+o exceeds lim
__device__ __forceinline__ int upper_bound_size(const u64 *wk, int n, int lim)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((int)(wk[mid] >> 34) <= lim) lo = mid + 1;
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
// wk: WCAP keys of working storage; tmp: an idle array of >= max(wn + 1 ints, wn keys).
template <int WCAP>
__device__ void plan_window(const u64 *src, int wn, int M, u64 *wk, u64 *tmp, u64 *list)
{
    constexpr int RMAX = WCAP / 64;
    constexpr u64 LOW34 = (1ull << 34) - 1;  // (o, id) of a key
    const int lane = lane_id();
    int *pm = (int *)tmp;  // pm[j] = least o among non-members at places < j, j = 0..m
    u64 *bkey = tmp;       // the batch's keys (after the exchanges, pm is no longer needed)

    for (int i = lane; i < wn; i += 64) wk[i] = src[i];
    wave_sync();

    int m = wn, outpos = 0;
    while (m > 0) {
        const int R = (m + 63) >> 6;
        // this lane's places 64 r + lane
        int wreg[RMAX], oreg[RMAX];
        unsigned valid = 0, mem = 0;  // bit r: place exists / is in the batch
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            wreg[r] = 0;
            oreg[r] = INT_MAX;
            if (r < R && 64 * r + lane < m) {
                const u64 k = wk[64 * r + lane];
                wreg[r] = (int)(k >> 34);
                oreg[r] = (int)((k >> 20) & 0x3fffu);
                valid |= 1u << r;
            }
        }
        // greedy fill: sizes ascend, so "add while it fits" is the longest prefix within M
        const unsigned cap = (unsigned)M + 1u;
        unsigned carry = 0;
        int K = 0, memsum = 0;
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            if (r < R) {
                const unsigned incl = min(wave_incl_add_sat((unsigned)wreg[r], cap) + carry, cap);
                const bool in = ((valid >> r) & 1u) && incl <= (unsigned)M;
                if (in) mem |= 1u << r;
                const u64 bal = __builtin_amdgcn_ballot_w64(in);
                K += __popcll(bal);
                memsum += wave_sum(in ? wreg[r] : 0);
                carry = (unsigned)__builtin_amdgcn_readlane((int)incl, 63);
            }
        }

        // Small batches in a window of at most two rows (the paper's online setting: a few requests
        // per batch, some tens waiting) are searched as the pseudo-code scans: members in sorted
        // order, each against all non-members at once from the registers.  Otherwise every member
        // is tested at once through the prefix minimum of o over the non-members.
        const bool by_member = R <= 2 && K <= 32;
        for (;;) {  // one exchange per turn; every exchange lowers the batch's sum of o
            const int slack = M - memsum;
            int astar = -1, bstar = -1, wa = 0, wb = 0;
            if (by_member) {
#pragma unroll
                for (int ra = 0; ra < 2; ++ra) {
                    if (ra < R && astar < 0) {
                        u64 todo = __builtin_amdgcn_ballot_w64((mem >> ra) & 1u);
                        while (todo != 0 && astar < 0) {
                            const int la = first_lane(todo);
                            todo &= todo - 1;
                            const int w_out = __builtin_amdgcn_readlane(wreg[ra], la);
                            const int o_out = __builtin_amdgcn_readlane(oreg[ra], la);
#pragma unroll
                            for (int rb = 0; rb < 2; ++rb) {
                                if (rb < R && astar < 0) {
                                    const bool ok = ((valid >> rb) & 1u) && !((mem >> rb) & 1u) &&
                                                    wreg[rb] <= w_out + slack && oreg[rb] < o_out;
                                    const u64 bal = __builtin_amdgcn_ballot_w64(ok);
                                    if (bal != 0) {
                                        astar = 64 * ra + la;
                                        bstar = 64 * rb + first_lane(bal);
                                        wa = w_out;
                                        wb = __builtin_amdgcn_readlane(wreg[rb], first_lane(bal));
                                    }
                                }
                            }
                        }
                    }
                }
                if (astar < 0) break;
            } else {
                int run = INT_MAX, oa = 0;
#pragma unroll
                for (int r = 0; r < RMAX; ++r) {
                    if (r < R) {
                        const bool out = ((valid >> r) & 1u) && !((mem >> r) & 1u);
                        const int upto = wave_incl_min(out ? oreg[r] : INT_MAX);
                        pm[64 * r + lane] = min(dpp<DPP_WAVE_SHR1>(INT_MAX, upto), run);  // lane 0: run alone
                        run = min(run, __builtin_amdgcn_readlane(upto, 63));
                    }
                }
                if (lane == 0) pm[m] = run;
                wave_sync();
                // a member has a partner iff some non-member that still fits has a smaller o; those
                // that fit are the places before the first size above w + slack
#pragma unroll
                for (int r = 0; r < RMAX; ++r) {
                    if (r < R && astar < 0) {
                        const bool is_mem = (mem >> r) & 1u;
                        if (__builtin_amdgcn_ballot_w64(is_mem) != 0) {
                            bool has = false;
                            if (is_mem) {
                                const int ub = upper_bound_size(wk, m, wreg[r] + slack);
                                has = pm[ub] < oreg[r];
                            }
                            const u64 bal = __builtin_amdgcn_ballot_w64(has);
                            if (bal != 0) {
                                astar = 64 * r + first_lane(bal);
                                wa = __builtin_amdgcn_readlane(wreg[r], first_lane(bal));
                                oa = __builtin_amdgcn_readlane(oreg[r], first_lane(bal));
                            }
                        }
                    }
                }
                wave_sync();
                if (astar < 0) break;
#pragma unroll
                for (int r = 0; r < RMAX; ++r) {
                    if (r < R && bstar < 0) {
                        const bool ok = ((valid >> r) & 1u) && !((mem >> r) & 1u) && oreg[r] < oa;
                        const u64 bal = __builtin_amdgcn_ballot_w64(ok);
                        if (bal != 0) {
                            bstar = 64 * r + first_lane(bal);
                            wb = __builtin_amdgcn_readlane(wreg[r], first_lane(bal));
                        }
                    }
                }
                if (bstar < 0) break;  // cannot happen: pm[] promised a partner before the bound
            }
            memsum += wb - wa;
            if (lane == (astar & 63)) mem &= ~(1u << (astar >> 6));
            if (lane == (bstar & 63)) mem |= 1u << (bstar >> 6);
        }

        // the batch in nondecreasing o, ties by id: rank of each member among the members
        int nmem = 0;
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            if (r < R) {
                const bool is_mem = (mem >> r) & 1u;
                const u64 bal = __builtin_amdgcn_ballot_w64(is_mem);
                if (is_mem) bkey[nmem + __popcll(bal & lanes_below())] = wk[64 * r + lane];
                nmem += __popcll(bal);
            }
        }
        wave_sync();
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            if (r < R) {
                const bool is_mem = (mem >> r) & 1u;
                if (__builtin_amdgcn_ballot_w64(is_mem) != 0) {
                    const u64 mine = wk[64 * r + lane];
                    const u64 me = mine & LOW34;
                    int rank = 0;
                    for (int j = 0; j < K; ++j) rank += ((bkey[j] & LOW34) < me) ? 1 : 0;
                    if (is_mem) list[outpos + rank] = mine;
                }
            }
        }
        wave_sync();
        // what remains closes up in place, still sorted: row by row, each row read before it is
        // written, and never written beyond itself
        int kept = 0;
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            if (r < R) {
                const bool keep = ((valid >> r) & 1u) && !((mem >> r) & 1u);
                const u64 k = ((valid >> r) & 1u) ? wk[64 * r + lane] : 0;
                const u64 bal = __builtin_amdgcn_ballot_w64(keep);
                wave_sync();
                if (keep) wk[kept + __popcll(bal & lanes_below())] = k;
                kept += __popcll(bal);
                wave_sync();
            }
        }
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
    int32_t H;    // ring slots: power of two >= longest decode length
    int32_t cap;  // the caller's bound on the backlog of a stream
    int32_t out_len;
    int32_t *completion_out;
    int64_t *stats_out;  // [B][4]
    int32_t *d_words;
    const int32_t *by_cost;  // [B] stream numbers in ascending order of estimated work, or NULL
};

// A batch takes as long as its longest stream, which should therefore not start last: the streams are
// taken in descending order of a rough measure of their work, requests x 8 for Sorted-F-Online (every
// refresh plans a window by Local Swap Search), requests x 1 for the planners that only sort.
// One workgroup: stable 8-bit radix passes on that measure.
__global__ __launch_bounds__(1024) void online_order_kernel(const int32_t *streams, int32_t B, int32_t *tmp, int32_t *sorted)
{
    __shared__ RadixLds<1024> L;
    __shared__ int sh_max[16];
    auto cost = [streams](int b) {
        const int count = streams[8 * (size_t)b + 1], planner = streams[8 * (size_t)b + 2];
        const int c = min(max(count, 0), 1 << 27);
        return planner == KVSCHED_PLANNER_SORTED_F ? 8 * c : c;
    };
    int mx = 0;
    for (int i = threadIdx.x; i < B; i += 1024) mx = max(mx, cost(i));
    for (int d = 32; d > 0; d >>= 1) mx = max(mx, __shfl_xor(mx, d));
    if ((threadIdx.x & 63) == 0) sh_max[threadIdx.x >> 6] = mx;
    __syncthreads();
    for (int w = 0; w < 16; ++w) mx = max(mx, sh_max[w]);
    const int passes = (bits_of(mx) + 7) / 8;
    int *src = (passes & 1) ? tmp : sorted, *dst = (passes & 1) ? sorted : tmp;  // the last pass lands in `sorted`
    for (int i = threadIdx.x; i < B; i += 1024) src[i] = i;
    __threadfence_block();
    __syncthreads();
    for (int pass = 0; pass < passes; ++pass) {
        radix_pass<1024>(src, dst, B, 8 * pass, cost, L);
        __threadfence_block();
        __syncthreads();
        int *sw = src; src = dst; dst = sw;
    }
}

template <int QCAP, int HCAP>
__global__ __launch_bounds__(64) void online_kernel(OnlineParams p)
{
    typedef StreamLds<QCAP, HCAP> Lds;
    __shared__ Lds L;
    constexpr int QM = QCAP - 1;
    const int lane = lane_id();
    const int b = p.by_cost ? uni(p.by_cost[p.B - 1 - (int)blockIdx.x]) : (int)blockIdx.x;  // most work first
    const int32_t *d = p.streams + 8 * (size_t)b;
    const int begin = uni(d[0]), count = uni(d[1]), planner = uni(d[2]), period = uni(d[3]), window = uni(d[4]);
    const int rnum = uni(d[5]), rden = uni(d[6]), outb = uni(d[7]);
    int64_t *stats = p.stats_out + 4 * (size_t)b;
    const bool bad_desc = begin < 0 || count < 0 || count > OMAXCOUNT || (long long)begin + count > p.N ||
                          planner < 0 || planner > KVSCHED_PLANNER_SORTED_F || period < 1 || window < 0 ||
                          window > OMAXW || rnum < 0 || rden < 0 || outb < 0 ||
                          (long long)outb + count > p.out_len;
    if (bad_desc) {
        if (lane == 0) {
            atomicOr(&p.d_words[KVS_W_STATUS], KVSCHED_DEV_BAD_STREAM);
            stats[0] = stats[1] = stats[2] = stats[3] = -1;
        }
        return;
    }
    if (count == 0) {
        if (lane == 0) stats[0] = stats[1] = stats[2] = stats[3] = 0;
        return;
    }
    const int H = p.H, HM = H - 1, M = p.M;
    const int32_t *a = p.a + begin, *s = p.s + begin, *o = p.o + begin;
    int32_t *cout = p.completion_out + outb;
    const Codec codec(planner);

    for (int i = lane; i < H; i += 64) L.ring[i] = 0;
    for (int i = lane; i < QCAP / 32; i += 64) L.dead[i] = 0;
    wave_sync();

    u64 *cur = L.qa, *oth = L.qb;
    int t = 0;
    int q = 0;             // backlog size = entries of the cached list
    int head = 0;          // list entries are list[(head + i) & QM], i < q
    int planned_left = 0;  // leading list entries that were placed by the last refresh
    int known = 0, started = 0;
    int t_plan = 0, backlog_at_plan = 0;
    long long refreshes = 0, sum_c = 0, sum_a = 0;  // sum_a: this lane's share
    int last_c = 0, max_backlog = 0;
    int next_a = uni(a[0]);
    int fault = 0;
    // No admission for H iterations in a row with a backlog is impossible (every running request
    // has left by then and a single request always fits), idle stretches are skipped in one step:
    // the budget below is never reached by well-formed input and bounds the loop otherwise.
    long long budget = (long long)count * (H + 2) + 16;

    while (started < count) {
        if (--budget < 0) { fault = KVSCHED_DEV_BAD_STREAM; break; }
        if (q == 0 && next_a > t) {  // nothing waits: jump to the next arrival, retiring the rounds passed
            const int span = min(next_a - t, H);
            for (int i = lane; i < span; i += 64) L.ring[(t + i) & HM] = 0;
            t = next_a;
            wave_sync();
        }
        // ---- 1. arrivals, up to 64 at a time
        while (known < count && next_a <= t) {
            const int idx = known + lane;
            const int aj = idx < count ? a[idx] : INT_MAX;
            const bool in = aj <= t;
            int sj = 1, oj = 1, bad = 0;
            if (in) {
                sj = s[idx];
                oj = o[idx];
                if (sj < 1 || oj < 1 || (long long)sj + oj > (long long)M) bad |= KVSCHED_DEV_BAD_LENGTH;
                if (oj > H) bad |= KVSCHED_DEV_O_MAX;
                if (aj < 0 || (idx > 0 && a[idx - 1] > aj)) bad |= KVSCHED_DEV_BAD_ARRIVAL;
            }
            const int kc = __popcll(__builtin_amdgcn_ballot_w64(in));
            for (int dlt = 32; dlt >= 1; dlt >>= 1) bad |= __shfl_xor(bad, dlt);
            fault = uni(bad);
            if (q + kc > p.cap) fault |= KVSCHED_DEV_BACKLOG;
            if (fault) break;
            // merge: a newcomer lands at (entries of the backlog before it) + (newcomers before it);
            // an entry of the backlog moves up by the newcomers before it
            const u64 key = in ? codec.make(sj + oj, oj, idx) : ~0ull;
            int rank = 0;
            for (int i = 0; i < kc; ++i) rank += (lane_u64(key, i) < key) ? 1 : 0;
            if (in) {
                oth[lower_bound_u64(cur, q, key) + rank] = key;
                L.list[(head + q + lane) & QM] = key;  // arrival order
                sum_a += aj;
            }
            for (int i0 = 0; i0 < q; i0 += 64) {
                const int i = i0 + lane;
                const u64 k = i < q ? cur[i] : 0;
                int nb = 0;
                for (int j = 0; j < kc; ++j) nb += (lane_u64(key, j) < k) ? 1 : 0;
                if (i < q) oth[i + nb] = k;
            }
            wave_sync();
            u64 *sw = cur; cur = oth; oth = sw;
            q += kc;
            known += kc;
            next_a = known < count ? uni(a[known]) : INT_MAX;
        }
        if (fault) break;
        max_backlog = max(max_backlog, q);

        // ---- 2. refresh of the cached order
        bool refreshed = false;
        int wn = 0;
        if (q > 0) {
            const long long newly = q - planned_left;
            const bool due = planned_left == 0 || t - t_plan >= period ||
                             (rden > 0 && newly * rden >= (long long)rnum * backlog_at_plan);
            if (due) {
                if (planner == KVSCHED_PLANNER_SORTED_F && window > 0) {
                    wn = min(window, q);
                    plan_window<Lds::WCAP>(cur, wn, M, L.wk, oth, L.list);
                }
                for (int i = wn + lane; i < q; i += 64) L.list[i] = cur[i];
                head = 0;
                planned_left = q;
                t_plan = t;
                backlog_at_plan = q;
                ++refreshes;
                refreshed = true;
                wave_sync();
            }
        }

        // ---- 3. admission of the longest feasible prefix of the list
        if (lane == 0) L.ring[t & HM] = 0;  // round t is behind every check from now on
        wave_sync();
        int adm = 0;
        int wait_to = t + 1;  // when the loop stops at a request: a round before which it cannot start
        while (adm < q) {
            const u64 key = uni64(L.list[(head + adm) & QM]);
            const int oo = codec.decode(key), id = codec.id(key);
            const int sr = codec.size(key) - oo;
            // round t + j rules out every start before t + min(excess, j): started later the request is
            // smaller at that round by as much, or no longer overlaps it
            int excess = 0;
            for (int j = lane + 1; j <= oo; j += 64) excess = max(excess, min(L.ring[(t + j) & HM] + sr + j - M, j));
            if (__builtin_amdgcn_ballot_w64(excess > 0) != 0) {
                wait_to = t + wave_max(excess);
                break;
            }
            for (int j = lane + 1; j <= oo; j += 64) L.ring[(t + j) & HM] += sr + j;
            if (lane == 0) cout[id] = t + oo;
            sum_c += t + oo;
            last_c = max(last_c, t + oo);
            ++adm;
        }
        // ---- the admitted requests leave the backlog
        if (adm > 0) {
            wave_sync();
            if (adm < q) {
                for (int j = lane; j < adm; j += 64) {
                    const int pos = lower_bound_u64(cur, q, L.list[(head + j) & QM]);
                    atomicOr(&L.dead[pos >> 5], 1u << (pos & 31));
                }
                wave_sync();
                int kept = 0;
                for (int i0 = 0; i0 < q; i0 += 64) {
                    const int i = i0 + lane;
                    const bool alive = i < q && !((L.dead[i >> 5] >> (i & 31)) & 1u);
                    const u64 bal = __builtin_amdgcn_ballot_w64(alive);
                    if (alive) oth[kept + __popcll(bal & lanes_below())] = cur[i];
                    kept += __popcll(bal);
                }
                wave_sync();
                for (int i = lane; i < (q + 31) / 32; i += 64) L.dead[i] = 0;
                u64 *sw = cur; cur = oth; oth = sw;
                wave_sync();
            }
            head = (head + adm) & QM;
            q -= adm;
            started += adm;
            planned_left = max(planned_left - adm, 0);
        }
        // ---- the rounds at which nothing can happen are passed in one step.  Until the request at
        // the head of the list can start (wait_to at the earliest), an iteration changes something
        // only if requests arrive or the list is re-planned.  Re-planning an unchanged backlog gives
        // the same list, so where the list is the plan of the present backlog (a refresh in this
        // iteration, and nothing admitted since unless the planner is a plain sort) the refreshes
        // of the rounds passed are only counted; otherwise the step ends at the next refresh due.
        int t_next = t + 1;
        if (q > 0) {
            t_next = min(wait_to, next_a);
            if (refreshed && (wn == 0 || adm == 0)) {
                const int every = (rden > 0 && rnum == 0) ? 1 : period;
                const int passed = (t_next - 1 - t) / every;
                if (passed > 0) {
                    refreshes += passed;
                    t_plan = t + passed * every;
                    backlog_at_plan = q;
                }
            } else {
                const bool grown = rden > 0 && (long long)(q - planned_left) * rden >= (long long)rnum * backlog_at_plan;
                const long long due_at = (planned_left == 0 || grown) ? t + 1 : max((long long)t + 1, (long long)t_plan + period);
                t_next = (int)min((long long)t_next, due_at);
            }
            for (int u = t + 1 + lane; u < t_next; u += 64) L.ring[u & HM] = 0;
        }
        t = t_next;
    }

    const long long sa = wave_sum64(sum_a);
    if (lane == 0) {
        if (fault) {
            atomicOr(&p.d_words[KVS_W_STATUS], fault);
            stats[0] = stats[1] = stats[2] = stats[3] = -1;
        } else {
            stats[0] = sum_c - sa;
            stats[1] = refreshes;
            stats[2] = last_c;
            stats[3] = max_backlog;
        }
    }
}

template <int QCAP, int HCAP>
int launch_online(const OnlineParams &p, hipStream_t st)
{
    hipLaunchKernelGGL((online_kernel<QCAP, HCAP>), dim3((unsigned)p.B), dim3(64), 0, st, p);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

}  // namespace

// Size classes (backlog capacity, ring slots) and the LDS a stream takes in each: 24 KB, 48 KB,
// 136 KB; the smallest that holds the caller's backlog bound and the longest decode is used.
int kvs_launch_online(int32_t B, const int32_t *streams, int32_t N, const int32_t *a, const int32_t *s,
                      const int32_t *o, int32_t M, int32_t backlog_cap, int32_t ring_slots, int32_t *completion_out,
                      int32_t out_len, int64_t *stats_out, int32_t *order_scratch, int32_t *d_words, hipStream_t st)
{
    if (ring_slots < 2 || (ring_slots & (ring_slots - 1)) || backlog_cap < 1) return KVSCHED_ERANGE;
    OnlineParams p;
    p.by_cost = nullptr;
    if (order_scratch) {  // [2 B]: the order, and the other buffer of the sort
        hipLaunchKernelGGL(online_order_kernel, dim3(1), dim3(1024), 0, st, streams, B, order_scratch + B, order_scratch);
        if (hipGetLastError() != hipSuccess) return KVSCHED_EHIP;
        p.by_cost = order_scratch;
    }
    p.B = B;
    p.streams = streams;
    p.N = N;
    p.a = a;
    p.s = s;
    p.o = o;
    p.M = M;
    p.H = ring_slots;
    p.cap = backlog_cap;
    p.out_len = out_len;
    p.completion_out = completion_out;
    p.stats_out = stats_out;
    p.d_words = d_words;
    if (backlog_cap <= 512 && ring_slots <= 2048) return launch_online<512, 2048>(p, st);
    if (backlog_cap <= 1024 && ring_slots <= 4096) return launch_online<1024, 4096>(p, st);
    if (backlog_cap <= KVSCHED_ONLINE_MAX_BACKLOG && ring_slots <= KVSCHED_ONLINE_MAX_O)
        return launch_online<KVSCHED_ONLINE_MAX_BACKLOG, KVSCHED_ONLINE_MAX_O>(p, st);
    return KVSCHED_ERANGE;
}
