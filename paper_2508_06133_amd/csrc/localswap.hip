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
// One step = one exclusive prefix-minimum scan, one ub() per member, two block-wide reductions.
//
// The step is a chain of dependent wave operations and barriers, so the whole construction runs in
// ONE small workgroup (LS_T threads = one wavefront per SIMD of a compute unit: with more waves the
// instructions every wave repeats share the issue ports and the step gets slower), each thread
// owning LS_E consecutive places of a tile and keeping its places of the first tile in registers.
// Once at most LS_CAP requests remain the working set lives in LDS, and while the sizes stay below
// LS_TABLE ub() is one read of a table rank[v] = number of remaining requests with w <= v (the
// arrangement is fixed within a batch, so the table is built once per batch); otherwise ub() is a
// binary search.
#include "phase1_util.h"

namespace {

constexpr int LS_T = 256;                // threads of the workgroup
constexpr int LS_E = 4;                  // consecutive places per thread in a tile
constexpr int LS_TILE = LS_T * LS_E;
constexpr int LS_NW = LS_T / 64;
constexpr int LS_CAP = 10240;            // remaining requests held in LDS (3 x 40 KB + the 32 KB table)
constexpr int LS_TABLE = 16384;          // sizes covered by the rank table
constexpr int LS_SMALL_VALUE = 1 << 15;  // values (o, or a s + b o) the straight-line steps can carry
constexpr int LS_INF = 0x7fffffff;
constexpr unsigned LS_MEMBER = 0x80000000u;  // membership flag kept in the sign bit of the o entry
constexpr int LS_NONE = 0x7fffffff;
constexpr unsigned long long LS_NO_KEY = ~0ull;

typedef __attribute__((address_space(3))) int lds_int;
typedef __attribute__((address_space(3))) const unsigned short lds_rank;

struct SwapLds {
    int wave_min[LS_NW];
    unsigned long long first_out[2];  // alternating slots: (place << 32 | o) of the first member that has a partner
    unsigned first_key[2];            // the same as place << 15 | o (small case)
    int first_in[2][4];               //                    {place, o, w} of that partner
    long long scan_w[LS_NW];
    long long scan_o[LS_NW];
    int scan_c[LS_NW];
    long long fill_mem, fill_S;
};

struct WorkLds {
    int w[LS_CAP];
    int o[LS_CAP];
    int pm[LS_CAP + LS_E];  // LS_CAP is a multiple of the tile: whole-tile stores of a tile that holds place m - 1 < LS_CAP stay inside
    unsigned short rank[LS_TABLE];
};

union PhaseLds {
    RadixLds<LS_T> radix;
    WorkLds work;
};

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_else(int keep, int v)
{
    return __builtin_amdgcn_update_dpp(keep, v, CTRL, ROW_MASK, 0xf, false);
}

// inclusive prefix minimum (MAX: maximum of non-negative values) over the 64 lanes, all active
template <bool MAX>
__device__ __forceinline__ int wave_scan(int v)
{
    constexpr int ID = MAX ? 0 : LS_INF;
    auto op = [](int x, int y) { return MAX ? max(x, y) : min(x, y); };
    v = op(v, dpp_else<0x111, 0xf>(ID, v));  // row_shr:1
    v = op(v, dpp_else<0x112, 0xf>(ID, v));  // row_shr:2
    v = op(v, dpp_else<0x114, 0xf>(ID, v));  // row_shr:4
    v = op(v, dpp_else<0x118, 0xf>(ID, v));  // row_shr:8
    v = op(v, dpp_else<0x142, 0xa>(ID, v));  // row_bcast15 into rows 1 and 3
    v = op(v, dpp_else<0x143, 0xc>(ID, v));  // row_bcast31 into rows 2 and 3
    return v;
}

// the value of the lane below (the identity in lane 0)
template <bool MAX>
__device__ __forceinline__ int wave_prev(int v)
{
    return dpp_else<0x138, 0xf>(MAX ? 0 : LS_INF, v);  // wave_shr:1
}

// first place in [lo, hi) whose w exceeds lim (hi if none); W ascending
template <class IntPtr>
__device__ __forceinline__ int upper_bound_w(IntPtr W, int lo, int hi, int lim)
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
    if (tid == 0) { L.fill_mem = 0; L.fill_S = 0; }
    long long carry_w = 0, carry_o = 0;
    int K = 0;
    for (int tile = 0; tile < m; tile += LS_T) {
        const int i = tile + tid;
        const int ov = i < m ? O[i] : 0;
        long long w = i < m ? (long long)W[i] : 0, q = ov;
        for (int d = 1; d < 64; d <<= 1) {
            const long long uw = __shfl_up(w, d), uq = __shfl_up(q, d);
            if (lane >= d) { w += uw; q += uq; }
        }
        if (lane == 63) { L.scan_w[wave] = w; L.scan_o[wave] = q; }
        __syncthreads();
        long long off_w = carry_w, off_o = carry_o, tot_w = carry_w, tot_o = carry_o;
        for (int v = 0; v < LS_NW; ++v) {
            const long long xw = L.scan_w[v], xo = L.scan_o[v];
            if (v < wave) { off_w += xw; off_o += xo; }
            tot_w += xw;
            tot_o += xo;
        }
        const long long pre = w + off_w;
        const bool fit = i < m && pre <= (long long)M;
        if (fit) {
            O[i] = (int)((unsigned)ov | LS_MEMBER);
            if (i + 1 >= m || pre + (long long)W[i + 1] > (long long)M) {  // the last one that fits
                L.fill_mem = pre;
                L.fill_S = q + off_o;
            }
        }
        const int c = __syncthreads_count(fit);
        K += c;
        carry_w = tot_w;
        carry_o = tot_o;
        if (c < LS_T) break;  // uniform: c is the same in every thread
    }
    __syncthreads();
    mem = L.fill_mem;
    S = L.fill_S;
    return K;
}

// rank[v] = number of the m sorted entries with w <= v, for v = 0..W[m-1] < LS_TABLE:
// boundaries of the runs of equal w are scattered into a zeroed table, then a running maximum
// fills the gaps (each thread owns a contiguous chunk, chunk totals scanned across the block).
__device__ void build_rank(const int *W, int m, unsigned short *rank, SwapLds &L)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int w_last = W[m - 1];
    for (int v = tid; v <= w_last; v += LS_T) rank[v] = 0;
    __syncthreads();
    for (int j = tid; j < m; j += LS_T) {
        const int wj = W[j];
        if (j + 1 == m || W[j + 1] != wj) rank[wj] = (unsigned short)(j + 1);
    }
    __syncthreads();
    const int chunk = (w_last + LS_T) / LS_T;
    const int lo = tid * chunk, hi = min(lo + chunk, w_last + 1);
    int run = 0;
    for (int v = lo; v < hi; ++v) run = max(run, (int)rank[v]);
    const int incl = wave_scan<true>(run);
    if (lane == 63) L.wave_min[wave] = incl;
    int before = wave_prev<true>(incl);
    __syncthreads();
    for (int u = 0; u < LS_NW; ++u)
        if (u < wave) before = max(before, L.wave_min[u]);
    for (int v = lo; v < hi; ++v) {
        before = max(before, (int)rank[v]);
        rank[v] = (unsigned short)before;
    }
    __syncthreads();
}

// One tile of the prefix-minimum scan: ov[e] = entries of places base + tid*LS_E + e (members and
// places past the end count as "none"); pm[e] receives the least o among non-members before each
// place (carry = the same over all earlier tiles, updated) and is stored to PM[base + ...] for
// places <= m.  Two barriers; PM is complete after the second.
template <class IntPtr>
__device__ __forceinline__ void scan_tile(const int (&ov)[LS_E], int (&pm)[LS_E], int &carry, SwapLds &L, IntPtr PM,
                                          int base, int m)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int run = LS_INF;
#pragma unroll
    for (int e = 0; e < LS_E; ++e) {
        pm[e] = run;
        if (ov[e] >= 0) run = min(run, ov[e]);
    }
    const int incl = wave_scan<false>(run);
    if (lane == 63) L.wave_min[wave] = incl;
    int before = wave_prev<false>(incl);
    __syncthreads();
    int total = carry;
    before = min(before, carry);
#pragma unroll
    for (int u = 0; u < LS_NW; ++u) {
        const int x = L.wave_min[u];
        if (u < wave) before = min(before, x);
        total = min(total, x);
    }
#pragma unroll
    for (int e = 0; e < LS_E; ++e) {
        pm[e] = min(pm[e], before);
        const int i = base + (int)threadIdx.x * LS_E + e;
        if (i <= m) PM[i] = pm[e];
    }
    carry = total;
    __syncthreads();
}

// Running state of one batch's exchanges, the same in every thread.
struct SwapState {
    long long mem, S;  // sum of s+o and of o over the members
    int hi;            // every member lies before place hi
    int w_hi;          // no member is larger than this
    int swaps;
};

// The exchanges of one batch, any size.  W, O, PM: m sorted entries (LDS or global memory; PM
// holds m + 1), members flagged in O's sign bit.  rank: table of build_rank or null.
template <class IntPtr, class RankPtr>
__device__ __forceinline__ void swap_loop(IntPtr W, IntPtr O, IntPtr PM, RankPtr rank, int m, int M, SwapState &st,
                                          SwapLds &L)
{
    long long mem = st.mem, S = st.S;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w_last = W[m - 1];
    // number of places whose w is at most lim; needs W[from - 1] <= lim and the answer <= to
    auto ub = [&](int from, int to, int lim) {
        if (rank) return (int)rank[min(lim, w_last)];  // rank[w_last] = m
        return upper_bound_w(W, from, to, lim);
    };
    // this thread's places of the first tile, in registers (LS_INF = a non-member that never helps)
    int own_o[LS_E], own_w[LS_E], own_pm[LS_E];
#pragma unroll
    for (int e = 0; e < LS_E; ++e) {
        const int i = tid * LS_E + e;
        own_o[e] = i < m ? O[i] : LS_INF;
        own_w[e] = i < m ? W[i] : 0;
    }
    if (tid < 2) { L.first_out[tid] = LS_NO_KEY; L.first_in[tid][0] = LS_NONE; }
    __syncthreads();
    int hi = st.hi, swaps = st.swaps, w_hi = st.w_hi;
    for (int it = 0;; ++it) {
        const int slot = it & 1;
        const int slack = (int)((long long)M - mem);
        const int U = ub(hi, m, w_hi + slack);  // places from U on fit against no member

        // ---- pm[j] = least o among non-members before place j, for j = 0..U (entries past U may
        //      be written too; nothing reads them)
        int carry = LS_INF;
        scan_tile(own_o, own_pm, carry, L, PM, 0, m);
        for (int tile = LS_TILE; tile <= U; tile += LS_TILE) {
            int ov[LS_E], pm[LS_E];
#pragma unroll
            for (int e = 0; e < LS_E; ++e) {
                const int i = tile + tid * LS_E + e;
                ov[e] = i < m ? O[i] : LS_INF;
            }
            scan_tile(ov, pm, carry, L, PM, tile, m);
        }

        // ---- first member with an improving partner that fits: per wave the lowest lane of the
        //      first tile that has one; waves combined by a minimum in LDS; the key carries its o
        unsigned long long cand = LS_NO_KEY;
        for (int tile = 0; tile < hi; tile += LS_TILE) {
            unsigned long long mine = LS_NO_KEY;
            int ov[LS_E], wv[LS_E];
#pragma unroll
            for (int e = 0; e < LS_E; ++e) {
                const int a = tile + tid * LS_E + e;
                if (tile == 0) { ov[e] = own_o[e]; wv[e] = own_w[e]; }
                else { ov[e] = a < hi ? O[a] : LS_INF; wv[e] = a < hi ? W[a] : 0; }
            }
            if (rank) {  // loads issued for all places at once; non-members read rank[0] = 0, pm[0] = none
                int j[LS_E], p[LS_E];
#pragma unroll
                for (int e = 0; e < LS_E; ++e) j[e] = rank[ov[e] < 0 ? min(wv[e] + slack, w_last) : 0];
#pragma unroll
                for (int e = 0; e < LS_E; ++e) p[e] = PM[j[e]];
#pragma unroll
                for (int e = LS_E - 1; e >= 0; --e) {
                    const int oo = (int)((unsigned)ov[e] & ~LS_MEMBER);
                    if (ov[e] < 0 && p[e] < oo)
                        mine = ((unsigned long long)(tile + tid * LS_E + e) << 32) | (unsigned)oo;
                }
            } else {
#pragma unroll
                for (int e = LS_E - 1; e >= 0; --e) {
                    const int a = tile + tid * LS_E + e;
                    if (ov[e] < 0) {  // a member
                        const int oo = (int)((unsigned)ov[e] & ~LS_MEMBER);
                        if (PM[upper_bound_w(W, a + 1, U, wv[e] + slack)] < oo)
                            mine = ((unsigned long long)a << 32) | (unsigned)oo;
                    }
                }
            }
            const unsigned long long bal = __builtin_amdgcn_ballot_w64(mine != LS_NO_KEY);
            if (bal != 0 && cand == LS_NO_KEY) {
                const int l = (int)__builtin_ctzll(bal);
                const unsigned lo32 = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)mine, l);
                const unsigned hi32 = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(mine >> 32), l);
                cand = ((unsigned long long)hi32 << 32) | lo32;
            }
        }
        if (lane == 0 && cand != LS_NO_KEY) atomicMin(&L.first_out[slot], cand);
        __syncthreads();
        const unsigned long long key = L.first_out[slot];
        if (key == LS_NO_KEY) break;  // uniform
        const int a_star = (int)(key >> 32), o_a = (int)(unsigned)key;
        const int w_a = W[a_star];

        // ---- its partner: the first non-member with smaller o, i.e. the one place where the
        //      prefix minimum is still >= o_out and the entry itself is below it
        {
            int fb = LS_NONE, fo = 0, fw = 0;
#pragma unroll
            for (int e = 0; e < LS_E; ++e) {
                const bool is = own_o[e] >= 0 && own_o[e] < o_a && own_pm[e] >= o_a;
                fb = is ? tid * LS_E + e : fb;
                fo = is ? own_o[e] : fo;
                fw = is ? own_w[e] : fw;
            }
            if (fb != LS_NONE) {
                L.first_in[slot][0] = fb;
                L.first_in[slot][1] = fo;
                L.first_in[slot][2] = fw;
            }
        }
        for (int tile = LS_TILE; tile < U; tile += LS_TILE) {
#pragma unroll
            for (int e = 0; e < LS_E; ++e) {
                const int b = tile + tid * LS_E + e;
                if (b < U) {
                    const int ov = O[b];
                    if (ov >= 0 && ov < o_a && PM[b] >= o_a) {
                        L.first_in[slot][0] = b;
                        L.first_in[slot][1] = ov;
                        L.first_in[slot][2] = W[b];
                    }
                }
            }
        }
        __syncthreads();
        const int b_star = L.first_in[slot][0], o_b = L.first_in[slot][1], w_b = L.first_in[slot][2];
        if (b_star == LS_NONE) break;  // cannot happen: pm said a partner exists; never spin

        // ---- exchange; every thread keeps the running sums, the owners rewrite the flags
        mem += (long long)w_b - (long long)w_a;
        S += (long long)o_b - (long long)o_a;
        if (b_star >= hi) { hi = b_star + 1; w_hi = w_b; }
        ++swaps;
        const int in_flag = (int)((unsigned)o_b | LS_MEMBER);
        if (((a_star & (LS_TILE - 1)) / LS_E) == tid) O[a_star] = o_a;
        if (((b_star & (LS_TILE - 1)) / LS_E) == tid) O[b_star] = in_flag;
#pragma unroll
        for (int e = 0; e < LS_E; ++e) {
            if (tid * LS_E + e == a_star) own_o[e] = o_a;
            if (tid * LS_E + e == b_star) own_o[e] = in_flag;
        }
        if (tid == 0) {  // the other slot was last read two barriers ago; ready it for the next step
            L.first_out[slot ^ 1] = LS_NO_KEY;
            L.first_in[slot ^ 1][0] = LS_NONE;
        }
    }
    st.mem = mem;
    st.S = S;
    st.hi = hi;
    st.w_hi = w_hi;
    st.swaps = swaps;
}

// The same steps for the common small case, straight-line: working set in LDS, rank table present,
// and every place that matters (U, see above) inside the first tile, so each thread works on the
// LS_E places it keeps in registers and nothing is conditional but the two block-wide decisions.
// Runs until no exchange is left (returns true) or the case no longer applies (returns false with
// st and the flags in O consistent, for swap_loop to continue).
__device__ __forceinline__ bool swap_steps_small(lds_int *W, lds_int *O, lds_int *PM, lds_rank *rank, int m, int M,
                                                 SwapState &st, SwapLds &L)
{
    constexpr unsigned NO_KEY = 0xffffffffu;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int w_last = W[m - 1];
    int own_o[LS_E], own_w[LS_E];
#pragma unroll
    for (int e = 0; e < LS_E; ++e) {
        const int i = tid * LS_E + e;
        own_o[e] = i < m ? O[i] : LS_INF;
        own_w[e] = i < m ? W[i] : 0;
    }
    if (tid < 2) { L.first_key[tid] = NO_KEY; L.first_in[tid][0] = LS_NONE; }
    __syncthreads();
    int slack = (int)((long long)M - st.mem), hi = st.hi, w_hi = st.w_hi, swaps = st.swaps;
    long long S = st.S;
    bool done = false;
    for (int it = 0;; ++it) {
        const int slot = it & 1;
        const int U = rank[min(w_hi + slack, w_last)];
        if (U >= LS_TILE) break;  // uniform

        // ---- prefix minimum of o over the non-members (a member reads as "none": its sign bit
        //      makes it the largest unsigned value)
        int pm[LS_E];
        int run = LS_INF;
#pragma unroll
        for (int e = 0; e < LS_E; ++e) {
            pm[e] = run;
            run = (int)min((unsigned)run, (unsigned)own_o[e]);
        }
        const int incl = wave_scan<false>(run);
        if (lane == 63) L.wave_min[wave] = incl;
        int before = wave_prev<false>(incl);
        __syncthreads();
#pragma unroll
        for (int u = 0; u < LS_NW; ++u) before = u < wave ? min(before, L.wave_min[u]) : before;
#pragma unroll
        for (int e = 0; e < LS_E; ++e) {
            pm[e] = min(pm[e], before);
            PM[tid * LS_E + e] = pm[e];  // the table has room for the whole tile
        }
        __syncthreads();

        // ---- first member with an improving partner that fits; key = place << 15 | o
        unsigned key = NO_KEY;
        {
            int j[LS_E], p[LS_E];
#pragma unroll
            for (int e = 0; e < LS_E; ++e) j[e] = rank[own_o[e] < 0 ? min(own_w[e] + slack, w_last) : 0];
#pragma unroll
            for (int e = 0; e < LS_E; ++e) p[e] = PM[j[e]];
#pragma unroll
            for (int e = LS_E - 1; e >= 0; --e) {
                const int oo = (int)((unsigned)own_o[e] & ~LS_MEMBER);
                key = (own_o[e] < 0 && p[e] < oo) ? (unsigned)(((tid * LS_E + e) << 15) | oo) : key;
            }
        }
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(key != NO_KEY);
        if (bal != 0) {
            const unsigned k = (unsigned)__builtin_amdgcn_readlane((int)key, (int)__builtin_ctzll(bal));
            if (lane == 0) atomicMin(&L.first_key[slot], k);
        }
        __syncthreads();
        const unsigned best = L.first_key[slot];
        if (best == NO_KEY) { done = true; break; }  // uniform
        const int a_star = (int)(best >> 15), o_a = (int)(best & 0x7fffu);
        const int w_a = W[a_star];

        // ---- its partner: the one non-member below o_out whose prefix minimum is not
        {
            int fb = LS_NONE, fo = 0, fw = 0;
#pragma unroll
            for (int e = 0; e < LS_E; ++e) {
                const bool is = (unsigned)own_o[e] < (unsigned)o_a && pm[e] >= o_a;
                fb = is ? tid * LS_E + e : fb;
                fo = is ? own_o[e] : fo;
                fw = is ? own_w[e] : fw;
            }
            if (fb != LS_NONE) {
                L.first_in[slot][0] = fb;
                L.first_in[slot][1] = fo;
                L.first_in[slot][2] = fw;
            }
        }
        __syncthreads();
        const int b_star = L.first_in[slot][0], o_b = L.first_in[slot][1], w_b = L.first_in[slot][2];
        if (b_star == LS_NONE) { done = true; break; }  // cannot happen; never spin

        // ---- exchange
        slack -= w_b - w_a;
        S += (long long)(o_b - o_a);
        if (b_star >= hi) { hi = b_star + 1; w_hi = w_b; }
        ++swaps;
        const int in_flag = (int)((unsigned)o_b | LS_MEMBER);
#pragma unroll
        for (int e = 0; e < LS_E; ++e) {
            own_o[e] = (tid * LS_E + e == a_star) ? o_a : own_o[e];
            own_o[e] = (tid * LS_E + e == b_star) ? in_flag : own_o[e];
        }
        if ((a_star / LS_E) == tid) O[a_star] = o_a;
        if ((b_star / LS_E) == tid) O[b_star] = in_flag;
        if (tid == 0) {  // the other slot was last read two barriers ago; ready it for the next step
            L.first_key[slot ^ 1] = NO_KEY;
            L.first_in[slot ^ 1][0] = LS_NONE;
        }
    }
    st.mem = (long long)M - slack;
    st.S = S;
    st.hi = hi;
    st.w_hi = w_hi;
    st.swaps = swaps;
    return done;
}

__global__ __launch_bounds__(LS_T) void local_swap_kernel(int32_t n, const int32_t *s, const int32_t *o, int32_t M,
                                                          int32_t ga, int32_t gb, int32_t *order_out, int32_t *batch_end_out, double *F_out,
                                                          int32_t *swaps_out, int32_t *num_batches_out, int *gw, int *go,
                                                          int *gid, int *alt_o, int *buf0, int *buf1, int *by_o,
                                                          int *batch_of, int32_t *words)
{
    __shared__ PhaseLds P;
    __shared__ SwapLds L;
    __shared__ int sh[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- well-formedness and key widths
    int omax = 0, wmax = 0, vmax = 0, bad = 0;
    for (int i = tid; i < n; i += LS_T) {
        const int sv = s[i], ov = o[i];
        const bool ok = sv >= 1 && ov >= 1 && (long long)sv + ov <= (long long)M;
        if (!ok) bad = 1;
        omax = max(omax, ov);
        wmax = max(wmax, (sv < 1 || ov < 1) ? 0 : (int)min((long long)sv + ov, (long long)M));
        vmax = max(vmax, ok ? ga * sv + gb * ov : 0);
    }
    if (tid < 4) sh[tid] = 0;
    __syncthreads();
    if (bad) atomicOr(&sh[2], 1);
    atomicMax(&sh[0], omax);
    atomicMax(&sh[1], wmax);
    atomicMax(&sh[3], vmax);
    __syncthreads();
    omax = sh[0];
    wmax = sh[1];
    vmax = sh[3];  // largest value an exchange compares: o, or the effective length of the G metric
    if (sh[2] != 0) {  // a request that can never run: report, emit no batches
        if (tid == 0) {
            atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            *num_batches_out = 0;
        }
        return;
    }

    // ---- key sorts: ids by (o, id), kept for the emission order, then on by s+o
    for (int i = tid; i < n; i += LS_T) buf0[i] = i;
    __syncthreads();
    int *cur = buf0, *alt = buf1;
    auto key_o = [o](int id) { return o[id]; };
    auto key_w = [s, o](int id) { return s[id] + o[id]; };
    for (int shift = 0; shift < bits_of(omax); shift += 8) {
        radix_pass(cur, alt, n, shift, key_o, P.radix);
        int *t = cur; cur = alt; alt = t;
    }
    for (int i = tid; i < n; i += LS_T) by_o[i] = cur[i];
    __syncthreads();
    for (int shift = 0; shift < bits_of(wmax); shift += 8) {
        radix_pass(cur, alt, n, shift, key_w, P.radix);
        int *t = cur; cur = alt; alt = t;
    }
    for (int i = tid; i < n; i += LS_T) {
        const int id = cur[i];
        gid[i] = id;
        go[i] = ga * s[id] + gb * o[id];  // what an exchange must lower: o, or the effective length of the G metric
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
        const int *W = gw + a;
        int *O = go + a;
        if (in_lds) {
            for (int i = tid; i < m; i += LS_T) {
                P.work.w[i] = gw[a + i];
                P.work.o[i] = go[a + i];
            }
            __syncthreads();
            W = P.work.w;
            O = P.work.o;
        }
        long long mem = 0, S = 0;
        int hi = 0, swaps = 0;
        const int K = greedy_fill(W, O, m, M, mem, S, L);
        if (K < 1) {  // cannot happen for well-formed input; never spin
            if (tid == 0) atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            break;
        }
        SwapState st;
        st.mem = mem;
        st.S = S;
        st.hi = K;
        st.w_hi = W[K - 1];
        st.swaps = 0;
        if (in_lds) {  // the same loop, compiled for LDS addresses
            lds_rank *rank = nullptr;
            bool done = false;
            if (W[m - 1] < LS_TABLE) {
                build_rank(W, m, P.work.rank, L);
                rank = (lds_rank *)P.work.rank;
                if (vmax < LS_SMALL_VALUE)  // the straight-line steps pack (place, value) into 32 bits
                    done = swap_steps_small((lds_int *)P.work.w, (lds_int *)P.work.o, (lds_int *)P.work.pm, rank, m, M, st, L);
            }
            if (!done) swap_loop((lds_int *)P.work.w, (lds_int *)P.work.o, (lds_int *)P.work.pm, rank, m, M, st, L);
        } else {
            swap_loop(gw + a, go + a, alt_o, (const unsigned short *)nullptr, m, M, st, L);
        }
        S = st.S;
        hi = st.hi;
        swaps = st.swaps;
        __syncthreads();
        if (tid == 0) {
            batch_end_out[nb] = a + K;
            F_out[nb] = (double)S / ((double)gb * (double)K * (double)K);
            if (swaps_out) swaps_out[nb] = swaps;
        }
        // members get the batch number; non-members of [0, hi) close up behind the K removed
        // places (stable), through the spare arrays
        int carry = 0;
        for (int tile = 0; tile < hi; tile += LS_T) {
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
            for (int u = 0; u < LS_NW; ++u) {
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
        for (int i = K + tid; i < hi; i += LS_T) {
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
    for (int i = tid; i < n; i += LS_T) order_out[i] = src[i];
}

}  // namespace

size_t kvs_local_swap_scratch_bytes(int32_t n)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    return np * 8 * sizeof(int) + 256;
}

int kvs_launch_local_swap(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t ga, int32_t gb,
                          int32_t *order_out,
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
    hipLaunchKernelGGL(local_swap_kernel, dim3(1), dim3(LS_T), 0, st, n, s, o, M, ga, gb, order_out, batch_end_out, F_out,
                       swaps_out, num_batches_out, gw, go, gid, alt_o, buf0, buf1, by_o, batch_of, d_words);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
