// Phase 2 under predicted decode lengths (Section 5, "Handling Prediction Uncertainty via Adaptive
// Output Length Refinement"; appendix algorithm "Sorted-F + A_min"), many candidate orders at once,
// one 64-lane wavefront per candidate.
//
// The scheduler does not know o_i.  It holds a running estimate e_i (started from the caller's
// est0: lower bounds for A_min, upper bounds for the conservative A_max) and runs the admission
// of Algorithm 1's Phase 2 on the memory the running requests are PROJECTED to hold; round t:
//   1. a running request that has produced a = t - p tokens leaves if a = o_i, else needs one
//      more: e_i <- max(e_i, a + 1);
//   2. waiting requests are started in the order's sequence while the projection stays <= M;
//   3. while the projection exceeds M, the running request of least (e_i, i) is stopped; it keeps
//      e_i, loses its progress and waits again at its own place of the order.
//
// State of a candidate, all in LDS (one wavefront per workgroup, 16 n + 4 H bytes):
//   * per position of the order: s, o, current estimate, start round (or waiting / done), id;
//   * the projected memory of the requests that are still inside their estimate, as a ring of
//     H >= max(estimate, o) slots (slot t is cleared at round t and then stands for round t + H);
//   * the requests that have outrun their estimate are not in the ring: each of them reserves
//     exactly the next round, s_j + (t + 1 - p_j), so two scalars (their count and the sum of
//     s_j - p_j) give their share of round t + 1, and a round costs nothing per such request;
//   * the running positions as a compact list; a request matters again only when it reaches its
//     estimate or its true length, so the list is scanned only at the earliest such round.
#include "kvsched_internal.h"

#include <limits.h>

namespace {

constexpr int PW = 64;
constexpr int P_WAITING = -1, P_DONE = -2;
constexpr int EST_OVERRUN = 0;  // estimate field of a request that has outrun it: e = t - p + 1

struct PredParams {
    const int32_t *orders;  // [C][n]
    int32_t C, n;
    const int32_t *s, *o;
    const int32_t *est0;  // [E][n]
    int32_t E;
    int32_t M;
    int32_t H;            // ring slots: power of two >= every estimate and every o
    int32_t round_limit;  // a run that lasts longer is reported, not continued
    int64_t *tel_out;         // [C]
    int32_t *completion_out;  // [C][n] by request id, or NULL
    int32_t *evictions_out;   // [C] or NULL
    int32_t *d_words;
};

__device__ __forceinline__ int p_uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ void p_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int p_wave_min(int v)
{
    for (int d = 32; d >= 1; d >>= 1) v = min(v, __shfl_xor(v, d));
    return p_uni(v);
}

__global__ __launch_bounds__(PW) void predicted_kernel(PredParams p)
{
    extern __shared__ int lds[];
    const int lane = threadIdx.x;
    const int cand = blockIdx.x;
    const int n = p.n, M = p.M, H = p.H, HM = H - 1;
    int *ring = lds;
    const int n2 = (n + 1) & ~1;
    int *S = ring + H;
    int *PS = S + n;  // start round of a running position, P_WAITING, P_DONE
    unsigned short *O = (unsigned short *)(PS + n);  // lengths and estimates are at most 16384
    unsigned short *EST = O + n2;
    unsigned short *ID = EST + n2;
    unsigned short *ACT = ID + n2;  // running positions, unordered

    const int32_t *row = p.orders + (size_t)cand * (size_t)n;
    const int32_t *est0 = p.est0 + (p.E > 1 ? (size_t)cand * (size_t)n : 0);
    int32_t *crow = p.completion_out ? p.completion_out + (size_t)cand * (size_t)n : nullptr;

    for (int i = lane; i < H; i += PW) ring[i] = 0;
    int bad = 0;
    for (int k = lane; k < n; k += PW) {
        const int id = min(max(row[k], 0), n - 1);
        const int sv = p.s[id], ov = p.o[id], ev = est0[id];
        if (sv < 1 || ov < 1 || ev < 1 || ov > H || ev > H || (long long)sv + ov > (long long)M ||
            (long long)sv + ev > (long long)M)
            bad = 1;
        S[k] = sv;
        O[k] = (unsigned short)ov;
        EST[k] = (unsigned short)ev;
        PS[k] = P_WAITING;
        ID[k] = (unsigned short)id;
    }
    if (__builtin_amdgcn_ballot_w64(bad) != 0) {  // cannot be scheduled: report, do not loop forever
        if (lane == 0) {
            p.tel_out[cand] = -1;
            if (p.evictions_out) p.evictions_out[cand] = 0;
            atomicOr(&p.d_words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
        }
        return;
    }
    p_sync();

    int t = 0;
    int head = 0;      // no waiting position lies before it
    int hpos = -1, hs = 0, he = 0, ho = 0;  // the waiting position the admission is stuck at, if any, with its s, e, o
    int nact = 0;      // entries of ACT
    int done = 0;
    int ov_cnt = 0;    // requests past their estimate ...
    long long ov_sp = 0;  // ... and the sum of s_j - p_j over them
    int next_due = INT_MAX;  // earliest round at which a running request reaches its estimate or its end
    int evictions = 0;
    long long tel = 0;
    bool over_limit = false;

    while (done < n) {
        if (t >= p.round_limit) { over_limit = true; break; }
        // nothing waits, nobody outruns an estimate: nothing can happen before the next due round
        if (head >= n && ov_cnt == 0 && next_due > t) {
            const int span = min(next_due - t, H);
            for (int i = lane; i < span; i += PW) ring[(t + i) & HM] = 0;
            t = next_due;
            p_sync();
        }
        if (lane == 0) ring[t & HM] = 0;  // round t is past
        p_sync();

        // ---- 1. running requests that reach their estimate or their end at this round.  A light
        //         pass finds them (usually one or two) and the next due round of the others; each
        //         is then handled by the whole wavefront; finished ones leave the list in a second pass.
        if (t >= next_due) {
            int due_min = INT_MAX;  // per lane: over the entries that stay as they are
            int due_new = INT_MAX;  // uniform: over the entries that started to overrun
            int removed = 0;
            for (int a0 = 0; a0 < nact; a0 += PW) {
                const int a = a0 + lane;
                const bool in = a < nact;
                const int pos = in ? ACT[a] : 0;
                const int ps = in ? PS[pos] : 0, ov = in ? O[pos] : 0, ev = in ? EST[pos] : 0;
                const int due = ps + (ev == EST_OVERRUN ? ov : min(ev, ov));
                const bool now = in && due <= t;
                if (in && !now) due_min = min(due_min, due);
                unsigned long long m = __builtin_amdgcn_ballot_w64(now);
                while (m != 0) {
                    const int l = __builtin_ctzll(m);
                    m &= m - 1;
                    const int pos_l = __builtin_amdgcn_readlane(pos, l), ps_l = __builtin_amdgcn_readlane(ps, l);
                    const int ov_l = __builtin_amdgcn_readlane(ov, l), ev_l = __builtin_amdgcn_readlane(ev, l);
                    const int sv_l = p_uni(S[pos_l]);
                    if (t - ps_l == ov_l) {  // finished
                        if (lane == 0) {
                            PS[pos_l] = P_DONE;
                            if (crow) crow[ID[pos_l]] = t;
                            ACT[a0 + l] = 0xffff;  // leaves the list
                        }
                        ++done;
                        ++removed;
                        tel += t;
                        if (ev_l == EST_OVERRUN) {
                            --ov_cnt;
                            ov_sp -= (long long)sv_l - ps_l;
                        } else {  // over-estimated: rounds t+1 .. p + e were reserved for it
                            for (int tq = t + 1 + lane; tq <= ps_l + ev_l; tq += PW) ring[tq & HM] -= sv_l + (tq - ps_l);
                        }
                    } else {  // goes on past its estimate: from now on it reserves the next round only
                        if (lane == 0) EST[pos_l] = EST_OVERRUN;
                        ++ov_cnt;
                        ov_sp += (long long)sv_l - ps_l;
                        due_new = min(due_new, ps_l + ov_l);
                    }
                }
            }
            next_due = min(p_wave_min(due_min), due_new);
            if (removed > 0) {  // close the list up, in place: a tile is read before it is written
                p_sync();
                int kept = 0;
                for (int a0 = 0; a0 < nact; a0 += PW) {
                    const int a = a0 + lane;
                    const int pos = a < nact ? ACT[a] : 0xffff;
                    const bool keep = pos != 0xffff;
                    const unsigned long long km = __builtin_amdgcn_ballot_w64(keep);
                    p_sync();
                    if (keep) ACT[kept + __popcll(km & ((1ull << lane) - 1ull))] = (unsigned short)pos;
                    kept += __popcll(km);
                    p_sync();
                }
                nact = kept;
            }
            p_sync();
        }

        // ---- 2. admission in the order's sequence
        const int ov_next = (int)(ov_sp + (long long)ov_cnt * (t + 1));  // the overrunners' share of round t + 1
        int t_skip = t + 1;  // the next round at which anything can happen
        while (head < n) {
            if (hpos < 0) {  // first waiting position at or after head; kept while it stays blocked
                for (int k0 = head; k0 < n && hpos < 0; k0 += PW) {
                    const int k = k0 + lane;
                    const unsigned long long w = __builtin_amdgcn_ballot_w64(k < n && PS[k] == P_WAITING);
                    if (w != 0) hpos = k0 + __builtin_ctzll(w);
                }
                if (hpos < 0) { head = n; break; }
                head = hpos;
                hs = p_uni(S[hpos]);
                he = p_uni(EST[hpos]);
                ho = p_uni(O[hpos]);
            }
            if (ov_cnt == 0) {
                // Nobody outruns an estimate, so until the next due round the projection does not
                // change: look for the earliest start from t on.  Round tq rules out the starts
                // t' < tq with t' < ring(tq) + s + tq - M; rounds more than H ahead hold nothing.
                // Each turn moves the start to the largest bound seen and looks only at the rounds
                // that entered the window (t', t' + e] since.
                int start = t, lo = t + 1;
                const int bias = hs - M;
                for (;;) {
                    const int hi = min(start + he, t + H);
                    int acc = INT_MIN;
                    for (int tq = lo + lane; tq <= hi; tq += PW) acc = max(acc, min(tq, ring[tq & HM] + bias + tq));
                    const int bound = -p_wave_min(-max(acc, INT_MIN + 1));
                    if (bound <= start) break;  // fits at `start`
                    start = bound;
                    lo = hi + 1;
                    if (start >= next_due) break;  // the running set changes first
                }
                if (start > t) {  // blocked now; nothing happens before min(start, next_due)
                    t_skip = min(start, next_due);
                    break;
                }
            } else {
                bool viol = false;
                for (int j = lane + 1; j <= he; j += PW) viol |= ring[(t + j) & HM] + (j == 1 ? ov_next : 0) + hs + j > M;
                if (__builtin_amdgcn_ballot_w64(viol) != 0) break;
            }
            for (int j = lane + 1; j <= he; j += PW) ring[(t + j) & HM] += hs + j;
            if (lane == 0) {
                PS[hpos] = t;
                ACT[nact] = (unsigned short)hpos;
            }
            ++nact;
            next_due = min(next_due, t + min(he, ho));
            head = hpos + 1;
            hpos = -1;
            p_sync();
        }

        // ---- 3. eviction while round t + 1 is projected above M (only that round can be: the ring
        //         held a feasible projection and only the overrunners' reservations are new)
        if (ov_cnt > 0) {
            p_sync();
            while (p_uni(ring[(t + 1) & HM]) + (int)(ov_sp + (long long)ov_cnt * (t + 1)) > M) {
                int best = INT_MAX;  // (current estimate, id) of the running requests, least first
                for (int a0 = 0; a0 < nact; a0 += PW) {
                    const int a = a0 + lane;
                    if (a < nact) {
                        const int pos = ACT[a];
                        const int ev = EST[pos];
                        const int cur = ev == EST_OVERRUN ? t - PS[pos] + 1 : ev;
                        best = min(best, (cur << 16) | (int)ID[pos]);
                    }
                }
                best = p_wave_min(best);
                if (best == INT_MAX) break;  // cannot happen: an empty system holds nothing
                // find it in the list again (ids of a permutation are distinct)
                int slot = -1, vpos = -1;
                for (int a0 = 0; a0 < nact && slot < 0; a0 += PW) {
                    const int a = a0 + lane;
                    bool hit = false;
                    int pos = 0;
                    if (a < nact) {
                        pos = ACT[a];
                        const int ev = EST[pos];
                        const int cur = ev == EST_OVERRUN ? t - PS[pos] + 1 : ev;
                        hit = ((cur << 16) | (int)ID[pos]) == best;
                    }
                    const unsigned long long m = __builtin_amdgcn_ballot_w64(hit);
                    if (m != 0) {
                        const int l = __builtin_ctzll(m);
                        slot = a0 + l;
                        vpos = __builtin_amdgcn_readlane(pos, l);
                    }
                }
                if (slot < 0) break;
                const int ps = p_uni(PS[vpos]), ev = p_uni(EST[vpos]), sv = p_uni(S[vpos]);
                if (ev == EST_OVERRUN) {
                    --ov_cnt;
                    ov_sp -= (long long)sv - ps;
                } else {
                    for (int tq = t + 1 + lane; tq <= ps + ev; tq += PW) ring[tq & HM] -= sv + (tq - ps);
                }
                p_sync();
                if (lane == 0) {
                    if (ev == EST_OVERRUN) EST[vpos] = (unsigned short)(t - ps + 1);  // what it is known to need
                    PS[vpos] = P_WAITING;
                    ACT[slot] = ACT[nact - 1];
                }
                --nact;
                if (vpos < head) { head = vpos; hpos = -1; }
                ++evictions;
                p_sync();
            }
        }
        // While requests outrun their estimates the projection of round t' + 1 grows by their count
        // every round; until the next due round nothing else changes.  Round t' needs work only if
        // that projection passes M (eviction) or leaves room for the first token of the blocked
        // request (a necessary condition for its admission): find the first such round.
        if (ov_cnt > 0 && (hpos >= 0 || head >= n) && next_due > t + 1) {
            const int room = hpos >= 0 ? hs + 1 : INT_MAX / 2;  // nothing waits: only the overflow matters
            int found = next_due;
            for (int base = t + 1; base < next_due && found == next_due; base += PW) {
                const int tr = base + lane;
                bool hit = false;
                if (tr < next_due) {
                    const long long x = (long long)ring[(tr + 1) & HM] + ov_sp + (long long)ov_cnt * (tr + 1);
                    hit = x > (long long)M || x + room <= (long long)M;
                }
                const unsigned long long m = __builtin_amdgcn_ballot_w64(hit);
                if (m != 0) found = base + __builtin_ctzll(m);
            }
            t_skip = found;
        }
        // rounds t + 1 .. t_skip - 1 change nothing
        if (t_skip > t + 1) {
            const int span = min(t_skip - t - 1, H);
            for (int i = lane; i < span; i += PW) ring[(t + 1 + i) & HM] = 0;
            t = t_skip;
            p_sync();
        } else {
            ++t;
        }
    }

    if (lane == 0) {
        if (over_limit) {
            p.tel_out[cand] = -1;
            atomicOr(&p.d_words[KVS_W_STATUS], KVSCHED_DEV_ROUND_LIMIT);
        } else {
            p.tel_out[cand] = tel;
        }
        if (p.evictions_out) p.evictions_out[cand] = evictions;
    }
}

__global__ __launch_bounds__(1024) void scan_estimates_kernel(const int32_t *est, size_t count, int32_t *words)
{
    __shared__ int sh[16];
    int mx = 0;
    for (size_t i = threadIdx.x; i < count; i += 1024) mx = max(mx, est[i]);
    for (int d = 32; d >= 1; d >>= 1) mx = max(mx, __shfl_xor(mx, d));
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w) mx = max(mx, sh[w]);
        words[KVS_W_ESTMAX] = mx;
    }
}

}  // namespace

int kvs_launch_scan_estimates(const int32_t *est, size_t count, int32_t *d_words, hipStream_t st)
{
    hipLaunchKernelGGL(scan_estimates_kernel, dim3(1), dim3(1024), 0, st, est, count, d_words);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}

size_t kvs_predicted_lds_bytes(int32_t n, int32_t H)
{
    return sizeof(int) * ((size_t)H + 2 * (size_t)n) + sizeof(unsigned short) * (4 * (((size_t)n + 1) & ~(size_t)1));
}

int kvs_launch_predicted(const int32_t *orders, int32_t C, int32_t n, const int32_t *s, const int32_t *o,
                         const int32_t *est0, int32_t E, int32_t M, int32_t H, int32_t round_limit, int64_t *tel_out,
                         int32_t *completion_out, int32_t *evictions_out, int32_t *d_words, hipStream_t st)
{
    const size_t bytes = kvs_predicted_lds_bytes(n, H);
    if (bytes > KVS_PREDICTED_MAX_LDS || n > 65535) return KVSCHED_ERANGE;
    // beyond 64 KB of dynamic LDS the kernel's limit has to be raised first; only as far as needed
    static size_t lds_limit = 64 * 1024;
    if (bytes > lds_limit) {
        if (hipFuncSetAttribute((const void *)predicted_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)bytes) != hipSuccess)
            return KVSCHED_EHIP;
        lds_limit = bytes;
    }
    PredParams p;
    p.orders = orders;
    p.C = C;
    p.n = n;
    p.s = s;
    p.o = o;
    p.est0 = est0;
    p.E = E;
    p.M = M;
    p.H = H;
    p.round_limit = round_limit;
    p.tel_out = tel_out;
    p.completion_out = completion_out;
    p.evictions_out = evictions_out;
    p.d_words = d_words;
    hipLaunchKernelGGL(predicted_kernel, dim3((unsigned)C), dim3(PW), bytes, st, p);
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
