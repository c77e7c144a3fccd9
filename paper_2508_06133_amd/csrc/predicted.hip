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
// State of a candidate in LDS (one wavefront per workgroup):
//   * the projected memory of the requests that are still inside their estimate, as a ring of
//     H >= max(estimate, o) slots (slot t is cleared at round t and then stands for round t + H);
//   * the requests that have outrun their estimate are not in the ring: each of them reserves
//     exactly the next round, s_j + (t + 1 - p_j), so two scalars (their count and the sum of
//     s_j - p_j) give their share of round t + 1, and a round costs nothing per such request;
//   * per position of the order only what changes and must outlive a stop: one bit "waits" (every
//     position from `frontier` on waits and none of them was ever started, so the bits are looked
//     at only after a request was stopped).  The estimate a stopped request keeps is needed twice
//     per stop (written when it is stopped, read when it is looked at again), so it lives in
//     global memory, 16 bits per position and candidate, written and read by the same wavefront;
//     a position that was never started takes its estimate from est0;
//   * the RUNNING requests as a compact unordered list of complete entries: three words
//     {s, position | id, o | estimate} side by side (a stride of three words is free of bank
//     conflicts) and, in an array of its own, the low 16 bits of the round at which the entry next
//     matters: it reaches its estimate or its true length, start + min(estimate, o), or start + o
//     once it has outrun its estimate.  The start round follows from that (a running request
//     started at most o <= 16384 rounds ago, so 16 bits and the current round give the round
//     itself).  The pass that finds the due entries and the next due round reads that array alone;
//     an entry that finishes leaves a hole that the list's last entry fills.
// Lengths and ids of the waiting positions are not kept at all: admission walks the order from the
// front, so the 64 positions around the first waiting one sit in registers (one position per lane,
// fetched from the order row and the length tables when the walk leaves the window).
// The list is what decides how many candidates fit a compute unit, and a wavefront here spends
// most of its time waiting on its own dependent instructions, so twice the wavefronts per SIMD
// is nearly twice the rate: a first launch runs every candidate with a list of at most `cap`
// entries, sized so that eight candidates share a compute unit (two wavefronts per SIMD: 20 KB each); a
// candidate whose list overflows gives up and is run again by a second launch whose list holds
// all n positions (three to four candidates per compute unit).
// A blocked request is not re-examined round by round: the search over the ring gives the earliest
// start its reservations allow, and that bound holds until memory is released (an eviction, or a
// request that finishes before its estimate), whoever outruns an estimate meanwhile.
#include "kvsched_internal.h"

#include <limits.h>

namespace {

constexpr int PW = 64;
constexpr int EST_OVERRUN = 0;  // estimate field of a request that has outrun it: e = t - p + 1
constexpr int MAX_HOLES = 64;  // finished entries of one pass whose places are filled from the list's end

struct PredParams {
    const int32_t *orders;  // [C][n]
    int32_t C, n;
    const int32_t *s, *o;
    const int32_t *est0;  // [E][n]
    int32_t E;
    int32_t M;
    int32_t H;            // ring slots: power of two >= every estimate and every o
    int32_t cap;          // entries of the running list (even)
    int32_t second;       // 0: every candidate, overflow sets retry[c]; 1: only candidates with retry[c] != 0
    int32_t *retry;       // [C]
    unsigned short *est_stopped;  // [C][n]: estimate kept by a stopped request, by position
    int32_t round_limit;  // a run that lasts longer is reported, not continued
    int64_t *tel_out;         // [C]
    int32_t *completion_out;  // [C][n] by request id, or NULL
    int32_t *evictions_out;   // [C] or NULL
    int32_t *d_words;
};

__device__ __forceinline__ int p_uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ long long p_uni64(long long v)
{
    const int lo = __builtin_amdgcn_readfirstlane((int)v), hi = __builtin_amdgcn_readfirstlane((int)(v >> 32));
    return (long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);
}

__device__ __forceinline__ void p_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Minimum over the 64 lanes by lane exchanges inside the vector unit (four steps within the rows of
// 16 lanes, two row broadcasts; lane 63 ends up with the result).
__device__ __forceinline__ int p_wave_min(int v)
{
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false));  // row_half_mirror
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xf, 0xf, false));  // row_mirror
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x142, 0xa, 0xf, false));  // row_bcast:15 into rows 1 and 3
    v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x143, 0xc, 0xf, false));  // row_bcast:31 into rows 2 and 3
    return __builtin_amdgcn_readlane(v, 63);
}

__global__ __launch_bounds__(PW) void predicted_kernel(PredParams p)
{
    extern __shared__ int lds[];
    const int lane = threadIdx.x;
    const int cand = blockIdx.x;
    if (p.second && p.retry[cand] == 0) return;
    const int n = p.n, M = p.M, H = p.H, HM = H - 1, cap = p.cap;
    const int stw = (n + 31) >> 5;
    int *ring = lds;
    unsigned *WAIT = (unsigned *)(ring + H);           // bit k & 31 of word k >> 5: position k waits (below the frontier)
    int *LE = (int *)(WAIT + stw);                     // the running list, three words an entry: s, position | id << 16, o | estimate << 16
    unsigned short *LDUE = (unsigned short *)(LE + 3 * cap);  // round an entry next matters at, low 16 bits
    unsigned short *est_stopped = p.est_stopped + (size_t)cand * (size_t)n;

    const int32_t *row = p.orders + (size_t)cand * (size_t)n;
    const int32_t *est0 = p.est0 + (p.E > 1 ? (size_t)cand * (size_t)n : 0);
    int32_t *crow = p.completion_out ? p.completion_out + (size_t)cand * (size_t)n : nullptr;

    for (int i = lane; i < H; i += PW) ring[i] = 0;
    for (int i = lane; i < stw; i += PW) WAIT[i] = 0;  // nobody was stopped yet
    int bad = 0;
    for (int k = lane; k < n; k += PW) {
        const int id = min(max(row[k], 0), n - 1);
        const int sv = p.s[id], ov = p.o[id], ev = est0[id];
        if (sv < 1 || ov < 1 || ev < 1 || ov > H || ev > H || (long long)sv + ov > (long long)M ||
            (long long)sv + ev > (long long)M)
            bad = 1;
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

    // the 64 positions [w_base, w_base + 64) of the order: lane l holds id, s, o of position w_base + l
    int w_base = -PW, w_id = 0, w_s = 1, w_o = 1, w_e = 1;
    int x_base = -PW, x_id = 0, x_s = 1, x_o = 1, x_e = 1;  // ... and the 64 behind them, fetched ahead of need
    int frontier = 0;  // every position from here on waits and was never started
    int c_pos = -1, c_s = 0, c_o = 0, c_id = 0, c_e = 0;  // the request stopped last: position, lengths, id, estimate kept

    int t = 0;
    int head = 0;      // no waiting position lies before it
    int hpos = -1, hs = 0, he = 0, ho = 0, hid = 0;  // the waiting position the admission is stuck at, if any
    int ring_start = 0;  // ... and a round before which the ring's reservations rule out its start
    int nact = 0;      // entries of the list
    int done = 0;
    int ov_cnt = 0;    // requests past their estimate ...
    long long ov_sp = 0;  // ... and the sum of s_j - p_j over them
    int next_due = INT_MAX;  // earliest round at which a running request reaches its estimate or its end
    int evictions = 0;
    long long tel = 0;
    bool over_limit = false, overflow = false;

    while (done < n) {
        // Everything the loop carries is the same in all lanes; saying so keeps it in scalar registers and the
        // control flow on the scalar unit (left to itself the compiler treats much of it as per-lane data:
        // copies of a dozen vector registers and an EXEC mask at every branch).
        t = p_uni(t), head = p_uni(head), hpos = p_uni(hpos), hs = p_uni(hs), he = p_uni(he), ho = p_uni(ho), hid = p_uni(hid);
        ring_start = p_uni(ring_start), nact = p_uni(nact), done = p_uni(done), ov_cnt = p_uni(ov_cnt), ov_sp = p_uni64(ov_sp);
        next_due = p_uni(next_due), evictions = p_uni(evictions), tel = p_uni64(tel), frontier = p_uni(frontier);
        c_pos = p_uni(c_pos), c_s = p_uni(c_s), c_o = p_uni(c_o), c_id = p_uni(c_id), c_e = p_uni(c_e);
        w_base = p_uni(w_base), x_base = p_uni(x_base);
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

        // ---- 1. running requests that reach their estimate or their end at this round.  One pass over
        //         the due rounds finds them (usually one or two) and the next due round of the others;
        //         each is then handled by the whole wavefront; a finished one leaves a hole in the list.
        if (t >= next_due) {
            int wait_min = INT_MAX;  // per lane: rounds until the entries that stay as they are matter again
            int due_new = INT_MAX;   // uniform: next due round of the entries handled here
            int holes = 0, hole_at = 0;  // lane i of hole_at: list place of the i-th finished entry
            for (int a0 = 0; a0 < nact; a0 += PW) {
                const int a = a0 + lane;
                const bool in = a < nact;
                const int wait = in ? (int)(short)(unsigned short)(LDUE[a] - t) : 1;  // due - t (at most 16384 ahead)
                const bool now = in && wait <= 0;
                if (in && !now) wait_min = min(wait_min, wait);
                unsigned long long m = __builtin_amdgcn_ballot_w64(now);
                while (m != 0) {
                    const int e = p_uni(a0 + __builtin_ctzll(m));  // the entry
                    m &= m - 1;
                    const int s_r = LE[3 * e], pi_r = LE[3 * e + 1], oe_r = LE[3 * e + 2];  // three reads in flight
                    const int oe_l = p_uni(oe_r), sv_l = p_uni(s_r);
                    const int ov_l = oe_l & 0xffff, ev_l = (int)((unsigned)oe_l >> 16);
                    // due now: it started min(estimate, o) rounds ago, o rounds ago if it had outrun its estimate
                    const int ps_l = t - (ev_l == EST_OVERRUN ? ov_l : min(ev_l, ov_l));
                    if (t - ps_l == ov_l) {  // finished
                        if (crow && lane == 0) crow[(unsigned)pi_r >> 16] = t;
                        ++done;
                        tel += t;
                        if (holes < MAX_HOLES) hole_at = lane == holes ? e : hole_at;
                        ++holes;
                        if (ev_l == EST_OVERRUN) {
                            --ov_cnt;
                            ov_sp -= (long long)sv_l - ps_l;
                        } else {  // over-estimated: rounds t+1 .. p + e were reserved for it
                            for (int tq = t + 1 + lane; tq <= ps_l + ev_l; tq += PW) ring[tq & HM] -= sv_l + (tq - ps_l);
                            ring_start = 0;  // memory released: the blocked request may fit earlier
                        }
                    } else {  // goes on past its estimate: from now on it reserves the next round only
                        if (lane == 0) {
                            LE[3 * e + 2] = ov_l;  // (estimate field EST_OVERRUN)
                            LDUE[e] = (unsigned short)(ps_l + ov_l);
                        }
                        ++ov_cnt;
                        ov_sp += (long long)sv_l - ps_l;
                        due_new = min(due_new, ps_l + ov_l);
                    }
                }
            }
            const int w = p_wave_min(wait_min);
            next_due = min(w == INT_MAX ? INT_MAX : t + w, due_new);
            if (holes > 0) {
                p_sync();
                if (holes <= MAX_HOLES) {
                    // fill each hole with the list's last entry, the hole furthest back first: the last
                    // entry is then never a hole that is still to be filled
                    // (lane 0 alone moves the entries: its reads and writes stay in order; the four reads
                    // of a move go out together)
                    for (int h = holes - 1; h >= 0; --h) {
                        const int at = __builtin_amdgcn_readlane(hole_at, h);
                        --nact;
                        if (at != nact && lane == 0) {
                            const int e0 = LE[3 * nact], e1 = LE[3 * nact + 1], e2 = LE[3 * nact + 2];
                            const unsigned short due = LDUE[nact];
                            LE[3 * at] = e0, LE[3 * at + 1] = e1, LE[3 * at + 2] = e2;
                            LDUE[at] = due;
                        }
                    }
                    p_sync();
                } else {  // (more than a tile of requests finishing in one round) close the list up: the due ones that have finished go
                    int kept = 0;
                    for (int a0 = 0; a0 < nact; a0 += PW) {
                        const int a = a0 + lane;
                        const bool in = a < nact;
                        const int e0 = in ? LE[3 * a] : 0, e1 = in ? LE[3 * a + 1] : 0, e2 = in ? LE[3 * a + 2] : 0;
                        const int due = in ? LDUE[a] : 0;
                        // finished: due now, and what it was due for is its true length (the entries that
                        // went on past their estimate at this round were given a later due round above)
                        const int ev = (int)((unsigned)e2 >> 16);
                        const bool fin = in && (unsigned short)due == (unsigned short)t &&
                                         (ev == EST_OVERRUN || ev >= (e2 & 0xffff));
                        const bool keep = in && !fin;
                        const unsigned long long km = __builtin_amdgcn_ballot_w64(keep);
                        p_sync();
                        if (keep) {
                            const int to = kept + __popcll(km & ((1ull << lane) - 1ull));
                            LE[3 * to] = e0, LE[3 * to + 1] = e1, LE[3 * to + 2] = e2;
                            LDUE[to] = (unsigned short)due;
                        }
                        kept += __popcll(km);
                        p_sync();
                    }
                    nact = kept;
                }
            }
            p_sync();
        }

        // ---- 2. admission in the order's sequence
        const int ov_next = (int)(ov_sp + (long long)ov_cnt * (t + 1));  // the overrunners' share of round t + 1
        int t_skip = t + 1;  // the next round at which anything can happen
        while (head < n) {
            head = p_uni(head), hpos = p_uni(hpos), frontier = p_uni(frontier), nact = p_uni(nact), next_due = p_uni(next_due);
            ring_start = p_uni(ring_start), t_skip = p_uni(t_skip);
            if (hpos < 0) {  // first waiting position at or after head; kept while it stays blocked
                if (head < frontier) {  // among the stopped ones: 32 positions a lane, 2048 a turn
                    for (int w0 = head >> 5; w0 < stw && hpos < 0; w0 += PW) {
                        const int wi = w0 + lane;
                        unsigned wait = wi < stw ? WAIT[wi] : 0u;
                        if (wi == (head >> 5)) wait &= ~0u << (head & 31);  // not before head
                        const unsigned long long any = __builtin_amdgcn_ballot_w64(wait != 0);
                        if (any != 0) {
                            const int l = __builtin_ctzll(any);
                            hpos = (w0 + l) * 32 + __builtin_ctz((unsigned)__builtin_amdgcn_readlane((int)wait, l));
                        }
                    }
                    if (hpos < 0) hpos = frontier;  // none: the first position never started
                } else {
                    hpos = head;
                }
                hpos = p_uni(hpos);
                if (hpos >= n) { hpos = -1; head = n; break; }
                head = hpos;
                if (hpos == c_pos) {
                    // the request stopped last: what admission needs of it was at hand when it was stopped
                    hs = c_s, ho = c_o, hid = c_id, he = c_e;
                } else if (hpos < frontier) {
                    // an older stopped one: fetched alone (two dependent loads), the window stays at the frontier
                    hid = p_uni(min(max(row[hpos], 0), n - 1));
                    hs = p_uni(p.s[hid]);
                    ho = p_uni(p.o[hid]);
                    he = p_uni((int)est_stopped[hpos]);  // a stopped request kept its estimate
                } else {
                    if (hpos < w_base || hpos >= w_base + PW) {  // the 64 positions around it
                        const int base = hpos & ~(PW - 1);
                        if (base == x_base) {  // fetched ahead
                            w_id = x_id, w_s = x_s, w_o = x_o, w_e = x_e;
                        } else {
                            const int k = base + lane;
                            w_id = 0, w_s = 1, w_o = 1, w_e = 1;
                            if (k < n) {
                                w_id = min(max(row[k], 0), n - 1);
                                w_s = p.s[w_id];
                                w_o = p.o[w_id];
                                w_e = est0[w_id];
                            }
                        }
                        w_base = base;
                        x_base = base + PW;  // the loads for the next 64 are issued now and waited for when used
                        const int k = x_base + lane;
                        x_id = 0, x_s = 1, x_o = 1, x_e = 1;
                        if (k < n) {
                            x_id = min(max(row[k], 0), n - 1);
                            x_s = p.s[x_id];
                            x_o = p.o[x_id];
                            x_e = est0[x_id];
                        }
                    }
                    hs = __builtin_amdgcn_readlane(w_s, hpos - w_base);
                    ho = __builtin_amdgcn_readlane(w_o, hpos - w_base);
                    hid = __builtin_amdgcn_readlane(w_id, hpos - w_base);
                    he = __builtin_amdgcn_readlane(w_e, hpos - w_base);  // one that never ran starts from est0
                }
                ring_start = 0;
            }
            if (t < ring_start) {  // the ring rules this round out (nothing was released since that was found)
                if (ov_cnt == 0) t_skip = min(ring_start, next_due);
                break;
            }
            // The requests past their estimate hold round t + 1 as well; that test is one slot of the ring, so it
            // goes first (when it fails no request starts this round, whatever the ring's reservations say).
            if (ov_cnt > 0 && p_uni(ring[(t + 1) & HM]) + ov_next + hs + 1 > M) break;
            if (nact == cap) { overflow = true; break; }  // (first launch only: the second one's list holds every position)
            // A start at t against the reservations in the ring, the request's own entered in the same pass and
            // taken back if some round cannot hold them (rare: the ring's verdict is known for a blocked request).
            // Two tiles of 64 rounds a turn, their reads in flight together; a slot behind the window is read
            // and left alone.  Every lane touches only its own slots until the wavefront meets again.
            bool viol = false;
            for (int j = lane + 1; j <= he; j += 2 * PW) {
                const int i0 = (t + j) & HM, i1 = (t + j + PW) & HM;
                const int r0 = ring[i0] + hs + j, r1 = ring[i1] + hs + j + PW;
                const bool in1 = j + PW <= he;
                viol |= r0 > M;
                viol |= in1 && r1 > M;
                ring[i0] = r0;
                if (in1) ring[i1] = r1;
            }
            if (__builtin_amdgcn_ballot_w64(viol) != 0) {
                for (int j = lane + 1; j <= he; j += PW) ring[(t + j) & HM] -= hs + j;
                p_sync();
                // Blocked by them.  They change only by admissions (none while this request is blocked)
                // and releases, so they are searched once for the earliest start they allow: round tq
                // rules out the starts t' < tq with t' < ring(tq) + s + tq - M; rounds more than H ahead
                // hold nothing.  Each turn moves the start to the largest bound seen and looks only at the
                // rounds that entered the window (t', t' + e] since.
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
                ring_start = start;  // (> t)
                if (ov_cnt == 0) t_skip = min(start, next_due);  // nothing happens before
                break;
            }
            ring_start = t;  // the ring allows a start now
            if (lane == 0) {
                if (hpos < frontier) WAIT[hpos >> 5] &= ~(1u << (hpos & 31));  // a stopped one starts again
                LE[3 * nact] = hs, LE[3 * nact + 1] = hpos | (hid << 16), LE[3 * nact + 2] = ho | (he << 16);
                LDUE[nact] = (unsigned short)(t + min(he, ho));
            }
            if (hpos >= frontier) frontier = hpos + 1;
            ++nact;
            next_due = min(next_due, t + min(he, ho));
            head = hpos + 1;
            hpos = -1;
            p_sync();
        }
        if (overflow) break;

        // ---- 3. eviction while round t + 1 is projected above M (only that round can be: the ring
        //         held a feasible projection and only the overrunners' reservations are new)
        if (ov_cnt > 0) {
            p_sync();
            while (p_uni(ring[(t + 1) & HM]) + (int)(ov_sp + (long long)ov_cnt * (t + 1)) > M) {
                int best = INT_MAX, best_at = -1;  // (current estimate, id) of the running requests, least first, and its place
                for (int a0 = 0; a0 < nact; a0 += PW) {
                    const int a = a0 + lane;
                    if (a < nact) {
                        const int oe = LE[3 * a + 2];
                        const int ev = (int)((unsigned)oe >> 16);
                        // past its estimate: it has run o - (due - t) rounds and needs one more
                        const int cur = ev == EST_OVERRUN ? (oe & 0xffff) - (int)(unsigned short)(LDUE[a] - (unsigned short)t) + 1 : ev;
                        const int key = (cur << 16) | (int)((unsigned)LE[3 * a + 1] >> 16);
                        if (key < best) best = key, best_at = a;
                    }
                }
                const int least = p_wave_min(best);
                if (least == INT_MAX) break;  // cannot happen: an empty system holds nothing
                // ids of a permutation are distinct: one lane holds it
                const unsigned long long holder = __builtin_amdgcn_ballot_w64(best == least);
                const int slot = __builtin_amdgcn_readlane(best_at, __builtin_ctzll(holder));
                if (slot < 0) break;
                const int s_r = LE[3 * slot], pi_r = LE[3 * slot + 1], oe_r = LE[3 * slot + 2], due16 = LDUE[slot];
                const int vpos = p_uni(pi_r) & 0xffff;
                const int ev = (int)((unsigned)p_uni(oe_r) >> 16), sv = p_uni(s_r), ov = p_uni(oe_r) & 0xffff;
                const int due = t + (int)(unsigned short)((unsigned short)p_uni(due16) - (unsigned short)t);
                const int ps = due - (ev == EST_OVERRUN ? ov : min(ev, ov));
                if (ev == EST_OVERRUN) {
                    --ov_cnt;
                    ov_sp -= (long long)sv - ps;
                } else {
                    for (int tq = t + 1 + lane; tq <= ps + ev; tq += PW) ring[tq & HM] -= sv + (tq - ps);
                    ring_start = 0;  // memory released
                }
                p_sync();
                c_pos = vpos, c_s = sv, c_o = ov, c_id = (int)((unsigned)p_uni(pi_r) >> 16);
                c_e = ev == EST_OVERRUN ? t - ps + 1 : ev;  // what it is known to need
                if (lane == 0) {
                    est_stopped[vpos] = (unsigned short)c_e;
                    WAIT[vpos >> 5] |= 1u << (vpos & 31);  // waits again
                    const int last = nact - 1;
                    const int e0 = LE[3 * last], e1 = LE[3 * last + 1], e2 = LE[3 * last + 2];
                    const unsigned short due_last = LDUE[last];
                    LE[3 * slot] = e0, LE[3 * slot + 1] = e1, LE[3 * slot + 2] = e2;
                    LDUE[slot] = due_last;
                }
                --nact;
                if (vpos < head) { head = vpos; hpos = -1; }
                ++evictions;
                p_sync();
            }
        }
        // While requests outrun their estimates the projection of round t' + 1 grows by their count
        // every round; until the next due round nothing else changes.  Round t' needs work only if
        // that projection passes M (eviction) or, from the round on that the ring allows the blocked
        // request to start at, leaves room for its first token (both necessary for its admission):
        // find the first such round.
        if (ov_cnt > 0 && (hpos >= 0 || head >= n) && next_due > t + 1) {
            const int room = hpos >= 0 ? hs + 1 : INT_MAX / 2;  // nothing waits: only the overflow matters
            const int from = hpos >= 0 ? ring_start : INT_MAX;
            int found = next_due;
            for (int base = t + 1; base < next_due && found == next_due; base += PW) {
                const int tr = base + lane;
                bool hit = false;
                if (tr < next_due) {
                    const long long x = (long long)ring[(tr + 1) & HM] + ov_sp + (long long)ov_cnt * (tr + 1);
                    hit = x > (long long)M || (tr >= from && x + room <= (long long)M);
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
        if (overflow) {
            p.retry[cand] = 1;  // the second launch runs this candidate with a list of n entries
        } else {
            if (over_limit) {
                p.tel_out[cand] = -1;
                atomicOr(&p.d_words[KVS_W_STATUS], KVSCHED_DEV_ROUND_LIMIT);
            } else {
                p.tel_out[cand] = tel;
            }
            if (p.evictions_out) p.evictions_out[cand] = evictions;
        }
    }
}

__global__ void clear_retry_kernel(int32_t *retry, int32_t C)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < C) retry[i] = 0;
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

// LDS of one candidate whose running list has `cap` entries.
static size_t predicted_lds_bytes(int32_t n, int32_t H, int32_t cap)
{
    const size_t stw = ((size_t)n + 31) >> 5;
    return sizeof(int) * ((size_t)H + stw + 3 * (size_t)cap) + sizeof(unsigned short) * (size_t)cap;
}

// ... with a list that holds every position: what a candidate may need at worst.
size_t kvs_predicted_lds_bytes(int32_t n, int32_t H) { return predicted_lds_bytes(n, H, (n + 1) & ~1); }

int kvs_launch_predicted(const int32_t *orders, int32_t C, int32_t n, const int32_t *s, const int32_t *o,
                         const int32_t *est0, int32_t E, int32_t M, int32_t H, int32_t round_limit, int64_t *tel_out,
                         int32_t *completion_out, int32_t *evictions_out, int32_t *retry, uint16_t *est_stopped,
                         int32_t *d_words, hipStream_t st)
{
    const int32_t cap_all = (n + 1) & ~1;
    const size_t bytes_all = predicted_lds_bytes(n, H, cap_all);
    if (bytes_all > KVS_PREDICTED_MAX_LDS || n > 65535) return KVSCHED_ERANGE;
    // beyond 64 KB of dynamic LDS the kernel's limit has to be raised first; only as far as needed
    static size_t lds_limit = 64 * 1024;
    if (bytes_all > lds_limit) {
        if (hipFuncSetAttribute((const void *)predicted_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)bytes_all) != hipSuccess)
            return KVSCHED_EHIP;
        lds_limit = bytes_all;
    }
    // First launch: the longest list with which eight candidates share a compute unit's 160 KB (LDS is
    // handed out in whole KB); worth it when that is at least 128 entries and fewer than all.
    const size_t budget = 20 * 1024;
    const size_t fixed = predicted_lds_bytes(n, H, 0);
    int32_t cap_first = fixed < budget ? (int32_t)((budget - fixed) / 14) & ~1 : 0;
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
    p.retry = retry;
    p.est_stopped = est_stopped;
    p.round_limit = round_limit;
    p.tel_out = tel_out;
    p.completion_out = completion_out;
    p.evictions_out = evictions_out;
    p.d_words = d_words;
    if (cap_first >= 128 && cap_first < cap_all && retry) {
        hipLaunchKernelGGL(clear_retry_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, st, retry, C);
        p.cap = cap_first;
        p.second = 0;
        hipLaunchKernelGGL(predicted_kernel, dim3((unsigned)C), dim3(PW), predicted_lds_bytes(n, H, cap_first), st, p);
        p.cap = cap_all;
        p.second = 1;
        hipLaunchKernelGGL(predicted_kernel, dim3((unsigned)C), dim3(PW), bytes_all, st, p);
    } else {
        p.cap = cap_all;
        p.second = 0;
        hipLaunchKernelGGL(predicted_kernel, dim3((unsigned)C), dim3(PW), bytes_all, st, p);
    }
    return hipGetLastError() == hipSuccess ? KVSCHED_OK : KVSCHED_EHIP;
}
