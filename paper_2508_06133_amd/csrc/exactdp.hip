// Phase 1 of Algorithm 1 ("Batch Construction") with every batch the exact minimiser of
// (F, -|X|), found by Algorithm 2 ("Exact Optimal Request Selection via Dynamic Programming"):
//   dp[k][m] = least sum of o over sets of k requests whose load is exactly m,
// requests taken one by one, k running downward, a state replaced only by a strictly smaller
// value; at the end every state is scored F = dp[k][m] / k^2.
//
// On the GPU one request is one launch over all (k, m) states at once, reading the table of the
// previous request and writing a second one (which is what "k downward" achieves in place): one
// wavefront covers 64 consecutive loads m of one cardinality k, and its ballot of "this state was
// improved by request t" is the only record kept of the chosen sets (bits[t][k][m / 64]).  The set
// of the best state is recovered by walking those records backwards: at state (k, m) the last
// request that improved it is a member, and the walk continues at (k - 1, m - load) among the
// earlier requests.  That is the set Algorithm 2 carries in path[k][m].
//
// feas_mode 0: load = sum (s+o) <= M, requests in input order (Algorithm 2 as printed).
// feas_mode 1: the constraint of Algorithm 1's Phase 1 (all of X started together stays within M
//   at every completion time): requests in order of decreasing o, load = sum s, and request j may
//   join k - 1 others only if load + o_j k <= M (j then has the least o, so this is the memory at
//   its completion; the constraints at later completions are not touched by j).
#include "phase1_util.h"

namespace {

constexpr int DP_T = 1024;  // threads of the single-workgroup helper kernels
constexpr int DP_NW = DP_T / 64;
constexpr int DP_INF = 0x7fffffff;
constexpr int DP_STEP_T = 256;
constexpr int DP_ARGMIN_BLOCKS = 256;

struct HelperLds {
    RadixLds<DP_T> radix;
    long long scan[DP_NW];
    int scan_c[DP_NW];
    int sh[4];
    long long red_S[DP_NW];
    int red_k[DP_NW];
    int red_m[DP_NW];
};

__device__ __forceinline__ int cost_of(int sv, int ov, int feas_mode)
{
    return feas_mode ? sv + 1 : sv + ov;  // every feasible set of k requests has sum of cost <= M
}

// Length of the longest prefix of list[0..r) (ascending cost) whose costs sum to at most M: no
// feasible set is larger.  All threads return the same value.
__device__ int prefix_fit(const int *list, int r, const int *s, const int *o, int feas_mode, int M, HelperLds &L)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    long long carry = 0;
    int K = 0;
    for (int tile = 0; tile < r; tile += DP_T) {
        const int i = tile + tid;
        long long w = 0;
        if (i < r) {
            const int id = list[i];
            w = cost_of(s[id], o[id], feas_mode);
        }
        for (int d = 1; d < 64; d <<= 1) {
            const long long u = __shfl_up(w, d);
            if (lane >= d) w += u;
        }
        if (lane == 63) L.scan[wave] = w;
        __syncthreads();
        long long off = carry, total = carry;
        for (int v = 0; v < DP_NW; ++v) {
            const long long x = L.scan[v];
            if (v < wave) off += x;
            total += x;
        }
        const int c = __syncthreads_count(i < r && w + off <= (long long)M);
        K += c;
        carry = total;
        if (c < DP_T) break;  // uniform
    }
    __syncthreads();
    return K;
}

// Validation, the three orders of the ids (emission order (o, id); processing order; ascending
// cost), the first bound on the batch size.
// Returns that bound, or -1 for malformed lengths (reported; no batches).
__device__ int prepare_body(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t feas_mode, int *proc,
                            int *by_o, int *by_cost, int *buf0, int *buf1, int *batch_of, int32_t *words,
                            int32_t *num_batches_out, HelperLds &L)
{
    const int tid = threadIdx.x;
    int omax = 0, cmax = 0, bad = 0;
    for (int i = tid; i < n; i += DP_T) {
        const int sv = s[i], ov = o[i];
        if (sv < 1 || ov < 1 || (long long)sv + ov > (long long)M) bad = 1;
        else {
            omax = max(omax, ov);
            cmax = max(cmax, cost_of(sv, ov, feas_mode));
        }
        batch_of[i] = -1;
    }
    if (tid < 4) L.sh[tid] = 0;
    __syncthreads();
    if (bad) atomicOr(&L.sh[2], 1);
    atomicMax(&L.sh[0], omax);
    atomicMax(&L.sh[1], cmax);
    __syncthreads();
    omax = L.sh[0];
    cmax = L.sh[1];
    if (L.sh[2] != 0) {  // a request that can never run: report, emit no batches
        if (tid == 0) {
            atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            words[KVS_W_REMAIN] = 0;
            words[KVS_W_KMAX] = 0;
            *num_batches_out = 0;
        }
        return -1;
    }
    auto sort_by = [&](int *out, auto key, int kmax_key) {
        for (int i = tid; i < n; i += DP_T) buf0[i] = i;
        __syncthreads();
        int *cur = buf0, *alt = buf1;
        for (int shift = 0; shift < bits_of(kmax_key); shift += 8) {
            radix_pass(cur, alt, n, shift, key, L.radix);
            int *t = cur; cur = alt; alt = t;
        }
        for (int i = tid; i < n; i += DP_T) out[i] = cur[i];
        __syncthreads();
    };
    sort_by(by_o, [o](int id) { return o[id]; }, omax);
    if (feas_mode) sort_by(proc, [o, omax](int id) { return omax - o[id]; }, omax);
    else {
        for (int i = tid; i < n; i += DP_T) proc[i] = i;
        __syncthreads();
    }
    sort_by(by_cost, [s, o, feas_mode](int id) { return cost_of(s[id], o[id], feas_mode); }, cmax);
    __threadfence_block();
    __syncthreads();
    return prefix_fit(by_cost, n, s, o, feas_mode, M, L);
}

__global__ __launch_bounds__(DP_T) void dp_prepare_kernel(int32_t n, const int32_t *s, const int32_t *o, int32_t M,
                                                          int32_t feas_mode, int *proc, int *by_o, int *by_cost,
                                                          int *buf0, int *buf1, int *batch_of, int32_t *words,
                                                          int32_t *num_batches_out)
{
    __shared__ HelperLds L;
    const int kmax = prepare_body(n, s, o, M, feas_mode, proc, by_o, by_cost, buf0, buf1, batch_of, words,
                                  num_batches_out, L);
    if (kmax >= 0 && threadIdx.x == 0) {
        words[KVS_W_REMAIN] = n;
        words[KVS_W_KMAX] = kmax;
    }
}

__global__ __launch_bounds__(DP_STEP_T) void dp_init_kernel(int *a, int *b, size_t count)
{
    const size_t i = (size_t)blockIdx.x * DP_STEP_T + threadIdx.x;
    if (i < count) {
        const int v = i == 0 ? 0 : DP_INF;  // dp[0][0] = 0
        a[i] = v;
        b[i] = v;
    }
}

// Request proc[t] offered to every state: row k = blockIdx.y + 1, loads blockIdx.x * 256 ...
__global__ __launch_bounds__(DP_STEP_T) void dp_step_kernel(const int *proc, int t, const int32_t *s, const int32_t *o,
                                                            int32_t M, int32_t ga, int32_t gb, int32_t feas_mode,
                                                            const int *src, int *dst, unsigned long long *bits_t, int Mp)
{
    const int k = blockIdx.y + 1;
    const int m = blockIdx.x * DP_STEP_T + threadIdx.x;  // < Mp by the launch shape
    const int id = proc[t];
    const int oi = o[id];
    const int load = feas_mode ? s[id] : s[id] + oi;
    const int gi = ga * s[id] + gb * oi;  // what dp sums: o, or the effective length of the G metric
    const size_t at = (size_t)k * Mp + m;
    const int old = src[at];
    int cand = DP_INF;
    if (m <= M && m >= load) {
        const int prev = src[at - Mp - load];
        const bool fits = feas_mode == 0 || (long long)m + (long long)oi * k <= (long long)M;
        if (prev != DP_INF && fits) cand = prev + gi;
    }
    const bool take = cand < old;
    dst[at] = take ? cand : old;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(take);
    if ((threadIdx.x & 63) == 0) bits_t[(size_t)k * (Mp >> 6) + (m >> 6)] = bal;
}

// sign of Sa/ka^2 - Sb/kb^2 (S < 2^31, k <= 4096: the products stay below 2^55)
__device__ __forceinline__ int dp_cmp_F(long long Sa, int ka, long long Sb, int kb)
{
    const long long l = Sa * (long long)kb * (long long)kb, r = Sb * (long long)ka * (long long)ka;
    return l < r ? -1 : (l > r ? 1 : 0);
}

// Is state a a better final choice than state b?  Least F; among equal F the larger k
// (KVSCHED_TIE_LARGER) or the smaller; then the smaller load (the first met scanning m upward).
__device__ __forceinline__ bool dp_better(long long Sa, int ka, int ma, long long Sb, int kb, int mb, int tie_rule)
{
    if (ka == 0) return false;
    if (kb == 0) return true;
    const int c = dp_cmp_F(Sa, ka, Sb, kb);
    if (c != 0) return c < 0;
    if (ka != kb) return tie_rule == KVSCHED_TIE_LARGER ? ka > kb : ka < kb;
    return ma < mb;
}

// Block-wide best of per-thread candidates; every thread receives it.
__device__ void reduce_best(int32_t tie_rule, HelperLds &L, long long &bS, int &bk, int &bm)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int d = 32; d > 0; d >>= 1) {
        const long long oS = __shfl_down(bS, d);
        const int ok = __shfl_down(bk, d), om = __shfl_down(bm, d);
        if (dp_better(oS, ok, om, bS, bk, bm, tie_rule)) { bS = oS; bk = ok; bm = om; }
    }
    __syncthreads();  // the reduction slots may still be read from an earlier call
    if (lane == 0) { L.red_S[wave] = bS; L.red_k[wave] = bk; L.red_m[wave] = bm; }
    __syncthreads();
    if (tid == 0) {
        for (int v = 1; v < DP_NW; ++v)
            if (dp_better(L.red_S[v], L.red_k[v], L.red_m[v], bS, bk, bm, tie_rule)) {
                bS = L.red_S[v]; bk = L.red_k[v]; bm = L.red_m[v];
            }
        L.red_S[0] = bS;
        L.red_k[0] = bk;
        L.red_m[0] = bm;
    }
    __syncthreads();
    bS = L.red_S[0];
    bk = L.red_k[0];
    bm = L.red_m[0];
}

// Best final state among rows k_first, k_first + k_step, ... <= kmax of a table (global or LDS);
// every thread receives it (bk = 0: none).
template <class TablePtr>
__device__ void argmin_body(TablePtr dp, int k_first, int k_step, int kmax, int32_t M, int Mp, int32_t tie_rule,
                            HelperLds &L, long long &bS, int &bk, int &bm)
{
    const int tid = threadIdx.x;
    bS = 0;
    bk = 0;
    bm = 0;
    for (int k = k_first; k <= kmax; k += k_step) {
        for (int m = tid; m <= M; m += DP_T) {
            const int v = dp[(size_t)k * Mp + m];
            if (v != DP_INF && dp_better(v, k, m, bS, bk, bm, tie_rule)) { bS = v; bk = k; bm = m; }
        }
    }
    reduce_best(tie_rule, L, bS, bk, bm);
}

// Thread 0: the outputs of batch nb (or the report that no state exists, which cannot happen for
// well-formed input: a single request always fits).
__device__ void publish_batch(long long bS, int bk, int32_t gb, int32_t done, int32_t nb, int32_t *batch_end_out,
                              double *F_out, int32_t *words)
{
    if (bk >= 1) {
        batch_end_out[nb] = done + bk;
        F_out[nb] = (double)bS / ((double)gb * (double)bk * (double)bk);
    } else {
        atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
    }
}

// Stage 1: workgroup b reduces rows 1 + b, 1 + b + G, ...; stage 2: one workgroup reduces the G partials.
__global__ __launch_bounds__(DP_T) void dp_argmin_rows_kernel(const int *dp, int kmax, int32_t M, int Mp,
                                                              int32_t tie_rule, long long *partial)
{
    __shared__ HelperLds L;
    long long bS;
    int bk, bm;
    argmin_body(dp, 1 + (int)blockIdx.x, (int)gridDim.x, kmax, M, Mp, tie_rule, L, bS, bk, bm);
    if (threadIdx.x == 0) {
        partial[3 * blockIdx.x + 0] = bS;
        partial[3 * blockIdx.x + 1] = bk;
        partial[3 * blockIdx.x + 2] = bm;
    }
}

__global__ __launch_bounds__(DP_T) void dp_argmin_kernel(const long long *partial, int G, int32_t tie_rule, int32_t gb,
                                                         int32_t done, int32_t nb, int32_t *batch_end_out,
                                                         double *F_out, int32_t *words)
{
    __shared__ HelperLds L;
    long long bS = 0;
    int bk = 0, bm = 0;
    for (int g = threadIdx.x; g < G; g += DP_T) {
        const long long S = partial[3 * g];
        const int k = (int)partial[3 * g + 1], m = (int)partial[3 * g + 2];
        if (dp_better(S, k, m, bS, bk, bm, tie_rule)) { bS = S; bk = k; bm = m; }
    }
    reduce_best(tie_rule, L, bS, bk, bm);
    if (threadIdx.x == 0) {
        words[KVS_W_BESTK] = bk;
        words[KVS_W_BESTM] = bm;
        publish_batch(bS, bk, gb, done, nb, batch_end_out, F_out, words);
    }
}

// One wavefront follows the records back from the best state and stamps the members with the
// batch number.  A set of k needs k requests, so only records of requests t >= k - 1 exist (rows
// above t + 1 are not launched and hold nothing of this batch).  Every pass lowers `bound`, so the
// loop ends.
__device__ void walk_body(const unsigned long long *bits, const int *proc, int r, int kmax, int Mp, const int32_t *s,
                          const int32_t *o, int32_t feas_mode, int32_t nb, int *batch_of, int k, int m)
{
    const int lane = threadIdx.x & 63;
    const size_t per_t = (size_t)(kmax + 1) * (Mp >> 6);
    int bound = r - 1;
    while (k > 0 && bound >= 0 && m >= 0) {
        const int t = bound - lane;
        bool hit = false;
        if (t >= k - 1) hit = (bits[(size_t)t * per_t + (size_t)k * (Mp >> 6) + (m >> 6)] >> (m & 63)) & 1ull;
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(hit);
        if (bal == 0) {
            bound -= 64;
            continue;
        }
        const int tstar = bound - (int)__builtin_ctzll(bal);  // the latest such request
        const int id = proc[tstar];
        if (lane == 0) batch_of[id] = nb;
        m -= feas_mode ? s[id] : s[id] + o[id];
        k -= 1;
        bound = tstar - 1;
    }
}

__global__ __launch_bounds__(64) void dp_walk_kernel(const unsigned long long *bits, const int *proc, int r, int kmax,
                                                     int Mp, const int32_t *s, const int32_t *o, int32_t feas_mode,
                                                     int32_t nb, int *batch_of, const int32_t *words)
{
    walk_body(bits, proc, r, kmax, Mp, s, o, feas_mode, nb, batch_of, words[KVS_W_BESTK], words[KVS_W_BESTM]);
}

// Members leave proc[] and by_cost[] (both keep their order); kept = the new count, kmax = the new
// bound on the batch size.
__device__ void compact_body(int *proc, int *by_cost, int *tmp, int r, int32_t nb, const int *batch_of, const int32_t *s,
                             const int32_t *o, int32_t feas_mode, int32_t M, HelperLds &L, int &kept, int &kmax)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    kept = 0;
    for (int pass = 0; pass < 2; ++pass) {
        int *list = pass == 0 ? proc : by_cost;
        int carry = 0;
        for (int tile = 0; tile < r; tile += DP_T) {
            const int i = tile + tid;
            int id = 0, keep = 0;
            if (i < r) {
                id = list[i];
                keep = batch_of[id] != nb;
            }
            int c = keep;
            for (int d = 1; d < 64; d <<= 1) {
                const int u = __shfl_up(c, d);
                if (lane >= d) c += u;
            }
            if (lane == 63) L.scan_c[wave] = c;
            __syncthreads();
            int off = carry, total = carry;
            for (int u = 0; u < DP_NW; ++u) {
                const int x = L.scan_c[u];
                if (u < wave) off += x;
                total += x;
            }
            if (keep) tmp[off + c - 1] = id;
            carry = total;
            __syncthreads();
        }
        kept = carry;
        __threadfence_block();
        __syncthreads();
        for (int i = tid; i < kept; i += DP_T) list[i] = tmp[i];
        __threadfence_block();
        __syncthreads();
    }
    kmax = kept > 0 ? prefix_fit(by_cost, kept, s, o, feas_mode, M, L) : 0;
}

__global__ __launch_bounds__(DP_T) void dp_compact_kernel(int *proc, int *by_cost, int *tmp, int r, int32_t nb,
                                                          const int *batch_of, const int32_t *s, const int32_t *o,
                                                          int32_t feas_mode, int32_t M, int32_t *words)
{
    __shared__ HelperLds L;
    int kept, kmax;
    compact_body(proc, by_cost, tmp, r, nb, batch_of, s, o, feas_mode, M, L, kept, kmax);
    if (threadIdx.x == 0) {  // the words the host reads
        words[KVS_W_REMAIN] = kept;
        words[KVS_W_KMAX] = kmax;
    }
}

// The (o, id)-sorted ids ordered by batch number (stable): each batch in nondecreasing o.
__device__ void emit_body(int32_t n, const int *by_o, int *buf0, int *buf1, const int *batch_of, int32_t nb,
                          int32_t *order_out, int32_t *num_batches_out, HelperLds &L)
{
    const int tid = threadIdx.x;
    const int *src = by_o;
    int *dst = buf0, *other = buf1;
    auto key_b = [batch_of](int id) { return batch_of[id]; };
    bool first = true;
    for (int shift = 0; shift < bits_of(nb - 1); shift += 8) {
        radix_pass(src, dst, n, shift, key_b, L.radix);
        if (first) { src = dst; dst = other; first = false; }
        else { int *t = (int *)src; src = dst; dst = t; }
    }
    for (int i = tid; i < n; i += DP_T) order_out[i] = src[i];
    if (tid == 0) *num_batches_out = nb;
}

__global__ __launch_bounds__(DP_T) void dp_emit_kernel(int32_t n, const int *by_o, int *buf0, int *buf1,
                                                       const int *batch_of, int32_t nb, int32_t *order_out,
                                                       int32_t *num_batches_out)
{
    __shared__ HelperLds L;
    emit_body(n, by_o, buf0, buf1, batch_of, nb, order_out, num_batches_out, L);
}

// The whole Phase 1 in one workgroup when both tables fit in LDS (the settings Algorithm 2 is meant
// for: about a hundred requests, M of a few hundred to a few thousand): no launch per request and
// no host round trip per batch.  Row length Mp = 2^lg >= M + 1; the records still go to global
// memory.  Same arithmetic and the same order of updates as the kernels above.
constexpr int DP_SMALL_STATES = 12288;  // (kmax + 1) * Mp at most; two int tables = 96 KB of LDS
constexpr int DP_SMALL_N = 1024;

__global__ __launch_bounds__(DP_T) void dp_small_kernel(int32_t n, const int32_t *s, const int32_t *o, int32_t M,
                                                        int32_t ga, int32_t gb, int32_t feas_mode, int32_t tie_rule, int lg, int *proc, int *by_o,
                                                        int *by_cost, int *buf0, int *buf1, int *batch_of,
                                                        unsigned long long *bits, int32_t *order_out,
                                                        int32_t *batch_end_out, double *F_out, int32_t *num_batches_out,
                                                        int32_t *words)
{
    __shared__ HelperLds L;
    __shared__ int tab[2][DP_SMALL_STATES];
    __shared__ int req_o[DP_SMALL_N], req_load[DP_SMALL_N], req_g[DP_SMALL_N];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Mp = 1 << lg;
    int kmax = prepare_body(n, s, o, M, feas_mode, proc, by_o, by_cost, buf0, buf1, batch_of, words, num_batches_out, L);
    if (kmax < 0) return;
    int r = n, nb = 0;
    while (r > 0) {
        if (((kmax + 1) << lg) > DP_SMALL_STATES) {  // excluded by the host's choice of this kernel
            if (tid == 0) atomicOr(&words[KVS_W_STATUS], KVSCHED_DEV_BAD_LENGTH);
            break;
        }
        const int states = (kmax + 1) << lg;
        for (int i = tid; i < states; i += DP_T) {
            const int v = i == 0 ? 0 : DP_INF;
            tab[0][i] = v;
            tab[1][i] = v;
        }
        for (int t = tid; t < r; t += DP_T) {
            const int id = proc[t];
            req_o[t] = o[id];
            req_load[t] = feas_mode ? s[id] : s[id] + o[id];
            req_g[t] = ga * s[id] + gb * o[id];
        }
        __syncthreads();
        const size_t per_t = (size_t)(kmax + 1) << (lg - 6);
        for (int t = 0; t < r; ++t) {
            const int oi = req_o[t], load = req_load[t], gi = req_g[t];
            const int rows = t + 1 < kmax ? t + 1 : kmax;
            const int cnt = rows << lg;
            const int *src = tab[t & 1];
            int *dst = tab[(t + 1) & 1];
            for (int base = 0; base < cnt; base += DP_T) {
                const int idx = base + tid;
                if (idx < cnt) {  // whole wavefronts: cnt is a multiple of 64
                    const int k = (idx >> lg) + 1, m = idx & (Mp - 1), at = idx + Mp;
                    const int old = src[at];
                    int cand = DP_INF;
                    if (m <= M && m >= load) {
                        const int prev = src[at - Mp - load];
                        const bool fits = feas_mode == 0 || (long long)m + (long long)oi * k <= (long long)M;
                        if (prev != DP_INF && fits) cand = prev + gi;
                    }
                    const bool take = cand < old;
                    dst[at] = take ? cand : old;
                    const unsigned long long bal = __builtin_amdgcn_ballot_w64(take);
                    if (lane == 0) bits[(size_t)t * per_t + ((size_t)k << (lg - 6)) + (m >> 6)] = bal;
                }
            }
            __syncthreads();
        }
        long long bS;
        int bk, bm;
        argmin_body(tab[r & 1], 1, 1, kmax, M, Mp, tie_rule, L, bS, bk, bm);
        if (tid == 0) publish_batch(bS, bk, gb, n - r, nb, batch_end_out, F_out, words);
        if (bk < 1) break;  // uniform
        __threadfence_block();
        __syncthreads();
        if (wave == 0) walk_body(bits, proc, r, kmax, Mp, s, o, feas_mode, nb, batch_of, bk, bm);
        __threadfence_block();
        __syncthreads();
        int kept, knext;
        compact_body(proc, by_cost, buf0, r, nb, batch_of, s, o, feas_mode, M, L, kept, knext);
        if (kept >= r) break;  // cannot happen: a batch has at least one member; never spin
        r = kept;
        kmax = knext;
        ++nb;
    }
    __syncthreads();
    emit_body(n, by_o, buf0, buf1, batch_of, nb, order_out, num_batches_out, L);
}

bool launched() { return hipGetLastError() == hipSuccess; }

}  // namespace

size_t kvs_exact_dp_list_bytes(int32_t n)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    return np * 6 * sizeof(int) + 256;
}

size_t kvs_exact_dp_table_bytes(int32_t r, int32_t kmax, int32_t M)
{
    const size_t Mp = ((size_t)M + DP_STEP_T) & ~(size_t)(DP_STEP_T - 1);
    return 2 * (size_t)(kmax + 1) * Mp * sizeof(int) + (size_t)r * (size_t)(kmax + 1) * (Mp / 8) +
           3 * sizeof(long long) * DP_ARGMIN_BLOCKS + 256;
}

int kvs_launch_exact_dp_prepare(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t feas_mode,
                                void *lists, int32_t *d_words, int32_t *num_batches_out, hipStream_t st)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    int *proc = (int *)lists, *by_o = proc + np, *by_cost = by_o + np, *buf0 = by_cost + np, *buf1 = buf0 + np,
        *batch_of = buf1 + np;
    hipLaunchKernelGGL(dp_prepare_kernel, dim3(1), dim3(DP_T), 0, st, n, s, o, M, feas_mode, proc, by_o, by_cost, buf0,
                       buf1, batch_of, d_words, num_batches_out);
    return launched() ? KVSCHED_OK : KVSCHED_EHIP;
}

// One batch over the r remaining requests: tables, records, best state, members, compaction.
int kvs_launch_exact_dp_batch(int32_t n, int32_t r, int32_t kmax, const int32_t *s, const int32_t *o, int32_t M,
                              int32_t ga, int32_t gb, int32_t feas_mode, int32_t tie_rule, int32_t nb, void *lists, void *tables,
                              int32_t *batch_end_out, double *F_out, int32_t *d_words, hipStream_t st)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    int *proc = (int *)lists, *by_cost = proc + 2 * np, *buf0 = by_cost + np, *batch_of = buf0 + 2 * np;
    const int Mp = (int)(((size_t)M + DP_STEP_T) & ~(size_t)(DP_STEP_T - 1));
    const size_t table = (size_t)(kmax + 1) * Mp;
    int *dp[2] = {(int *)tables, (int *)tables + table};
    unsigned long long *bits = (unsigned long long *)((int *)tables + 2 * table);
    const size_t per_t = (size_t)(kmax + 1) * (Mp >> 6);
    hipLaunchKernelGGL(dp_init_kernel, dim3((unsigned)((table + DP_STEP_T - 1) / DP_STEP_T)), dim3(DP_STEP_T), 0, st,
                       dp[0], dp[1], table);
    if (!launched()) return KVSCHED_EHIP;
    for (int32_t t = 0; t < r; ++t) {
        const int rows = t + 1 < kmax ? t + 1 : kmax;  // after t + 1 requests no set is larger
        hipLaunchKernelGGL(dp_step_kernel, dim3((unsigned)(Mp / DP_STEP_T), (unsigned)rows), dim3(DP_STEP_T), 0, st,
                           proc, t, s, o, M, ga, gb, feas_mode, dp[t & 1], dp[(t + 1) & 1], bits + (size_t)t * per_t, Mp);
        if (!launched()) return KVSCHED_EHIP;
    }
    const int G = kmax < DP_ARGMIN_BLOCKS ? kmax : DP_ARGMIN_BLOCKS;
    long long *partial = (long long *)(bits + (size_t)r * per_t);
    hipLaunchKernelGGL(dp_argmin_rows_kernel, dim3((unsigned)G), dim3(DP_T), 0, st, dp[r & 1], kmax, M, Mp, tie_rule,
                       partial);
    if (!launched()) return KVSCHED_EHIP;
    hipLaunchKernelGGL(dp_argmin_kernel, dim3(1), dim3(DP_T), 0, st, partial, G, tie_rule, gb, n - r, nb, batch_end_out,
                       F_out, d_words);
    if (!launched()) return KVSCHED_EHIP;
    hipLaunchKernelGGL(dp_walk_kernel, dim3(1), dim3(64), 0, st, bits, proc, r, kmax, Mp, s, o, feas_mode, nb, batch_of,
                       d_words);
    if (!launched()) return KVSCHED_EHIP;
    hipLaunchKernelGGL(dp_compact_kernel, dim3(1), dim3(DP_T), 0, st, proc, by_cost, buf0, r, nb, batch_of, s, o,
                       feas_mode, M, d_words);
    return launched() ? KVSCHED_OK : KVSCHED_EHIP;
}

// Can the one-workgroup kernel take this problem?  kmax_bound: any bound on the batch size.
// Returns log2 of its row length, or 0.
int kvs_exact_dp_small_lg(int32_t n, int32_t kmax_bound, int32_t M)
{
    if (n > DP_SMALL_N) return 0;
    int lg = 6;
    while (((int64_t)1 << lg) < (int64_t)M + 1) ++lg;
    if (lg > 13) return 0;
    return (((int64_t)kmax_bound + 1) << lg) <= DP_SMALL_STATES ? lg : 0;
}

size_t kvs_exact_dp_small_record_bytes(int32_t n, int32_t kmax_bound, int lg)
{
    return (size_t)n * ((size_t)(kmax_bound + 1) << (lg - 6)) * sizeof(unsigned long long) + 256;
}

int kvs_launch_exact_dp_small(int32_t n, const int32_t *s, const int32_t *o, int32_t M, int32_t ga, int32_t gb,
                              int32_t feas_mode, int32_t tie_rule, int lg, void *lists, void *records, int32_t *order_out,
                              int32_t *batch_end_out, double *F_out, int32_t *num_batches_out, int32_t *d_words,
                              hipStream_t st)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    int *proc = (int *)lists, *by_o = proc + np, *by_cost = by_o + np, *buf0 = by_cost + np, *buf1 = buf0 + np,
        *batch_of = buf1 + np;
    hipLaunchKernelGGL(dp_small_kernel, dim3(1), dim3(DP_T), 0, st, n, s, o, M, ga, gb, feas_mode, tie_rule, lg, proc, by_o,
                       by_cost, buf0, buf1, batch_of, (unsigned long long *)records, order_out, batch_end_out, F_out,
                       num_batches_out, d_words);
    return launched() ? KVSCHED_OK : KVSCHED_EHIP;
}

int kvs_launch_exact_dp_emit(int32_t n, int32_t nb, void *lists, int32_t *order_out, int32_t *num_batches_out,
                             hipStream_t st)
{
    const size_t np = ((size_t)n + 64) & ~(size_t)63;
    int *proc = (int *)lists, *by_o = proc + np, *buf0 = proc + 3 * np, *buf1 = buf0 + np, *batch_of = buf1 + np;
    hipLaunchKernelGGL(dp_emit_kernel, dim3(1), dim3(DP_T), 0, st, n, by_o, buf0, buf1, batch_of, nb, order_out,
                       num_batches_out);
    return launched() ? KVSCHED_OK : KVSCHED_EHIP;
}
