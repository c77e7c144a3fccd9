/*
 * CPU oracle for the schedule-evaluation path.  TEST INFRASTRUCTURE ONLY: slow, single
 * threaded, written from the paper; the GPU library shares no code with it and must
 * never call it.
 *
 * Model (Section 2, "Batch Processing and Memory Constraint"; Optimal-IP of Section 6):
 * rounds are 0,1,2,...; a request started at round p occupies s + j tokens of KV memory at
 * round p + j for j = 1..o and completes at round c = p + o; at every round the occupied
 * memory of all running requests must not exceed M.  The paper's pseudo-code (Algorithm 1)
 * counts rounds from 1 and keeps a request for o + 1 rounds, which contradicts both the
 * integer program and the worked Example 1 (TEL 64 / 45); the integer program's convention
 * is the one used here.
 *
 * Functions
 *   oracle_check_instance     Theorem 1's preconditions: s,o >= 1, s + o <= M.
 *   oracle_simulate_literal   Algorithm 1, Phase 2, with the feasibility predicate of Eq. (1)
 *                             re-evaluated from the set of running requests for every
 *                             future round.  This is the reference semantics.
 *   oracle_simulate_profile   The same procedure with the running set's future memory kept
 *                             in an array instead of being re-summed (must equal the literal
 *                             one; the tests check that).  Used where the literal form is
 *                             too slow, and timed as the CPU baseline.
 *   oracle_sortedF            Algorithm 1, Phase 1, with the batch chosen among the feasible
 *                             prefixes of the requests sorted by (s+o, o, id); F of Section 4.
 *   oracle_local_swap         Algorithm 1, Phase 1, with every batch chosen by Local Swap Search
 *                             (the appendix algorithm of that name): greedy fill in ascending
 *                             s+o, then first-improving single exchanges.  Two forms: the literal
 *                             double scan, and one that leaves the inner scan at the first
 *                             request that no longer fits (the list is sorted by s+o, so none
 *                             after it fits either); the tests check that they agree.
 *   oracle_exact_phase1       Algorithm 1, Phase 1, with every batch the exact minimiser of
 *                             (F, -|X|): Algorithm 2's dynamic programme over (k, m) states with
 *                             the chosen set carried along, feasibility either the sum of peaks
 *                             (as Algorithm 2 prints it) or the simultaneous-start profile of
 *                             Algorithm 1's Phase 1 (a derived programme over (k, sum s) states).
 *   oracle_sortedG / oracle_local_swap_G / oracle_exact_phase1_G
 *                             the same three Phase-1 procedures with the generalised metric of
 *                             Section 7 ("Robustness to prefill weighting"),
 *                             G(X) = sum (alpha s_i + o_i) / |X|^2 with alpha = a / b given as two
 *                             integers: the effective length g_i = a s_i + b o_i (b times the paper's)
 *                             takes the place of o_i in the selection metric only; feasibility, the
 *                             sort keys and the emission order inside a batch keep the true lengths.
 *                             alpha = 0 is the F-metric.
 *   oracle_apply_move / oracle_best_neighbor
 *                             position-level swap / insert neighbours of an order, scored by
 *                             total end-to-end latency (Section 2, "Objective").
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)
#define ORACLE_ENOMEM (-2)

/* ------------------------------------------------------------------ instance checks */

int oracle_check_instance(int32_t n, const int32_t *s, const int32_t *o, int64_t M)
{
    if (n < 0 || M < 1) return ORACLE_EINVAL;
    for (int32_t i = 0; i < n; ++i) {
        if (s[i] < 1 || o[i] < 1) return ORACLE_EINVAL;
        if ((int64_t)s[i] + (int64_t)o[i] > M) return ORACLE_EINVAL;
    }
    return ORACLE_OK;
}

static int is_permutation(int32_t n, const int32_t *order)
{
    unsigned char *seen = (unsigned char *)calloc((size_t)n + 1, 1);
    if (!seen) return 0;
    int ok = 1;
    for (int32_t k = 0; k < n && ok; ++k) {
        int32_t r = order[k];
        if (r < 0 || r >= n || seen[r]) ok = 0;
        else seen[r] = 1;
    }
    free(seen);
    return ok;
}

/* --------------------------------------------------- Phase 2, literal (Eq. 1 re-summed) */

/* Memory held at round tq by request (s, o) started at round p: the summand of
 * M(X, t*) in Section 4, with the indicator taken inclusively and first use at p + 1. */
static int64_t held(int32_t s, int32_t o, int64_t p, int64_t tq)
{
    int64_t a = tq - p;
    return (a >= 1 && a <= (int64_t)o) ? (int64_t)s + a : 0;
}

int oracle_simulate_literal(int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                            const int32_t *order, int32_t *p_out, int32_t *c_out,
                            int64_t *tel_out)
{
    if (oracle_check_instance(n, s, o, M) != ORACLE_OK) return ORACLE_EINVAL;
    if (!is_permutation(n, order)) return ORACLE_EINVAL;
    int32_t *V = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1)); /* running requests */
    int64_t *p = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!V || !p) { free(V); free(p); return ORACLE_ENOMEM; }
    int32_t nV = 0, next = 0;
    int64_t tel = 0;
    for (int64_t t = 0; next < n; ++t) {
        /* (i) requests whose last token was produced at a round <= t have left */
        int32_t w = 0;
        for (int32_t a = 0; a < nV; ++a)
            if (p[V[a]] + o[V[a]] > t) V[w++] = V[a];
        nV = w;
        /* (ii) admit pending requests in order until the first one that does not fit */
        while (next < n) {
            int32_t r = order[next];
            p[r] = t; /* tentative */
            V[nV] = r;
            int64_t tmax = 0;
            for (int32_t a = 0; a <= nV; ++a) {
                int64_t cj = p[V[a]] + o[V[a]];
                if (cj > tmax) tmax = cj;
            }
            int feasible = 1;
            for (int64_t tq = t + 1; tq <= tmax && feasible; ++tq) {
                int64_t sum = 0;
                for (int32_t a = 0; a <= nV; ++a)
                    sum += held(s[V[a]], o[V[a]], p[V[a]], tq);
                if (sum > M) feasible = 0;
            }
            if (!feasible) break;
            ++nV;
            ++next;
            if (p_out) p_out[r] = (int32_t)t;
            if (c_out) c_out[r] = (int32_t)(t + o[r]);
            tel += t + o[r];
        }
        /* (iii) every running request produces one token; next round */
    }
    if (tel_out) *tel_out = tel;
    free(V);
    free(p);
    return ORACLE_OK;
}

/* ------------------------------------------- Phase 2 with the future memory in an array */

typedef struct {
    int64_t *P; /* P[tq] = memory held at round tq by everything admitted so far */
    int64_t cap;
} profile_t;

static int profile_reserve(profile_t *pf, int64_t need)
{
    if (need <= pf->cap) return 1;
    int64_t cap = pf->cap ? pf->cap : 1024;
    while (cap < need) cap *= 2;
    int64_t *q = (int64_t *)realloc(pf->P, sizeof(int64_t) * (size_t)cap);
    if (!q) return 0;
    memset(q + pf->cap, 0, sizeof(int64_t) * (size_t)(cap - pf->cap));
    pf->P = q;
    pf->cap = cap;
    return 1;
}

int oracle_simulate_profile(int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                            const int32_t *order, int32_t *p_out, int32_t *c_out,
                            int64_t *tel_out)
{
    if (oracle_check_instance(n, s, o, M) != ORACLE_OK) return ORACLE_EINVAL;
    if (!is_permutation(n, order)) return ORACLE_EINVAL;
    profile_t pf = {0, 0};
    int64_t tel = 0, t = 0;
    int32_t next = 0;
    while (next < n) {
        int32_t r = order[next];
        if (!profile_reserve(&pf, t + o[r] + 2)) { free(pf.P); return ORACLE_ENOMEM; }
        int feasible = 1;
        for (int64_t j = 1; j <= o[r]; ++j)
            if (pf.P[t + j] + s[r] + j > M) { feasible = 0; break; }
        if (!feasible) { ++t; continue; } /* nothing more is admitted this round */
        for (int64_t j = 1; j <= o[r]; ++j) pf.P[t + j] += s[r] + j;
        if (p_out) p_out[r] = (int32_t)t;
        if (c_out) c_out[r] = (int32_t)(t + o[r]);
        tel += t + o[r];
        ++next;
    }
    if (tel_out) *tel_out = tel;
    free(pf.P);
    return ORACLE_OK;
}

/* -------------------------------------------------------------- Phase 1 (sorted prefix) */

typedef struct { int64_t w; int64_t g; int32_t o; int32_t id; } skey_t;  /* g: effective length a s + b o */

static int cmp_size_o_id(const void *a, const void *b)
{
    const skey_t *x = (const skey_t *)a, *y = (const skey_t *)b;
    if (x->w != y->w) return x->w < y->w ? -1 : 1;
    if (x->o != y->o) return x->o < y->o ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

static int cmp_o_id(const void *a, const void *b)
{
    const skey_t *x = (const skey_t *)a, *y = (const skey_t *)b;
    if (x->o != y->o) return x->o < y->o ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

/* sign of F(Sa, ka) - F(Sb, kb) with F = S / k^2, in exact integers */
static int cmp_F(int64_t Sa, int64_t ka, int64_t Sb, int64_t kb)
{
    unsigned __int128 lhs = (unsigned __int128)Sa * (unsigned __int128)kb * (unsigned __int128)kb;
    unsigned __int128 rhs = (unsigned __int128)Sb * (unsigned __int128)ka * (unsigned __int128)ka;
    return (lhs > rhs) - (lhs < rhs);
}

/*
 * tie_rule 0: among equal F take the larger batch (the text of Section 4: minimise
 *             (F, -|X|)); tie_rule 1: take the smaller batch (the first minimum met when
 *             scanning k upward, as Algorithm 2's final loop does).
 * Batch feasibility: feas_mode 0, the sum of peaks, sum (s_i + o_i) <= M, as in Algorithms 2-4;
 * feas_mode 1, the constraint of Algorithm 1's Phase 1: with the whole batch started together
 * the memory at every member's completion time o_j, sum over {i: o_i >= o_j} of (s_i + o_j),
 * is <= M.  Both are monotone in the prefix length.
 * Outputs: order_out[n]; batch_end_out[b] = number of requests in batches 0..b;
 *          F_out[b] = F of batch b (one IEEE division of exact integers); *nb_out.
 */
int oracle_sortedG(int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t ga, int32_t gb,
                   int32_t tie_rule, int32_t feas_mode, int32_t *order_out, int32_t *batch_end_out,
                   double *F_out, int32_t *nb_out)
{
    if (oracle_check_instance(n, s, o, M) != ORACLE_OK) return ORACLE_EINVAL;
    if ((tie_rule != 0 && tie_rule != 1) || (feas_mode != 0 && feas_mode != 1)) return ORACLE_EINVAL;
    if (ga < 0 || gb < 1) return ORACLE_EINVAL;
    skey_t *rem = (skey_t *)malloc(sizeof(skey_t) * (size_t)(n + 1));
    int64_t *at_end = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!rem || !at_end) { free(rem); free(at_end); return ORACLE_ENOMEM; }
    for (int32_t i = 0; i < n; ++i) {
        rem[i].w = (int64_t)s[i] + o[i];
        rem[i].g = (int64_t)ga * s[i] + (int64_t)gb * o[i];
        rem[i].o = o[i];
        rem[i].id = i;
    }
    qsort(rem, (size_t)n, sizeof(skey_t), cmp_size_o_id);
    int32_t a = 0, nb = 0;
    while (a < n) {
        int64_t W = 0, S = 0, bestS = 0, bestk = 0;
        for (int64_t k = 1; a + k <= n; ++k) {
            const skey_t *e = &rem[a + k - 1];
            if (feas_mode == 0) {
                W += e->w;
                if (W > M) break;
            } else {
                /* at_end[j] = memory at the completion time of the j-th member when all start
                 * together; the newcomer adds s_e + o_j to every time o_j <= o_e, and its own
                 * completion time sees every member that lasts at least as long */
                int64_t own = 0, peak = 0;
                for (int64_t j = 0; j < k - 1; ++j) {
                    const skey_t *f = &rem[a + j];
                    if (e->o >= f->o) at_end[j] += (e->w - e->o) + f->o;
                    if (f->o >= e->o) own += (f->w - f->o) + e->o;
                }
                at_end[k - 1] = own + e->w;
                for (int64_t j = 0; j < k; ++j) if (at_end[j] > peak) peak = at_end[j];
                if (peak > M) break;
            }
            S += e->g;
            int better;
            if (bestk == 0) better = 1;
            else {
                int c = cmp_F(S, k, bestS, bestk);
                better = (c < 0) || (c == 0 && tie_rule == 0);
            }
            if (better) { bestS = S; bestk = k; }
        }
        /* the chosen batch runs shortest-output first */
        qsort(rem + a, (size_t)bestk, sizeof(skey_t), cmp_o_id);
        for (int64_t k = 0; k < bestk; ++k) order_out[a + k] = rem[a + k].id;
        a += (int32_t)bestk;
        if (batch_end_out) batch_end_out[nb] = a;
        if (F_out) F_out[nb] = (double)bestS / ((double)gb * (double)bestk * (double)bestk);
        ++nb;
    }
    if (nb_out) *nb_out = nb;
    free(rem);
    free(at_end);
    return ORACLE_OK;
}

int oracle_sortedF(int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t tie_rule,
                   int32_t feas_mode, int32_t *order_out, int32_t *batch_end_out, double *F_out,
                   int32_t *nb_out)
{
    return oracle_sortedG(n, s, o, M, 0, 1, tie_rule, feas_mode, order_out, batch_end_out, F_out, nb_out);
}

/* ---------------------------------------------------------- Phase 1 (Local Swap Search) */

/*
 * Local Swap Search, the search step: among the m candidates cand[0..m) (sorted by (s+o, o, id);
 * member[i] = 1 marks the batch) find the first exchange "member a out, outsider b in" that keeps the
 * batch within the budget (w_b - w_a <= slack, slack = M - load of the batch) and lowers the metric.
 * An exchange leaves |X| as it is, so the metric falls exactly when the numerator does: g_b < g_a.
 * "First" in the algorithm's scan order: members by sorted place, and for each member the outsiders
 * by sorted place.  stop_at_misfit != 0 leaves a member's scan at the first outsider that does not
 * fit (the outsiders behind it are at least as large).  Returns 1 and the pair, or 0.
 */
static int first_improving_exchange(const skey_t *cand, int32_t m, const unsigned char *member, int64_t slack,
                                    int stop_at_misfit, int32_t *a_out, int32_t *b_out)
{
    for (int32_t a = 0; a < m; ++a) {
        if (!member[a]) continue;
        for (int32_t b = 0; b < m; ++b) {
            if (member[b]) continue;
            if (cand[b].w - cand[a].w > slack) {
                if (stop_at_misfit) break;
                continue;
            }
            if (cand[b].g < cand[a].g) {
                *a_out = a;
                *b_out = b;
                return 1;
            }
        }
    }
    return 0;
}

/*
 * One batch by Local Swap Search: start from the greedy fill (walk the sorted candidates, take each
 * one that still fits under the sum of peaks), then apply the first improving exchange, search again
 * from the top, and so on until no exchange is left.  A request that came in by an exchange is
 * visited at its own sorted place from then on (membership is a mask over the sorted list).
 * Returns the number of exchanges; *S_out = the batch's numerator, *K_out = its size.
 */
static int64_t local_swap_batch(const skey_t *cand, int32_t m, int64_t M, int stop_at_misfit,
                                unsigned char *member, int64_t *S_out, int64_t *K_out)
{
    int64_t slack = M, numer = 0, size = 0, exchanges = 0;
    for (int32_t i = 0; i < m; ++i) {
        member[i] = (unsigned char)(cand[i].w <= slack);
        if (member[i]) {
            slack -= cand[i].w;
            numer += cand[i].g;
            ++size;
        }
    }
    int32_t a, b;
    while (first_improving_exchange(cand, m, member, slack, stop_at_misfit, &a, &b)) {
        member[a] = 0;
        member[b] = 1;
        slack -= cand[b].w - cand[a].w;
        numer += cand[b].g - cand[a].g;
        ++exchanges;
    }
    *S_out = numer;
    *K_out = size;
    return exchanges;
}

/*
 * Phase 1 of Algorithm 1 with Local Swap Search as the batch solver: choose a batch from the
 * remaining requests, append it in nondecreasing o (ties by id), remove it, repeat.
 * Outputs as oracle_sortedF, plus swaps_out[b] = exchanges made while forming batch b.
 */
int oracle_local_swap_G(int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t ga, int32_t gb,
                        int32_t early_exit, int32_t *order_out, int32_t *batch_end_out, double *F_out,
                        int32_t *swaps_out, int32_t *nb_out)
{
    if (oracle_check_instance(n, s, o, M) != ORACLE_OK) return ORACLE_EINVAL;
    if (ga < 0 || gb < 1) return ORACLE_EINVAL;
    skey_t *rem = (skey_t *)malloc(sizeof(skey_t) * (size_t)(n + 1));
    skey_t *batch = (skey_t *)malloc(sizeof(skey_t) * (size_t)(n + 1));
    unsigned char *inX = (unsigned char *)malloc((size_t)n + 1);
    if (!rem || !batch || !inX) { free(rem); free(batch); free(inX); return ORACLE_ENOMEM; }
    for (int32_t i = 0; i < n; ++i) {
        rem[i].w = (int64_t)s[i] + o[i];
        rem[i].g = (int64_t)ga * s[i] + (int64_t)gb * o[i];
        rem[i].o = o[i];
        rem[i].id = i;
    }
    qsort(rem, (size_t)n, sizeof(skey_t), cmp_size_o_id);
    int32_t m = n, done = 0, nb = 0;
    while (m > 0) {
        int64_t S = 0, K = 0;
        const int64_t swaps = local_swap_batch(rem, m, M, early_exit, inX, &S, &K);
        int32_t nbatch = 0, keep = 0;
        for (int32_t r = 0; r < m; ++r) {
            if (inX[r]) batch[nbatch++] = rem[r];
            else rem[keep++] = rem[r];  /* what remains stays sorted */
        }
        qsort(batch, (size_t)nbatch, sizeof(skey_t), cmp_o_id);
        for (int32_t k = 0; k < nbatch; ++k) order_out[done + k] = batch[k].id;
        done += nbatch;
        m = keep;
        if (batch_end_out) batch_end_out[nb] = done;
        if (F_out) F_out[nb] = (double)S / ((double)gb * (double)K * (double)K);
        if (swaps_out) swaps_out[nb] = (int32_t)swaps;
        ++nb;
    }
    if (nb_out) *nb_out = nb;
    free(rem);
    free(batch);
    free(inX);
    return ORACLE_OK;
}

int oracle_local_swap(int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t early_exit,
                      int32_t *order_out, int32_t *batch_end_out, double *F_out, int32_t *swaps_out,
                      int32_t *nb_out)
{
    return oracle_local_swap_G(n, s, o, M, 0, 1, early_exit, order_out, batch_end_out, F_out, swaps_out, nb_out);
}

/* -------------------------------------------------------------- Phase 1 (exact batches) */

typedef struct { int32_t o; int32_t id; } oid_t;

static int cmp_o_desc_id(const void *a, const void *b)
{
    const oid_t *x = (const oid_t *)a, *y = (const oid_t *)b;
    if (x->o != y->o) return x->o > y->o ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

/*
 * One exact batch over the requests ids[0..r) (ascending ids): the feasible subset of least metric,
 * found as Algorithm 2 finds it, by dynamic programming over (number of members, load).
 *   cost[c][L]  least numerator (sum of effective lengths) over the subsets of the requests offered
 *               so far that have c members and load exactly L; NONE if there is no such subset;
 *   lowered     one bit per (offer, c, L): that offer made cost[c][L] strictly smaller.
 * Requests are offered one at a time.  An offer extends subsets that do not hold the request yet,
 * i.e. the table as it stood before the offer: counts are visited downward, so a row is read before
 * this offer writes it.  A state is replaced only by a strictly smaller value.
 * feas_mode 0 (Algorithm 2 as printed): offers in input order, load = sum (s+o), which must stay <= M.
 * feas_mode 1 (the constraint of Algorithm 1's Phase 1: with all of X started together, memory
 *   at every completion time o_j, sum over {i in X: o_i >= o_j} of (s_i + o_j), is <= M):
 *   offers in order of decreasing o (ties by id), load = sum s; when request j joins c others it has
 *   the least o of the set, so the memory at time o_j is load + s_j + o_j (c + 1), which must be
 *   <= M; the constraints at the larger completion times were met when those requests joined and
 *   are not touched by j.  (Derived here; the paper gives no solver for this form.)
 * Choice of the state: least cost / c^2 over all states with c >= 1, compared exactly, scanning c
 *   upward and L upward.  tie_rule 1 keeps the first least value met (Algorithm 2's strict
 *   comparison); tie_rule 0 prefers the larger c among equal values (the text's (F, -|X|)), the
 *   first L met within that c.
 * Members of the chosen state: the subset a state stands for is the one of the last offer that
 *   lowered it, which extended the subset its predecessor (c - 1, L - load) stood for at that
 *   time.  So the offers are walked backward from the chosen state: an offer that lowered the
 *   state in hand is a member, and the walk goes on from the predecessor.
 * chosen[q] = 1 marks ids[q].  Returns 0, or ORACLE_ENOMEM.
 */
static int exact_batch(int32_t r, const int32_t *ids, const int32_t *s, const int32_t *o, int64_t M,
                       int32_t ga, int32_t gb, int32_t feas_mode, int32_t tie_rule, unsigned char *chosen,
                       int64_t *S_out, int64_t *K_out)
{
    const int64_t NONE = INT64_MAX;
    const size_t loads = (size_t)M + 1, counts = (size_t)r + 1, states = counts * loads;
    const size_t words = (states + 63) / 64;  /* bits of one offer */
    int64_t *cost = (int64_t *)malloc(sizeof(int64_t) * states);
    uint64_t *lowered = (uint64_t *)calloc((size_t)r * words, sizeof(uint64_t));
    oid_t *offer = (oid_t *)malloc(sizeof(oid_t) * (size_t)(r + 1));
    if (!cost || !lowered || !offer) { free(cost); free(lowered); free(offer); return ORACLE_ENOMEM; }
    for (size_t x = 0; x < states; ++x) cost[x] = NONE;
    cost[0] = 0;  /* the empty set */
    for (int32_t q = 0; q < r; ++q) { offer[q].o = o[ids[q]]; offer[q].id = q; }  /* id = place in ids[] */
    if (feas_mode == 1) qsort(offer, (size_t)r, sizeof(oid_t), cmp_o_desc_id);

    for (int32_t t = 0; t < r; ++t) {
        const int32_t i = ids[offer[t].id];
        const int64_t load = feas_mode == 1 ? (int64_t)s[i] : (int64_t)s[i] + o[i];
        const int64_t value = (int64_t)ga * s[i] + (int64_t)gb * o[i];
        uint64_t *bits = lowered + (size_t)t * words;
        for (int64_t c = t; c >= 0; --c) {  /* at most t members so far */
            for (int64_t L = 0; L + load <= M; ++L) {
                const int64_t from = cost[(size_t)c * loads + (size_t)L];
                if (from == NONE) continue;
                if (feas_mode == 1 && L + load + (int64_t)o[i] * (c + 1) > M) continue;
                const size_t to = (size_t)(c + 1) * loads + (size_t)(L + load);
                if (from + value < cost[to]) {
                    cost[to] = from + value;
                    bits[to / 64] |= 1ull << (to % 64);
                }
            }
        }
    }

    int64_t best_cost = 0, best_c = 0, best_L = 0;
    for (int64_t c = 1; c <= r; ++c) {
        for (int64_t L = 0; L <= M; ++L) {
            const int64_t v = cost[(size_t)c * loads + (size_t)L];
            if (v == NONE) continue;
            int take = best_c == 0;
            if (!take) {
                const int cmp = cmp_F(v, c, best_cost, best_c);
                take = cmp < 0 || (cmp == 0 && tie_rule == 0 && c > best_c);
            }
            if (take) { best_cost = v; best_c = c; best_L = L; }
        }
    }

    memset(chosen, 0, (size_t)r);
    int64_t c = best_c, L = best_L;
    for (int32_t t = r - 1; t >= 0 && c > 0; --t) {
        const size_t at = (size_t)c * loads + (size_t)L;
        if (!((lowered[(size_t)t * words + at / 64] >> (at % 64)) & 1)) continue;
        const int32_t q = offer[t].id, i = ids[q];
        chosen[q] = 1;
        L -= feas_mode == 1 ? (int64_t)s[i] : (int64_t)s[i] + o[i];
        --c;
    }
    *S_out = best_cost;
    *K_out = best_c;
    free(cost);
    free(lowered);
    free(offer);
    return c == 0 && L == 0 ? ORACLE_OK : ORACLE_EINVAL;  /* the walk must end at the empty set */
}

/*
 * Phase 1 of Algorithm 1 with exact batches: choose the batch, append it in nondecreasing o
 * (ties by id), remove it, repeat.  Outputs as oracle_sortedF.
 */
int oracle_exact_phase1_G(int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t ga, int32_t gb,
                          int32_t feas_mode, int32_t tie_rule, int32_t *order_out, int32_t *batch_end_out,
                          double *F_out, int32_t *nb_out)
{
    if (oracle_check_instance(n, s, o, M) != ORACLE_OK) return ORACLE_EINVAL;
    if (ga < 0 || gb < 1) return ORACLE_EINVAL;
    if ((tie_rule != 0 && tie_rule != 1) || (feas_mode != 0 && feas_mode != 1)) return ORACLE_EINVAL;
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    skey_t *batch = (skey_t *)malloc(sizeof(skey_t) * (size_t)(n + 1));
    unsigned char *inX = (unsigned char *)malloc((size_t)n + 1);
    if (!ids || !batch || !inX) { free(ids); free(batch); free(inX); return ORACLE_ENOMEM; }
    for (int32_t i = 0; i < n; ++i) ids[i] = i;
    int32_t r = n, done = 0, nb = 0, rc = ORACLE_OK;
    while (r > 0) {
        int64_t S = 0, K = 0;
        rc = exact_batch(r, ids, s, o, M, ga, gb, feas_mode, tie_rule, inX, &S, &K);
        if (rc != ORACLE_OK) break;
        int32_t nbatch = 0, keep = 0;
        for (int32_t q = 0; q < r; ++q) {
            if (inX[q]) { batch[nbatch].o = o[ids[q]]; batch[nbatch].id = ids[q]; batch[nbatch].w = 0; batch[nbatch].g = 0; ++nbatch; }
            else ids[keep++] = ids[q];
        }
        qsort(batch, (size_t)nbatch, sizeof(skey_t), cmp_o_id);
        for (int32_t k = 0; k < nbatch; ++k) order_out[done + k] = batch[k].id;
        done += nbatch;
        r = keep;
        if (batch_end_out) batch_end_out[nb] = done;
        if (F_out) F_out[nb] = (double)S / ((double)gb * (double)K * (double)K);
        ++nb;
    }
    if (nb_out) *nb_out = nb;
    free(ids);
    free(batch);
    free(inX);
    return rc;
}

int oracle_exact_phase1(int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t feas_mode,
                        int32_t tie_rule, int32_t *order_out, int32_t *batch_end_out, double *F_out,
                        int32_t *nb_out)
{
    return oracle_exact_phase1_G(n, s, o, M, 0, 1, feas_mode, tie_rule, order_out, batch_end_out, F_out, nb_out);
}

/* ----------------------------------------------------------------- neighbourhood moves */

/* type 0: exchange positions i and j.  type 1: take the entry at position i out and put it
 * back so that it lands at position j.  out may not alias base. */
int oracle_apply_move(int32_t n, const int32_t *base, int32_t type, int32_t i, int32_t j,
                      int32_t *out)
{
    if (i < 0 || j < 0 || i >= n || j >= n) return ORACLE_EINVAL;
    if (type == 0) {
        memcpy(out, base, sizeof(int32_t) * (size_t)n);
        out[i] = base[j];
        out[j] = base[i];
        return ORACLE_OK;
    }
    if (type == 1) {
        int32_t w = 0;
        for (int32_t k = 0; k < n; ++k) { /* base without position i ... */
            if (k == i) continue;
            if (w == j) out[w++] = base[i]; /* ... with base[i] placed at j */
            out[w++] = base[k];
        }
        if (w == j) out[w++] = base[i];
        return ORACLE_OK;
    }
    return ORACLE_EINVAL;
}

/* result_out = { index of the best move (lowest index among equal TEL), its TEL, TEL of base }.
 * literal != 0 scores with oracle_simulate_literal, else with oracle_simulate_profile. */
int oracle_best_neighbor(int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                         const int32_t *base, const int32_t *moves, int32_t K, int32_t literal,
                         int64_t *tel_out, int64_t *result_out)
{
    int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    if (!cand) return ORACLE_ENOMEM;
    int rc;
    int64_t base_tel = 0, best_tel = -1, best = -1;
    rc = literal ? oracle_simulate_literal(n, s, o, M, base, 0, 0, &base_tel)
                 : oracle_simulate_profile(n, s, o, M, base, 0, 0, &base_tel);
    for (int32_t m = 0; m < K && rc == ORACLE_OK; ++m) {
        rc = oracle_apply_move(n, base, moves[3 * m], moves[3 * m + 1], moves[3 * m + 2], cand);
        if (rc != ORACLE_OK) break;
        int64_t tel = 0;
        rc = literal ? oracle_simulate_literal(n, s, o, M, cand, 0, 0, &tel)
                     : oracle_simulate_profile(n, s, o, M, cand, 0, 0, &tel);
        if (tel_out) tel_out[m] = tel;
        if (best < 0 || tel < best_tel) { best = m; best_tel = tel; }
    }
    if (rc == ORACLE_OK && result_out) {
        result_out[0] = best;
        result_out[1] = best_tel;
        result_out[2] = base_tel;
    }
    free(cand);
    return rc;
}

/* Many orders in a row (row-major [C][n]); rows are independent.  tel_out[C];
 * c_out is [C][n] by request id or NULL. */
int oracle_simulate_many(int32_t n, const int32_t *s, const int32_t *o, int64_t M,
                         const int32_t *orders, int32_t C, int32_t literal, int64_t *tel_out,
                         int32_t *c_out)
{
    for (int32_t k = 0; k < C; ++k) {
        const int32_t *row = orders + (size_t)k * (size_t)n;
        int32_t *crow = c_out ? c_out + (size_t)k * (size_t)n : 0;
        int rc = literal ? oracle_simulate_literal(n, s, o, M, row, 0, crow, tel_out + k)
                         : oracle_simulate_profile(n, s, o, M, row, 0, crow, tel_out + k);
        if (rc != ORACLE_OK) return rc;
    }
    return ORACLE_OK;
}

/* ------------------------------------- Phase 2 under predicted decode lengths (A_min / A_max) */

/*
 * Section 5, "Handling Prediction Uncertainty via Adaptive Output Length Refinement", and the
 * appendix algorithm "Sorted-F + A_min".  The scheduler does not know o_i; it holds a running
 * estimate e_i (started from est0_i: the lower bound l_i for A_min, the upper bound u_i for the
 * conservative A_max, o_i itself for exact predictions) and runs Phase 2 with e_i in place of o_i:
 *
 * round t = 0, 1, 2, ...
 *   1. a running request started at p has produced a = t - p tokens.  If a = o_i it has finished:
 *      it leaves and c_i = t.  Otherwise it needs at least one more token: e_i <- max(e_i, a + 1).
 *   2. admission: the requests that wait are taken in the order's sequence; one is started at t if,
 *      with every running request j assumed to hold s_j + (tq - p_j) at the rounds
 *      tq = p_j + 1 .. p_j + e_j and nothing afterwards, memory stays <= M at every future round;
 *      the first that does not fit ends the round's admissions.
 *   3. eviction: while that projected memory exceeds M at some future round, the running request of
 *      least (e_i, i) is stopped: it loses what it has produced, keeps its e_i, and waits again at
 *      its own place of the order.
 * The paper's pseudo-code counts rounds from 1 and writes the update as max(e_i, t - p_i); with
 * rounds from 0 and a request occupying the rounds p + 1 .. p + o (the convention used throughout
 * this file) "has produced e_i tokens without completing" reads a + 1.
 *
 * literal != 0: the projected memory is re-summed from the running set for every future round;
 * else it is kept in an array and adjusted when an estimate grows, a request finishes before its
 * estimate, or one is stopped.
 * Outputs: p_out / c_out [n] start and completion round of the run that completed; tel = sum c_i;
 * evictions_out[i] = times request i was stopped; runs_out (may be NULL) receives up to max_runs
 * rows {request, start round, end round, 0 completed | 1 stopped}, *n_runs_out their number.
 */
int oracle_simulate_predicted(int32_t n, const int32_t *s, const int32_t *o, const int32_t *est0, int64_t M,
                              const int32_t *order, int32_t literal, int32_t *p_out, int32_t *c_out,
                              int64_t *tel_out, int32_t *evictions_out, int32_t *runs_out, int32_t max_runs,
                              int32_t *n_runs_out)
{
    if (oracle_check_instance(n, s, o, M) != ORACLE_OK) return ORACLE_EINVAL;
    if (!is_permutation(n, order)) return ORACLE_EINVAL;
    int64_t horizon = 4;
    for (int32_t i = 0; i < n; ++i) {
        if (est0[i] < 1 || (int64_t)s[i] + est0[i] > M) return ORACLE_EINVAL;
        if (est0[i] > horizon) horizon = est0[i];
        if (o[i] > horizon) horizon = o[i];
    }
    horizon += 2;  /* reservations never reach further ahead than the largest estimate */
    int32_t *est = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    int32_t *state = (int32_t *)calloc((size_t)n + 1, sizeof(int32_t)); /* 0 waits, 1 runs, 2 done */
    int64_t *p = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    int64_t *P = (int64_t *)calloc((size_t)horizon, sizeof(int64_t));  /* P[tq mod horizon], tq > t */
    if (!est || !state || !p || !P) { free(est); free(state); free(p); free(P); return ORACLE_ENOMEM; }
    memcpy(est, est0, sizeof(int32_t) * (size_t)n);
    if (evictions_out) memset(evictions_out, 0, sizeof(int32_t) * (size_t)n);
    int32_t done = 0, n_runs = 0;
    int64_t tel = 0;
#define PROJ(i, tq) (((tq) - p[i] >= 1 && (tq) - p[i] <= (int64_t)est[i]) ? (int64_t)s[i] + ((tq) - p[i]) : 0)
#define LOG_RUN(i, end, kind)                                                              \
    do {                                                                                   \
        if (runs_out && n_runs < max_runs) {                                               \
            runs_out[4 * n_runs] = (i); runs_out[4 * n_runs + 1] = (int32_t)p[i];          \
            runs_out[4 * n_runs + 2] = (int32_t)(end); runs_out[4 * n_runs + 3] = (kind);  \
        }                                                                                  \
        ++n_runs;                                                                          \
    } while (0)
    for (int64_t t = 0; done < n; ++t) {
        P[t % horizon] = 0;  /* round t is past */
        /* 1. progress of the running requests */
        for (int32_t i = 0; i < n; ++i) {
            if (state[i] != 1) continue;
            const int64_t a = t - p[i];
            if (a == o[i]) {  /* finished; what it had reserved beyond this round is released */
                if (!literal)
                    for (int64_t tq = t + 1; tq <= p[i] + est[i]; ++tq) P[tq % horizon] -= s[i] + (tq - p[i]);
                state[i] = 2;
                ++done;
                tel += t;
                if (p_out) p_out[i] = (int32_t)p[i];
                if (c_out) c_out[i] = (int32_t)t;
                LOG_RUN(i, t, 0);
            } else if (a + 1 > est[i]) {  /* still going: one more round is reserved */
                est[i] = (int32_t)(a + 1);
                if (!literal) P[(t + 1) % horizon] += s[i] + (a + 1);
            }
        }
        /* 2. admission in the order's sequence */
        for (int32_t k = 0; k < n; ++k) {
            const int32_t r = order[k];
            if (state[r] != 0) continue;
            int feasible = 1;
            if (literal) {
                p[r] = t;
                state[r] = 1;  /* tentatively */
                for (int64_t tq = t + 1; tq < t + horizon && feasible; ++tq) {
                    int64_t sum = 0;
                    for (int32_t j = 0; j < n; ++j)
                        if (state[j] == 1) sum += PROJ(j, tq);
                    if (sum > M) feasible = 0;
                }
                if (!feasible) state[r] = 0;
            } else {
                for (int64_t j = 1; j <= est[r] && feasible; ++j)
                    if (P[(t + j) % horizon] + s[r] + j > M) feasible = 0;
                if (feasible) {
                    for (int64_t j = 1; j <= est[r]; ++j) P[(t + j) % horizon] += s[r] + j;
                    p[r] = t;
                    state[r] = 1;
                }
            }
            if (!feasible) break;
        }
        /* 3. eviction while the projection overflows */
        for (;;) {
            int over = 0;
            for (int64_t tq = t + 1; tq < t + horizon && !over; ++tq) {
                int64_t sum = 0;
                if (literal) {
                    for (int32_t j = 0; j < n; ++j)
                        if (state[j] == 1) sum += PROJ(j, tq);
                } else {
                    sum = P[tq % horizon];
                }
                if (sum > M) over = 1;
            }
            if (!over) break;
            int32_t victim = -1;
            for (int32_t j = 0; j < n; ++j)
                if (state[j] == 1 && (victim < 0 || est[j] < est[victim])) victim = j;
            if (victim < 0) break;  /* cannot happen: an empty system holds nothing */
            if (!literal)
                for (int64_t tq = t + 1; tq <= p[victim] + est[victim]; ++tq)
                    P[tq % horizon] -= s[victim] + (tq - p[victim]);
            state[victim] = 0;
            if (evictions_out) ++evictions_out[victim];
            LOG_RUN(victim, t, 1);
        }
    }
#undef PROJ
#undef LOG_RUN
    if (tel_out) *tel_out = tel;
    if (n_runs_out) *n_runs_out = n_runs;
    free(est); free(state); free(p); free(P);
    return ORACLE_OK;
}
