/*
 * CPU oracle for scheduling under online arrivals.  TEST INFRASTRUCTURE ONLY: slow, single
 * threaded, written from the paper; the GPU library shares no code with it and must never
 * call it.
 *
 * Section 6, "Heuristics under Online Arrival" and Section 7, "Experiment under Online Poisson
 * Arrivals": request i becomes known at round a_i; at every iteration t the scheduler holds a
 * cached priority list over the backlog (arrived, not yet started), admits the longest prefix
 * of that list that passes the memory check of Eq. (1) against the requests that are running,
 * and from time to time recomputes the list.  Memory model and timing as in the offline
 * oracle (started at p: s + j tokens at round p + j, j = 1..o; completes at p + o); the latency
 * of a request is c_i - a_i.
 *
 * One iteration t, in this order:
 *   1. requests with a_i <= t that are not yet known join the END of the cached list, in
 *      arrival order (ties by id);
 *   2. if the backlog is not empty and a refresh is due, the whole backlog is re-ordered by the
 *      planner and becomes the new cached list.  A refresh is due when
 *        - the planned part of the list is used up (every entry left arrived after the last
 *          refresh; this also covers "never planned"), or
 *        - `period` iterations have passed since the last refresh, or
 *        - refresh_den > 0 and (entries that arrived since the last refresh and still wait)
 *          * refresh_den >= refresh_num * (backlog size at the last refresh);
 *   3. running requests that have completed (c_j <= t) leave; list entries are admitted from
 *      the front while they fit, stopping at the first that does not;
 *   4. t <- t + 1.
 *
 * Planners (what a refresh does with the backlog):
 *   0  arrival order (id)                          -- FCFS
 *   1  ascending decode length (o, id)             -- shortest decode first, MC-SF
 *   2  ascending footprint (s + o, o, id)          -- the paper's fallback order
 *   3  Sorted-F-Online: the backlog is sorted by (s + o, o, id); the first min(window, backlog)
 *      entries are re-ordered by Phase 1 of Algorithm 1 with Local Swap Search batches (over
 *      that window alone, budget M); the rest keeps the footprint order behind them.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)
#define ORACLE_ENOMEM (-2)

/* from kvsched_oracle.c */
int oracle_check_instance(int32_t n, const int32_t *s, const int32_t *o, int64_t M);
int oracle_local_swap(int32_t n, const int32_t *s, const int32_t *o, int64_t M, int32_t early_exit,
                      int32_t *order_out, int32_t *batch_end_out, double *F_out, int32_t *swaps_out,
                      int32_t *nb_out);

typedef struct { int64_t k1; int64_t k2; int32_t id; } okey_t;

static int cmp_okey(const void *a, const void *b)
{
    const okey_t *x = (const okey_t *)a, *y = (const okey_t *)b;
    if (x->k1 != y->k1) return x->k1 < y->k1 ? -1 : 1;
    if (x->k2 != y->k2) return x->k2 < y->k2 ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

static int cmp_i32(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Re-order list[0..len) (request ids) as the planner prescribes. */
static int plan(int32_t planner, int32_t window, const int32_t *s, const int32_t *o, int64_t M,
                int32_t *list, int32_t len)
{
    okey_t *keys = (okey_t *)malloc(sizeof(okey_t) * (size_t)(len + 1));
    if (!keys) return ORACLE_ENOMEM;
    for (int32_t q = 0; q < len; ++q) {
        const int32_t i = list[q];
        keys[q].id = i;
        keys[q].k1 = planner == 0 ? 0 : planner == 1 ? (int64_t)o[i] : (int64_t)s[i] + o[i];
        keys[q].k2 = planner >= 2 ? (int64_t)o[i] : 0;
    }
    qsort(keys, (size_t)len, sizeof(okey_t), cmp_okey);
    for (int32_t q = 0; q < len; ++q) list[q] = keys[q].id;
    free(keys);
    if (planner != 3) return ORACLE_OK;

    const int32_t wn = window < len ? window : len;
    if (wn <= 0) return ORACLE_OK;
    /* the look-ahead window as an instance of its own, members in ascending id so that the
     * batch solver's lowest-id tie-breaks are those of the whole problem */
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)wn);
    int32_t *sw = (int32_t *)malloc(sizeof(int32_t) * (size_t)wn);
    int32_t *ow = (int32_t *)malloc(sizeof(int32_t) * (size_t)wn);
    int32_t *ord = (int32_t *)malloc(sizeof(int32_t) * (size_t)wn);
    int rc = ORACLE_ENOMEM;
    if (ids && sw && ow && ord) {
        memcpy(ids, list, sizeof(int32_t) * (size_t)wn);
        qsort(ids, (size_t)wn, sizeof(int32_t), cmp_i32);
        for (int32_t q = 0; q < wn; ++q) { sw[q] = s[ids[q]]; ow[q] = o[ids[q]]; }
        rc = oracle_local_swap(wn, sw, ow, M, 0, ord, 0, 0, 0, 0);
        if (rc == ORACLE_OK)
            for (int32_t q = 0; q < wn; ++q) list[q] = ids[ord[q]];
    }
    free(ids); free(sw); free(ow); free(ord);
    return rc;
}

/* memory held at round tq by request (s, o) started at round p (first use at p + 1, the peak
 * s + o held at the completion round) */
static int64_t held_at(int32_t s, int32_t o, int64_t p, int64_t tq)
{
    const int64_t age = tq - p;
    return (age >= 1 && age <= (int64_t)o) ? (int64_t)s + age : 0;
}

/*
 * a[] nondecreasing, a_i >= 0.  period >= 1, window >= 0, refresh_num >= 0, refresh_den >= 0
 * (0 switches the backlog-growth trigger off).  literal != 0: Eq. (1) re-summed from the running
 * set for every future round; else the running set's future memory kept in an array.
 * Outputs: p_out[n], c_out[n] by request id;
 *          stats_out[4] = { sum (c_i - a_i), refreshes, last completion round, largest backlog }.
 */
int oracle_online(int32_t n, const int32_t *a, const int32_t *s, const int32_t *o, int64_t M,
                  int32_t planner, int32_t period, int32_t window, int32_t refresh_num,
                  int32_t refresh_den, int32_t literal, int32_t *p_out, int32_t *c_out,
                  int64_t *stats_out)
{
    if (oracle_check_instance(n, s, o, M) != ORACLE_OK) return ORACLE_EINVAL;
    if (planner < 0 || planner > 3 || period < 1 || window < 0 || refresh_num < 0 || refresh_den < 0)
        return ORACLE_EINVAL;
    int64_t horizon = 2;
    for (int32_t i = 0; i < n; ++i) {
        if (a[i] < 0 || (i > 0 && a[i] < a[i - 1])) return ORACLE_EINVAL;
        horizon += o[i];
    }
    if (n > 0) horizon += a[n - 1];  /* no schedule of this kind ends later: at worst one by one */

    int32_t *list = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    int32_t *V = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
    int64_t *p = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    int64_t *P = literal ? 0 : (int64_t *)calloc((size_t)horizon + 1, sizeof(int64_t));
    if (!list || !V || !p || (!literal && !P)) { free(list); free(V); free(p); free(P); return ORACLE_ENOMEM; }

    int32_t len = 0, planned_left = 0, known = 0, started = 0, nV = 0;
    int64_t t_plan = 0, backlog_at_plan = 0, refreshes = 0, total = 0, last_c = 0, max_backlog = 0;
    int rc = ORACLE_OK;
    for (int64_t t = 0; started < n && rc == ORACLE_OK; ++t) {
        /* 1. arrivals */
        while (known < n && a[known] <= t) list[len++] = known++;
        if (len > max_backlog) max_backlog = len;
        /* 2. refresh of the cached order */
        if (len > 0) {
            const int64_t newly = len - planned_left;
            const int due = planned_left == 0 || t - t_plan >= period ||
                            (refresh_den > 0 && newly * refresh_den >= (int64_t)refresh_num * backlog_at_plan);
            if (due) {
                rc = plan(planner, window, s, o, M, list, len);
                if (rc != ORACLE_OK) break;
                t_plan = t;
                backlog_at_plan = len;
                planned_left = len;
                ++refreshes;
            }
        }
        /* 3. departures, then admission of the longest feasible prefix */
        int32_t w = 0;
        for (int32_t q = 0; q < nV; ++q)
            if (p[V[q]] + o[V[q]] > t) V[w++] = V[q];
        nV = w;
        int32_t head = 0;
        while (head < len) {
            const int32_t r = list[head];
            int feasible = 1;
            if (literal) {
                p[r] = t;
                V[nV] = r;
                int64_t tmax = 0;
                for (int32_t q = 0; q <= nV; ++q)
                    if (p[V[q]] + o[V[q]] > tmax) tmax = p[V[q]] + o[V[q]];
                for (int64_t tq = t + 1; tq <= tmax && feasible; ++tq) {
                    int64_t sum = 0;
                    for (int32_t q = 0; q <= nV; ++q) sum += held_at(s[V[q]], o[V[q]], p[V[q]], tq);
                    if (sum > M) feasible = 0;
                }
            } else {
                for (int64_t j = 1; j <= o[r] && feasible; ++j)
                    if (P[t + j] + s[r] + j > M) feasible = 0;
            }
            if (!feasible) break;
            if (literal) ++nV;
            else for (int64_t j = 1; j <= o[r]; ++j) P[t + j] += s[r] + j;
            p[r] = t;
            if (p_out) p_out[r] = (int32_t)t;
            if (c_out) c_out[r] = (int32_t)(t + o[r]);
            total += t + o[r] - a[r];
            if (t + o[r] > last_c) last_c = t + o[r];
            ++started;
            ++head;
            if (planned_left > 0) --planned_left;
        }
        memmove(list, list + head, sizeof(int32_t) * (size_t)(len - head));
        len -= head;
    }
    if (rc == ORACLE_OK && stats_out) {
        stats_out[0] = total;
        stats_out[1] = refreshes;
        stats_out[2] = last_c;
        stats_out[3] = max_backlog;
    }
    free(list); free(V); free(p); free(P);
    return rc;
}
