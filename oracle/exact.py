"""Exact / exhaustive references on tiny instances -- TEST INFRASTRUCTURE ONLY.

  dp_best_batch        Algorithm 2 (exact DP over (k, m) states) for the Phase-1 batch.
  brute_best_batch     the same optimum by enumerating all subsets.
  optimal_start_times  exhaustive search over start rounds of the integer program of
                       Section 6 (Optimal-IP): the true optimum, for n <= 5 or so.
  lower_bound          an area / length bound on TEL valid for every feasible schedule.
"""
from __future__ import annotations

import itertools
from fractions import Fraction

import numpy as np

from .check import memory_per_round


def dp_best_batch(s, o, M):
    """Algorithm 2.  dp[k][m] = least sum of o over k-subsets with sum (s+o) == m <= M; the
    answer minimises dp[k][m] / k^2.  Returns (F as Fraction, set of k values attaining it,
    one subset per such k as a frozenset)."""
    n = len(s)
    INF = None
    dp = [dict() for _ in range(n + 1)]  # dp[k][m] -> (value, subset)
    dp[0][0] = (0, frozenset())
    for i in range(n):
        mi = int(s[i]) + int(o[i])
        for k in range(n - 1, -1, -1):
            for m, (val, sub) in list(dp[k].items()):
                nm = m + mi
                if nm > M:
                    continue
                nv = val + int(o[i])
                cur = dp[k + 1].get(nm, INF)
                if cur is None or nv < cur[0]:
                    dp[k + 1][nm] = (nv, sub | {i})
    best = None
    for k in range(1, n + 1):
        for m, (val, sub) in dp[k].items():
            F = Fraction(val, k * k)
            if best is None or F < best:
                best = F
    ks, subs = set(), {}
    for k in range(1, n + 1):
        for m, (val, sub) in dp[k].items():
            if Fraction(val, k * k) == best:
                ks.add(k)
                subs.setdefault(k, sub)
    return best, ks, subs


def batch_profile_peak(s, o, ids) -> int:
    """Largest memory of the set `ids` started together (Section 4's M(X, t) at the completion
    times): max over j in X of sum over {i in X : o_i >= o_j} of (s_i + o_j)."""
    return max(sum(int(s[i]) + int(o[j]) for i in ids if o[i] >= o[j]) for j in ids)


def brute_best_batch(s, o, M, profile: bool = False):
    """min of F(X) = sum o / |X|^2 over non-empty subsets with sum (s+o) <= M, or (profile) with
    the simultaneous-start memory profile <= M.  Returns (F*, set of sizes attaining it)."""
    n = len(s)
    best, ks = None, set()
    for mask in range(1, 1 << n):
        ids = [i for i in range(n) if mask >> i & 1]
        if profile:
            if batch_profile_peak(s, o, ids) > M:
                continue
        elif sum(int(s[i]) + int(o[i]) for i in ids) > M:
            continue
        F = Fraction(sum(int(o[i]) for i in ids), len(ids) ** 2)
        if best is None or F < best:
            best, ks = F, {len(ids)}
        elif F == best:
            ks.add(len(ids))
    return best, ks


def optimal_start_times(s, o, M, horizon=None):
    """Exhaustive Optimal-IP: min over start rounds p_i in [0, horizon] of sum (p_i + o_i)
    subject to memory <= M at every round.  Returns (TEL*, p*)."""
    n = len(s)
    T = int(np.sum(o)) if horizon is None else int(horizon)
    best, best_p = None, None
    for p in itertools.product(range(T + 1), repeat=n):
        tel = sum(p[i] + int(o[i]) for i in range(n))
        if best is not None and tel >= best:
            continue
        if (memory_per_round(s, o, p) <= M).all():
            best, best_p = tel, p
    return best, best_p


def lower_bound(s, o, M) -> int:
    """TEL >= sum_k max(ceil(A_k / M), o_(k)).

    By the k-th completion at least k requests have finished; they consumed at least A_k =
    the sum of the k smallest token-round areas a_i = s_i*o_i + o_i*(o_i+1)/2 out of the M
    tokens available per round, and the longest of them needed at least the k-th smallest
    decode length o_(k) rounds."""
    s = np.asarray(s, dtype=np.int64)
    o = np.asarray(o, dtype=np.int64)
    area = np.sort(s * o + o * (o + 1) // 2)
    A = np.cumsum(area)
    osort = np.sort(o)
    return int(np.maximum(-(-A // int(M)), osort).sum())
