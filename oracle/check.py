"""Direct-definition checks of a schedule -- TEST INFRASTRUCTURE ONLY.

Written independently of the simulators in kvsched_oracle.c: it builds the whole
(request x round) occupancy table from the start rounds and the memory model of
Section 2 ("the memory required to generate the j-th output token is s_i + j") under
the integer program's timing (start k => rounds k+1..k+o_i, Section 6), and tests
 (a) the memory constraint at every round,
 (b) that each start round is the earliest one >= the previous request's start at which
     the request fits next to all requests placed before it (the greedy in-order
     admission of Algorithm 1, Phase 2).
Dense numpy; small instances only.
"""
from __future__ import annotations

import numpy as np


def occupancy(s, o, p, horizon=None):
    """U[i, t] = tokens held by request i at round t (0 when it is not running)."""
    s = np.asarray(s, dtype=np.int64)
    o = np.asarray(o, dtype=np.int64)
    p = np.asarray(p, dtype=np.int64)
    T = int((p + o).max()) + 1 if horizon is None else int(horizon)
    t = np.arange(T, dtype=np.int64)[None, :]
    age = t - p[:, None]
    running = (age >= 1) & (age <= o[:, None])
    return np.where(running, s[:, None] + age, 0)


def memory_per_round(s, o, p, horizon=None):
    return occupancy(s, o, p, horizon).sum(axis=0)


def is_feasible(s, o, p, M) -> bool:
    return bool((memory_per_round(s, o, p) <= M).all())


def fits(s, o, p_placed, ids_placed, r, t, M) -> bool:
    """Does request r started at round t fit beside the already placed requests?"""
    ids = list(ids_placed) + [r]
    starts = list(p_placed) + [t]
    ss = np.asarray(s)[ids]
    oo = np.asarray(o)[ids]
    horizon = int(max(np.asarray(starts) + oo)) + 1
    mem = memory_per_round(ss, oo, starts, horizon)
    return bool((mem[t + 1 :] <= M).all())


def is_greedy_in_order(s, o, M, order, p) -> bool:
    """p is exactly what in-order earliest admission produces for `order`."""
    placed_ids, placed_p = [], []
    t_prev = 0
    for r in order:
        r = int(r)
        t = int(p[r])
        if t < t_prev:
            return False
        for tt in range(t_prev, t):
            if fits(s, o, placed_p, placed_ids, r, tt, M):
                return False  # could have started earlier
        if not fits(s, o, placed_p, placed_ids, r, t, M):
            return False
        placed_ids.append(r)
        placed_p.append(t)
        t_prev = t
    return True
