"""Receding-horizon driver on the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Offline adaptation of the paper's Sorted-F-Online (Section 6, "Heuristics under Online
Arrival"): all requests present at round 0; plan on a look-ahead window of the not yet
committed part of the order by trying position moves inside it (move 0 is the identity), take
the best, run the order, wait until `complete_every` more requests have completed, commit every
position started by then, plan again.
"""
from __future__ import annotations

import numpy as np

from . import apply_move, best_neighbor, simulate


def horizon_step(s, o, M, order, moves, completed_in, complete_every, literal=False):
    n = len(order)
    tel, (best, best_tel, base_tel) = best_neighbor(s, o, M, order, moves, literal=literal)
    new_order = apply_move(order, moves[best])
    p, c, _ = simulate(s, o, M, new_order, literal=literal)
    k = min(n, completed_in + complete_every)
    T = int(np.sort(c)[k - 1])  # round by which k requests have completed
    completed = int((c <= T).sum())
    committed = int((p[new_order] <= T).sum())  # a prefix: starts are nondecreasing along the order
    assert (p[new_order][:committed] <= T).all()
    return new_order, c, tel, (best, best_tel, base_tel, committed, completed, T)


def receding_horizon(s, o, M, base_order, draw_moves, window, complete_every, literal=False, max_steps=None):
    """draw_moves(lo, hi) -> moves [K, 3] inside positions [lo, hi).  Returns (order, completion, records)."""
    n = len(base_order)
    order = np.array(base_order, dtype=np.int32)
    committed, completed, log, c = 0, 0, [], None
    while committed < n and (max_steps is None or len(log) < max_steps):
        lo, hi = committed, min(n, committed + window)
        moves = draw_moves(lo, hi)
        order, c, tel, r = horizon_step(s, o, M, order, moves, completed, complete_every, literal)
        log.append(dict(lo=lo, hi=hi, best=r[0], best_tel=r[1], base_tel=r[2], committed=r[3], completed=r[4], T=r[5],
                        tel=tel))
        committed, completed = r[3], r[4]
    return order, c, log
