"""The receding-horizon driver of the CPU oracle against an example worked by hand
(tests/golden/horizon_worked.txt): the latencies of every candidate, the chosen move, the timeline and
the commit rule (T = the k-th smallest completion, requests completed by T, positions started by T) of
every step.  The example has two completions that coincide at T and a start exactly at T, so that an
index or a comparison that is off by one changes a number.
"""
import os

import numpy as np
import pytest

from conftest import read_golden
from oracle import horizon as ohorizon


def ints(text):
    return [int(x) for x in text.split()]


def worked_moves(lo, hi):
    """The example's candidates for a window [lo, hi): identity, swap(lo, lo+1), swap(lo+1, lo+2),
    insert(lo+2 -> lo), as far as they fit."""
    mv = [(0, lo, lo)]
    if hi - lo >= 2:
        mv.append((0, lo, lo + 1))
    if hi - lo >= 3:
        mv += [(0, lo + 1, lo + 2), (1, lo + 2, lo)]
    return np.array(mv, dtype=np.int32)


def load_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "horizon_worked.txt"))
    s, o = np.array(ints(g["s"]), dtype=np.int32), np.array(ints(g["o"]), dtype=np.int32)
    return g, s, o, int(g["M"]), np.array(ints(g["base_order"]), dtype=np.int32)


@pytest.mark.parametrize("literal", [True, False])
def test_hand_worked_receding_horizon(golden_dir, literal):
    g, s, o, M, base = load_example(golden_dir)
    order, c, log = ohorizon.receding_horizon(s, o, M, base, worked_moves, int(g["window"]), int(g["complete_every"]),
                                              literal=literal)
    assert len(log) == int(g["steps"])
    for k, rec in enumerate(log, start=1):
        assert [rec["lo"], rec["hi"]] == ints(g[f"step{k}_lo_hi"])
        assert list(rec["tel"]) == ints(g[f"step{k}_tel"])
        assert rec["best"] == int(g[f"step{k}_best"])
        assert rec["best_tel"] == min(ints(g[f"step{k}_tel"])) and rec["base_tel"] == ints(g[f"step{k}_tel"])[0]
        assert [rec["T"], rec["completed"], rec["committed"]] == ints(g[f"step{k}_T_completed_committed"])
    assert list(order) == ints(g["step3_order"]) and list(c) == ints(g["step3_completion"])


@pytest.mark.parametrize("literal", [True, False])
def test_hand_worked_single_steps(golden_dir, literal):
    g, s, o, M, base = load_example(golden_dir)
    order, completed = base, 0
    for k in (1, 2, 3):
        lo, hi = ints(g[f"step{k}_lo_hi"])
        new_order, c, tel, res = ohorizon.horizon_step(s, o, M, order, worked_moves(lo, hi), completed,
                                                       int(g["complete_every"]), literal=literal)
        T, done, committed = ints(g[f"step{k}_T_completed_committed"])
        assert list(new_order) == ints(g[f"step{k}_order"]) and list(c) == ints(g[f"step{k}_completion"])
        assert res == (int(g[f"step{k}_best"]), min(ints(g[f"step{k}_tel"])), ints(g[f"step{k}_tel"])[0], committed, done, T)
        order, completed = new_order, done


def test_worked_example_is_consistent_with_the_model(golden_dir):
    # the file's own numbers against the definition: occupancy of every round within M, completions =
    # start + o, starts nondecreasing along the order, totals = sums of completions
    g, s, o, M, _ = load_example(golden_dir)
    for k in (1, 2, 3):
        order, p, c = ints(g[f"step{k}_order"]), np.array(ints(g[f"step{k}_start"])), np.array(ints(g[f"step{k}_completion"]))
        assert (c == p + o).all() and (np.diff(p[order]) >= 0).all()
        assert int(c.sum()) == ints(g[f"step{k}_tel"])[int(g[f"step{k}_best"])]
        for tq in range(1, int(c.max()) + 1):
            held = [(s[i] + tq - p[i]) for i in range(len(s)) if p[i] < tq <= c[i]]
            assert sum(held) <= M
