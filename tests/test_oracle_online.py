"""Pins of the online-arrival oracle (Section 6, "Heuristics under Online Arrival")."""
import os

import numpy as np
import pytest

import oracle
from oracle import check
from paper_2508_06133_amd import workloads
from conftest import read_golden

FCFS, MCSF, FOOT, SORTF = (oracle.PLANNER_ARRIVAL, oracle.PLANNER_SHORTEST_DECODE,
                           oracle.PLANNER_FOOTPRINT, oracle.PLANNER_SORTED_F)
NEVER = 1 << 30  # a refresh period no run reaches


def _ints(txt):
    return [int(x) for x in txt.split()]


def _random_offline(rng):
    n = int(rng.integers(1, 40))
    smax, omax = int(rng.integers(1, 30)), int(rng.integers(1, 30))
    M = int(rng.integers(smax + omax, 5 * (smax + omax)))
    s = rng.integers(1, smax + 1, n).astype(np.int32)
    o = rng.integers(1, omax + 1, n).astype(np.int32)
    return s, o, M


def _random_online(rng, nmax=40, tmax=60):
    s, o, M = _random_offline(rng)
    n = len(s)
    a = np.sort(rng.integers(0, int(rng.integers(1, tmax)), n)).astype(np.int32)
    return a, s, o, M


@pytest.mark.parametrize("literal", [True, False])
def test_hand_worked_trace(golden_dir, literal):
    g = read_golden(os.path.join(golden_dir, "online_worked.txt"))
    a, s, o = _ints(g["a"]), _ints(g["s"]), _ints(g["o"])
    p, c, stats = oracle.online(a, s, o, int(g["M"]), SORTF, int(g["period"]), int(g["window"]),
                                tuple(_ints(g["refresh"])), literal=literal)
    assert list(p) == _ints(g["start"])
    assert list(c) == [x + y for x, y in zip(_ints(g["start"]), o)]
    assert stats == (int(g["total_latency"]), int(g["refreshes"]), int(g["last_completion"]), int(g["max_backlog"]))


def test_example1_online_with_everything_present(golden_dir):
    # Example 1 (Section 4) with all requests arriving at round 0: shortest-decode-first gives
    # the paper's 64, the F-based order its 45.
    g = read_golden(os.path.join(golden_dir, "example1.txt"))
    s1, o1, n1 = _ints(g["type1"])
    s2, o2, n2 = _ints(g["type2"])
    s = [s1] * n1 + [s2] * n2
    o = [o1] * n1 + [o2] * n2
    a = [0] * (n1 + n2)
    M = int(g["M"])
    assert oracle.online(a, s, o, M, MCSF, 1, 0, (0, 0), literal=True)[2][0] == int(g["tel_mcsf"])
    assert oracle.online(a, s, o, M, SORTF, 10, 300, (1, 2), literal=True)[2][0] == int(g["tel_sortedF"])


def test_all_present_at_round_zero_reduces_to_the_offline_executor():
    # With a_i = 0 the cached list of a simple planner is one fixed order, so the run must equal
    # Phase 2 of Algorithm 1 on that order; for Sorted-F-Online with one refresh and a window that
    # covers everything it must equal Local Swap Search's order run through Phase 2.
    rng = np.random.default_rng(11)
    for trial in range(150):
        s, o, M = _random_offline(rng)
        n = len(s)
        a = np.zeros(n, dtype=np.int32)
        w = s.astype(np.int64) + o
        ids = np.arange(n)
        orders = {
            FCFS: ids,
            MCSF: np.lexsort((ids, o)),
            FOOT: np.lexsort((ids, o, w)),
            SORTF: oracle.local_swap(s, o, M)[0],
        }
        for planner, order in orders.items():
            p0, c0, tel0 = oracle.simulate(s, o, M, order, literal=True)
            for period in (1, 3, NEVER):
                if planner == SORTF and period != NEVER:
                    continue  # re-planning the remainder regroups it; only the single plan is the offline order
                for literal in (True, False):
                    p, c, stats = oracle.online(a, s, o, M, planner, period, n, (0, 0), literal=literal)
                    assert (p == p0).all() and (c == c0).all() and stats[0] == tel0, (trial, planner, period)
                    assert stats[2] == c0.max() and stats[3] == n


def test_literal_and_profile_forms_agree_under_arrivals():
    rng = np.random.default_rng(12)
    for trial in range(200):
        a, s, o, M = _random_online(rng)
        planner = int(rng.integers(0, 4))
        period = int(rng.integers(1, 8))
        window = int(rng.integers(0, 12))
        refresh = (int(rng.integers(0, 4)), int(rng.integers(0, 4)))
        x = oracle.online(a, s, o, M, planner, period, window, refresh, literal=True)
        y = oracle.online(a, s, o, M, planner, period, window, refresh, literal=False)
        assert (x[0] == y[0]).all() and (x[1] == y[1]).all() and x[2] == y[2], trial


def _replay_simple_planner(a, s, o, M, key, p):
    """From the definition, for a planner that re-sorts the whole backlog at every iteration:
    at each round the requests started are exactly the longest prefix of the sorted backlog that
    fits beside everything started earlier (dense occupancy tables, oracle/check.py)."""
    n = len(s)
    placed_ids, placed_p = [], []
    for t in range(int(p.max()) + 1):
        backlog = sorted((i for i in range(n) if a[i] <= t and p[i] >= t), key=key)
        blocked = False
        for r in backlog:
            fits = check.fits(s, o, placed_p, placed_ids, r, t, M)
            if p[r] == t:
                if blocked or not fits:
                    return False  # started behind a blocked request, or without room
                placed_ids.append(r)
                placed_p.append(t)
            else:
                if not blocked and fits:
                    return False  # head of the list had room and was not started
                blocked = True
    return True


def test_every_iteration_planners_against_the_definition():
    rng = np.random.default_rng(13)
    for trial in range(60):
        a, s, o, M = _random_online(rng, nmax=25, tmax=40)
        w = s.astype(np.int64) + o
        keys = {
            FCFS: lambda i: i,
            MCSF: lambda i: (int(o[i]), i),
            FOOT: lambda i: (int(w[i]), int(o[i]), i),
        }
        for planner, key in keys.items():
            p, c, stats = oracle.online(a, s, o, M, planner, 1, 0, (0, 0), literal=True)
            assert (p >= a).all() and (c == p + o).all()
            assert check.is_feasible(s, o, p, M)
            assert _replay_simple_planner(a, s, o, M, key, p), (trial, planner)
            assert stats[0] == int((c.astype(np.int64) - a).sum()) and stats[2] == int(c.max())
    # a planted mistake must be seen: start one blocked request a round early
    a, s, o, M = [0, 0], [5, 5], [3, 3], 10
    p, c, _ = oracle.online(a, s, o, M, FCFS, 1, 0, (0, 0), literal=True)
    assert list(p) == [0, 3]
    assert not check.is_feasible(s, o, np.array([0, 2]), M)
    assert not _replay_simple_planner(np.array(a), np.array(s), np.array(o), M, lambda i: i, np.array([0, 4]))


def test_sorted_f_online_schedules_are_valid_and_use_the_window():
    rng = np.random.default_rng(14)
    for trial in range(100):
        a, s, o, M = _random_online(rng)
        period = int(rng.integers(1, 12))
        window = int(rng.integers(0, 15))
        p, c, stats = oracle.online(a, s, o, M, SORTF, period, window, (1, 2))
        assert (p >= a).all() and (c == p + o).all() and check.is_feasible(s, o, p, M)
        assert stats[0] >= int(o.sum())
    # window 0 leaves only the footprint order: the run equals the footprint planner's with the
    # same refresh times
    for trial in range(50):
        a, s, o, M = _random_online(rng)
        period = int(rng.integers(1, 6))
        x = oracle.online(a, s, o, M, SORTF, period, 0, (1, 2))
        y = oracle.online(a, s, o, M, FOOT, period, 0, (1, 2))
        assert (x[0] == y[0]).all() and x[2] == y[2]


def test_refresh_triggers_in_closed_form():
    # (a) room for everything: each arrival finds an empty list, is planned and started at once;
    #     refreshes = number of rounds with arrivals, latency = decode length.
    a = np.array([0, 0, 3, 4, 4, 4, 9], dtype=np.int32)
    s = np.full(7, 2, dtype=np.int32)
    o = np.array([5, 1, 2, 7, 1, 3, 2], dtype=np.int32)
    for planner in (FCFS, MCSF, FOOT, SORTF):
        p, c, stats = oracle.online(a, s, o, 10_000, planner, 10, 300, (1, 2), literal=True)
        assert (p == a).all() and stats == (int(o.sum()), 4, 11, 3)
    # (b) one request blocked for 49 rounds behind a long one, nobody else arrives: the list is
    #     refreshed when it is first filled and then every `period` iterations until it starts.
    a, s, o, M = [0, 1], [50, 60], [50, 30], 100
    for period, expect in ((10, 1 + 5), (7, 1 + 8), (49, 1 + 2), (50, 1 + 1), (1, 1 + 50)):
        p, c, stats = oracle.online(a, s, o, M, FCFS, period, 0, (0, 0), literal=True)
        assert list(p) == [0, 50] and stats[1] == expect, period
    # (c) growth trigger: behind the blocked request one newcomer per round; the backlog at the last
    #     refresh was B, the next refresh comes when ceil(B * num / den) newcomers wait.
    n_new = 12
    a = [0, 1] + [2 + k for k in range(n_new)]
    s = [50, 60] + [1] * n_new
    o = [50, 30] + [1] * n_new
    p, c, stats = oracle.online(a, s, o, M, FCFS, NEVER, 0, (1, 2), literal=True)
    # refreshes at t=0 (B=1), t=1 (list used up, B=1), then t=2 (1 newcomer >= 1/2, B=2), t=3 (B=3),
    # t=5 (2 newcomers >= 3/2, B=5), t=8 (3 >= 5/2, B=8), t=12 (4 >= 4, B=12)
    assert stats[1] == 7
    p, c, stats = oracle.online(a, s, o, M, FCFS, NEVER, 0, (2, 1), literal=True)
    # threshold 2 B: t=0, t=1 (B=1), t=3 (2 newcomers, B=3), t=9 (6 newcomers, B=9)
    assert stats[1] == 4
    p, c, stats = oracle.online(a, s, o, M, FCFS, NEVER, 0, (0, 0), literal=True)
    assert stats[1] == 2  # trigger off: only the two "list used up" refreshes


def test_rejects_malformed_input():
    with pytest.raises(oracle.OracleError):
        oracle.online([1, 0], [1, 1], [1, 1], 10, FCFS)  # arrivals out of order
    with pytest.raises(oracle.OracleError):
        oracle.online([0], [8], [8], 10, FCFS)  # can never fit
    with pytest.raises(oracle.OracleError):
        oracle.online([0], [1], [1], 10, 4)  # unknown planner
    with pytest.raises(oracle.OracleError):
        oracle.online([0], [1], [1], 10, FCFS, period=0)


def test_poisson_workload_shape():
    lam = workloads.online_lambda_star()
    a, s, o, M = workloads.online_instance(0, 1.0)
    assert M == workloads.ONLINE_M and (np.diff(a) >= 0).all() and a.min() >= 0 and a.max() < workloads.ONLINE_T
    assert abs(len(a) - lam * workloads.ONLINE_T) < 5 * np.sqrt(lam * workloads.ONLINE_T)
    assert (s + o <= M).all() and s.min() >= 1 and o.min() >= 1
    a2, s2, o2, _ = workloads.online_instance(0, 1.0)
    assert (a == a2).all() and (s == s2).all() and (o == o2).all()
    # overload ordering the paper reports (Section 7): with a deep backlog the F-based policy
    # beats shortest-decode-first, which beats arrival order
    a, s, o, M = workloads.online_instance(1, 2.4)
    lat = [oracle.online(a, s, o, M, pl, per, 300, (1, 2))[2][0] for pl, per in ((FCFS, 1), (MCSF, 1), (SORTF, 10))]
    assert lat[2] < lat[1] < lat[0]
