"""Pins of the oracle for Phase 2 under predicted decode lengths (running estimates, ordered
eviction: Section 5 and the appendix algorithm "Sorted-F + A_min")."""
import os

import numpy as np
import pytest

import oracle
from paper_2508_06133_amd import workloads
from conftest import read_golden


def _ints(txt):
    return [int(x) for x in txt.split()]


def _instance(rng, nmax=12):
    n = int(rng.integers(1, nmax + 1))
    smax, omax = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    M = int(rng.integers(smax + omax, 4 * (smax + omax)))
    s = rng.integers(1, smax + 1, n).astype(np.int32)
    o = rng.integers(1, omax + 1, n).astype(np.int32)
    return s, o, M, rng.permutation(n).astype(np.int32)


def _lower(rng, o):
    return np.array([int(rng.integers(1, x + 1)) for x in o], dtype=np.int32)


def _upper(rng, s, o, M):
    return np.array([int(rng.integers(x, M - sv + 1)) for sv, x in zip(s, o)], dtype=np.int32)


def _true_memory(s, o, runs, T):
    """Tokens really held per round, from the log of runs: a run started at p holds s + j at
    round p + j while it lasts (a stopped run to its last round, a completed one for o rounds)."""
    mem = np.zeros(T + 2, dtype=np.int64)
    for r, start, end, kind in runs:
        for tq in range(start + 1, end + 1):
            mem[tq] += int(s[r]) + (tq - start)
    return mem


@pytest.mark.parametrize("literal", [True, False])
def test_hand_worked_example(golden_dir, literal):
    g = read_golden(os.path.join(golden_dir, "predicted_worked.txt"))
    s, o, M, order = _ints(g["s"]), _ints(g["o"]), int(g["M"]), _ints(g["order"])
    p, c, tel, ev, runs = oracle.simulate_predicted(s, o, _ints(g["lower"]), M, order, literal, max_runs=16)
    assert list(p) == _ints(g["amin_start"]) and list(c) == _ints(g["amin_completion"])
    assert tel == int(g["amin_tel"]) and list(ev) == _ints(g["amin_evictions"])
    assert runs.reshape(-1).tolist() == _ints(g["amin_runs"])
    p, c, tel, ev, runs = oracle.simulate_predicted(s, o, _ints(g["upper"]), M, order, literal, max_runs=16)
    assert list(p) == _ints(g["amax_start"]) and list(c) == _ints(g["amax_completion"])
    assert tel == int(g["amax_tel"]) and ev.sum() == 0 and len(runs) == 4


def test_exact_predictions_reduce_to_phase_two():
    rng = np.random.default_rng(61)
    for trial in range(200):
        s, o, M, order = _instance(rng)
        p0, c0, tel0 = oracle.simulate(s, o, M, order, literal=True)
        for literal in (True, False):
            p, c, tel, ev, _ = oracle.simulate_predicted(s, o, o, M, order, literal)
            assert (p == p0).all() and (c == c0).all() and tel == tel0 and ev.sum() == 0, trial
    for cfg in (2, 3):
        inst = workloads.instance(cfg, n=300)
        order = oracle.sortedF(inst.s, inst.o, inst.M)[0]
        p0, c0, tel0 = oracle.simulate(inst.s, inst.o, inst.M, order, literal=False)
        p, c, tel, ev, _ = oracle.simulate_predicted(inst.s, inst.o, inst.o, inst.M, order)
        assert (c == c0).all() and tel == tel0 and ev.sum() == 0


def test_literal_and_array_forms_agree():
    rng = np.random.default_rng(62)
    for trial in range(300):
        s, o, M, order = _instance(rng)
        est = _lower(rng, o) if trial % 3 else _upper(rng, s, o, M)
        if trial % 5 == 0:  # mixed: some under-, some over-estimated
            est = np.where(rng.random(len(o)) < 0.5, _lower(rng, o), _upper(rng, s, o, M)).astype(np.int32)
        a = oracle.simulate_predicted(s, o, est, M, order, True, max_runs=4000)
        b = oracle.simulate_predicted(s, o, est, M, order, False, max_runs=4000)
        assert (a[0] == b[0]).all() and (a[1] == b[1]).all() and a[2] == b[2]
        assert (a[3] == b[3]).all() and (a[4] == b[4]).all(), trial


def test_memory_really_held_never_exceeds_the_budget_and_runs_are_consistent():
    rng = np.random.default_rng(63)
    seen_evictions = 0
    for trial in range(300):
        s, o, M, order = _instance(rng, 14)
        est = np.where(rng.random(len(o)) < 0.7, _lower(rng, o), _upper(rng, s, o, M)).astype(np.int32)
        p, c, tel, ev, runs = oracle.simulate_predicted(s, o, est, M, order, False, max_runs=4000)
        mem = _true_memory(s, o, runs, int(c.max()))
        assert (mem <= M).all(), trial
        assert tel == int(c.astype(np.int64).sum()) and (c == p + o).all()
        # every request has exactly one completed run, its last; stopped runs are shorter than o
        for i in range(len(s)):
            mine = [r for r in runs if r[0] == i]
            assert [r[3] for r in mine] == [1] * int(ev[i]) + [0]
            assert mine[-1][1] == p[i] and mine[-1][2] == c[i]
            assert all(r[2] - r[1] < o[i] for r in mine[:-1])
            assert all(mine[k][2] <= mine[k + 1][1] for k in range(len(mine) - 1))
        seen_evictions += int(ev.sum())
    assert seen_evictions > 50  # the cases do exercise the eviction step


def test_over_estimates_never_evict_and_cost_latency():
    # A_max (upper bounds throughout) over-reserves: no eviction, and on the chat workload a higher
    # total latency than exact predictions (the degradation the paper describes)
    rng = np.random.default_rng(64)
    for trial in range(100):
        s, o, M, order = _instance(rng)
        p, c, tel, ev, runs = oracle.simulate_predicted(s, o, _upper(rng, s, o, M), M, order, False, max_runs=100)
        assert ev.sum() == 0 and len(runs) == len(s)
    inst = workloads.instance(2)
    order = oracle.sortedF(inst.s, inst.o, inst.M)[0]
    upper = np.minimum(2 * inst.o, inst.M - inst.s).astype(np.int32)
    exact = oracle.simulate_predicted(inst.s, inst.o, inst.o, inst.M, order)[2]
    amax = oracle.simulate_predicted(inst.s, inst.o, upper, inst.M, order)[2]
    assert amax > exact


def test_the_stopped_request_has_the_least_estimate():
    # two requests side by side, the one with the smaller estimate is stopped when the other
    # outgrows its estimate: (s=4, o=3, l=3) and (s=1, o=6, l=2), budget 12.
    # t=0 both start (rounds 1,2: 5+2, 6+3; round 3: 7).  t=2: the second goes on (estimate 3): round 3
    # holds 7 + 4 = 11.  t=3: the first finishes; the second alone from here: c = 6.  No eviction.
    p, c, tel, ev, runs = oracle.simulate_predicted([4, 1], [3, 6], [3, 2], 12, [0, 1], True, max_runs=8)
    assert list(c) == [3, 6] and ev.sum() == 0
    # budget 10: at t=2 round 3 would hold 11 > 10; estimates are 3 and 3 -> the lower id (the first)
    # is stopped although it is the second that grew.  It restarts at t=3 (rounds 4-6: 5,6,7 beside
    # 5 at round 4) and is stopped again at t=4, when the second's estimate 5 puts 6 + 6 on round 5
    # and its own 3 is the smaller; it runs for good from t=6, when the second has finished.
    p, c, tel, ev, runs = oracle.simulate_predicted([4, 1], [3, 6], [3, 2], 10, [0, 1], True, max_runs=8)
    assert list(ev) == [2, 0] and list(c) == [9, 6]
    assert runs.tolist() == [[0, 0, 2, 1], [0, 3, 4, 1], [1, 0, 6, 0], [0, 6, 9, 0]]
    # with the first estimated longer (l = 4, o = 4) the second (estimate 3 < 4) is the one stopped
    p, c, tel, ev, runs = oracle.simulate_predicted([4, 1], [4, 6], [4, 2], 10, [0, 1], True, max_runs=8)
    assert list(ev) == [0, 1] and runs[0].tolist() == [1, 0, 2, 1]


def test_rejects_malformed_input():
    with pytest.raises(oracle.OracleError):
        oracle.simulate_predicted([1], [1], [0], 10, [0])  # estimate < 1
    with pytest.raises(oracle.OracleError):
        oracle.simulate_predicted([5], [2], [6], 10, [0])  # s + estimate > M
    with pytest.raises(oracle.OracleError):
        oracle.simulate_predicted([1, 1], [1, 1], [1, 1], 10, [0, 0])  # not a permutation
