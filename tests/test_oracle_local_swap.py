"""Pins of the Local Swap Search oracle (Phase 1 with the appendix's swap-based batch solver)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import exact
from paper_2508_06133_amd import workloads
from conftest import read_golden


def _ints(txt):
    return [int(x) for x in txt.split()]


def _random_instance(rng, n, M, smax, omax):
    s = rng.integers(1, smax + 1, n).astype(np.int32)
    o = rng.integers(1, omax + 1, n).astype(np.int32)
    return s, o, M


@pytest.mark.parametrize("early_exit", [False, True])
def test_hand_worked_example(golden_dir, early_exit):
    g = read_golden(os.path.join(golden_dir, "local_swap_worked.txt"))
    s, o, M = _ints(g["s"]), _ints(g["o"]), int(g["M"])
    order, ends, F, swaps = oracle.local_swap(s, o, M, early_exit)
    assert list(order) == _ints(g["order"])
    assert list(ends) == _ints(g["batch_end"])
    assert list(swaps) == _ints(g["swaps"])
    assert list(F) == [float(Fraction(x)) for x in g["F"].split()]


def test_example1_of_the_paper(golden_dir):
    # Example 1 (Section 4): the 21 short requests fill the budget, no exchange fits the long
    # one in, so the order is the paper's Sorted-F order with total latency 45.
    g = read_golden(os.path.join(golden_dir, "example1.txt"))
    s1, o1, n1 = _ints(g["type1"])
    s2, o2, n2 = _ints(g["type2"])
    s = np.array([s1] * n1 + [s2] * n2, dtype=np.int32)
    o = np.array([o1] * n1 + [o2] * n2, dtype=np.int32)
    M = int(g["M"])
    order, ends, F, swaps = oracle.local_swap(s, o, M)
    assert list(ends) == [21, 22] and list(swaps) == [0, 0]
    assert F[0] == float(Fraction(g["F_type2"])) and F[1] == float(Fraction(g["F_type1"]))
    assert oracle.simulate(s, o, M, order)[2] == int(g["tel_sortedF"])


def test_literal_scan_equals_early_exit_scan():
    rng = np.random.default_rng(7)
    for trial in range(200):
        n = int(rng.integers(1, 60))
        smax, omax = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        M = int(rng.integers(smax + omax, 6 * (smax + omax)))
        s, o, M = _random_instance(rng, n, M, smax, omax)
        a = oracle.local_swap(s, o, M, False)
        b = oracle.local_swap(s, o, M, True)
        for x, y in zip(a, b):
            assert (x == y).all(), trial
    for cfg in (2, 3):
        inst = workloads.instance(cfg)
        a = oracle.local_swap(inst.s, inst.o, inst.M, False)
        b = oracle.local_swap(inst.s, inst.o, inst.M, True)
        for x, y in zip(a, b):
            assert (x == y).all()


def _first_improving_trajectory(s, o, M):
    """Pure-Python restatement on sets: at every step list ALL admissible improving pairs and take
    the least in (sorted place of r_out, sorted place of r_in)."""
    n = len(s)
    w = [int(s[i]) + int(o[i]) for i in range(n)]
    remaining = sorted(range(n), key=lambda i: (w[i], int(o[i]), i))
    order, ends, swaps_all = [], [], []
    while remaining:
        X, mem = [], 0
        for r in remaining:
            if mem + w[r] <= M:
                X.append(r)
                mem += w[r]
        swaps = 0
        while True:
            place = {r: k for k, r in enumerate(remaining)}
            pairs = [(place[a], place[b], a, b) for a in X for b in remaining
                     if b not in X and mem + w[b] - w[a] <= M and o[b] < o[a]]
            if not pairs:
                break
            _, _, a, b = min(pairs)
            X.remove(a)
            X.append(b)
            mem += w[b] - w[a]
            swaps += 1
        order += sorted(X, key=lambda i: (int(o[i]), i))
        ends.append(len(order))
        swaps_all.append(swaps)
        remaining = [r for r in remaining if r not in X]
    return order, ends, swaps_all


def test_against_exhaustive_pair_enumeration():
    rng = np.random.default_rng(11)
    for trial in range(150):
        n = int(rng.integers(1, 14))
        s, o, M = _random_instance(rng, n, int(rng.integers(16, 60)), 8, 8)
        order, ends, F, swaps = oracle.local_swap(s, o, M)
        e_order, e_ends, e_swaps = _first_improving_trajectory(s, o, M)
        assert list(order) == e_order and list(ends) == e_ends and list(swaps) == e_swaps, trial


def _batch_properties(s, o, M, order, ends, F, swaps):
    """What must hold for ANY correct run, checked from the definition with numpy."""
    n = len(s)
    w = s.astype(np.int64) + o
    assert sorted(order.tolist()) == list(range(n))
    start = 0
    remaining = np.ones(n, dtype=bool)
    for b, end in enumerate(ends):
        X = order[start:end]
        rem_ids = np.flatnonzero(remaining)
        # size = what the greedy fill in ascending s+o takes (an exchange keeps the size)
        ws = np.sort(w[rem_ids])
        K = int(np.searchsorted(np.cumsum(ws), M, side="right"))
        assert len(X) == K and K >= 1
        mem = int(w[X].sum())
        assert mem <= M
        S = int(o[X].astype(np.int64).sum())
        assert F[b] == S / (K * K)
        # emitted in nondecreasing o, ties by id
        keys = list(zip(o[X].tolist(), X.tolist()))
        assert keys == sorted(keys)
        # local optimum: no admissible exchange lowers the sum of o
        out_ids = rem_ids[~np.isin(rem_ids, X)]
        if len(out_ids):
            dm = w[out_ids][None, :] - w[X][:, None]
            do = o[out_ids].astype(np.int64)[None, :] - o[X].astype(np.int64)[:, None]
            assert not ((mem + dm <= M) & (do < 0)).any()
        # every exchange lowers the sum of o by at least one from the greedy fill's
        order_w = rem_ids[np.lexsort((rem_ids, o[rem_ids], w[rem_ids]))]
        assert S <= int(o[order_w[:K]].astype(np.int64).sum()) - int(swaps[b])
        remaining[X] = False
        start = end
    assert start == n


def test_properties_random_and_configs():
    rng = np.random.default_rng(13)
    for trial in range(100):
        n = int(rng.integers(1, 120))
        s, o, M = _random_instance(rng, n, int(rng.integers(100, 2000)), 50, 50)
        _batch_properties(s, o, M, *oracle.local_swap(s, o, M, True))
    for cfg in (1, 2, 3):
        inst = workloads.instance(cfg)
        _batch_properties(inst.s, inst.o, inst.M, *oracle.local_swap(inst.s, inst.o, inst.M, True))


def test_never_beats_the_exact_batch():
    # Algorithm 2's DP gives the least F over all feasible subsets; a heuristic batch cannot be lower.
    rng = np.random.default_rng(17)
    for trial in range(60):
        n = int(rng.integers(2, 12))
        s, o, M = _random_instance(rng, n, int(rng.integers(16, 50)), 8, 8)
        order, ends, F, _ = oracle.local_swap(s, o, M)
        K = int(ends[0])
        F_batch = Fraction(int(o[order[:K]].sum()), K * K)
        assert exact.dp_best_batch(s, o, M)[0] <= F_batch
