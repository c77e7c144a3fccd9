"""Pins of the three Phase-1 oracles under the generalised metric G(X) = sum (alpha s_i + o_i) / |X|^2
(Section 7, "Robustness to prefill weighting"), alpha = a / b."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import exact
from paper_2508_06133_amd import workloads
from conftest import read_golden

ALPHAS = [(0, 1), (13, 1000), (1, 1), (5, 1), (1, 3), (7, 2)]


def _instance(rng, nmax=10):
    n = int(rng.integers(1, nmax + 1))
    smax, omax = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    M = int(rng.integers(smax + omax, 5 * (smax + omax)))
    return rng.integers(1, smax + 1, n).astype(np.int32), rng.integers(1, omax + 1, n).astype(np.int32), M


def _G(s, o, ids, a, b):
    """The metric from its definition, as an exact fraction."""
    return sum(Fraction(a, b) * int(s[i]) + int(o[i]) for i in ids) / len(ids) ** 2


def _feasible(s, o, ids, M, feas_mode):
    if feas_mode == 0:
        return sum(int(s[i]) + int(o[i]) for i in ids) <= M
    return exact.batch_profile_peak(s, o, ids) <= M


def _first_batches(order, ends):
    start = 0
    for e in ends:
        yield [int(x) for x in order[start:e]]
        start = int(e)


def test_alpha_zero_is_the_f_metric_whatever_the_denominator():
    rng = np.random.default_rng(41)
    for trial in range(60):
        s, o, M = _instance(rng, 30)
        for b in (1, 3, 1000):
            for f0, g0 in ((oracle.sortedF(s, o, M), oracle.sortedF(s, o, M, alpha=(0, b))),
                           (oracle.local_swap(s, o, M), oracle.local_swap(s, o, M, alpha=(0, b))),
                           (oracle.exact_phase1(s, o, M), oracle.exact_phase1(s, o, M, alpha=(0, b)))):
                for x, y in zip(f0, g0):
                    assert (x == y).all()


@pytest.mark.parametrize("feas_mode", [0, 1])
@pytest.mark.parametrize("tie_rule", [0, 1])
def test_exact_batches_minimise_g_over_all_feasible_subsets(feas_mode, tie_rule):
    rng = np.random.default_rng(42 + feas_mode)
    for trial in range(40):
        s, o, M = _instance(rng, 9)
        a, b = ALPHAS[trial % len(ALPHAS)]
        order, ends, Gv = oracle.exact_phase1(s, o, M, feas_mode, tie_rule, alpha=(a, b))
        remaining = set(range(len(s)))
        for k, X in enumerate(_first_batches(order, ends)):
            rem = sorted(remaining)
            best, sizes = None, set()
            for mask in range(1, 1 << len(rem)):
                ids = [rem[i] for i in range(len(rem)) if mask >> i & 1]
                if not _feasible(s, o, ids, M, feas_mode):
                    continue
                g = _G(s, o, ids, a, b)
                if best is None or g < best:
                    best, sizes = g, {len(ids)}
                elif g == best:
                    sizes.add(len(ids))
            assert _feasible(s, o, X, M, feas_mode) and _G(s, o, X, a, b) == best, (trial, k)
            assert len(X) == (max(sizes) if tie_rule == 0 else min(sizes))
            assert Gv[k] == float(best) or abs(Gv[k] - float(best)) <= 1e-12 * float(best)
            assert [(int(o[i]), i) for i in X] == sorted((int(o[i]), i) for i in X)  # emitted by true o
            remaining -= set(X)
        assert not remaining


@pytest.mark.parametrize("feas_mode", [0, 1])
def test_sorted_prefix_batches_from_the_definition(feas_mode):
    rng = np.random.default_rng(44)
    for trial in range(80):
        s, o, M = _instance(rng, 25)
        a, b = ALPHAS[trial % len(ALPHAS)]
        tie_rule = trial % 2
        order, ends, Gv = oracle.sortedF(s, o, M, tie_rule, feas_mode, alpha=(a, b))
        remaining = sorted(range(len(s)), key=lambda i: (int(s[i]) + int(o[i]), int(o[i]), i))
        for k, X in enumerate(_first_batches(order, ends)):
            best, bestk = None, 0
            for kk in range(1, len(remaining) + 1):
                ids = remaining[:kk]
                if not _feasible(s, o, ids, M, feas_mode):
                    break
                g = _G(s, o, ids, a, b)
                if best is None or g < best or (g == best and tie_rule == 0):
                    best, bestk = g, kk
            assert sorted(X) == sorted(remaining[:bestk]), (trial, k)
            assert abs(Gv[k] - float(best)) <= 1e-12 * float(best)
            assert [(int(o[i]), i) for i in X] == sorted((int(o[i]), i) for i in X)
            remaining = remaining[bestk:]
        assert not remaining


def test_local_swap_against_exhaustive_pair_enumeration():
    # at every step list ALL admissible pairs that lower sum (a s + b o) and take the least in
    # (sorted place of r_out, sorted place of r_in)
    rng = np.random.default_rng(45)
    for trial in range(120):
        s, o, M = _instance(rng, 13)
        a, b = ALPHAS[trial % len(ALPHAS)]
        n = len(s)
        w = [int(s[i]) + int(o[i]) for i in range(n)]
        g = [a * int(s[i]) + b * int(o[i]) for i in range(n)]
        remaining = sorted(range(n), key=lambda i: (w[i], int(o[i]), i))
        e_order, e_ends, e_swaps = [], [], []
        while remaining:
            X, mem = [], 0
            for r in remaining:
                if mem + w[r] <= M:
                    X.append(r)
                    mem += w[r]
            swaps = 0
            while True:
                place = {r: k for k, r in enumerate(remaining)}
                pairs = [(place[x], place[y], x, y) for x in X for y in remaining
                         if y not in X and mem + w[y] - w[x] <= M and g[y] < g[x]]
                if not pairs:
                    break
                _, _, x, y = min(pairs)
                X.remove(x)
                X.append(y)
                mem += w[y] - w[x]
                swaps += 1
            e_order += sorted(X, key=lambda i: (int(o[i]), i))
            e_ends.append(len(e_order))
            e_swaps.append(swaps)
            remaining = [r for r in remaining if r not in X]
        for early in (False, True):
            order, ends, Gv, swaps = oracle.local_swap(s, o, M, early, alpha=(a, b))
            assert list(order) == e_order and list(ends) == e_ends and list(swaps) == e_swaps, (trial, a, b)
        start = 0
        for k, e in enumerate(e_ends):
            X = e_order[start:e]
            assert abs(Gv[k] - float(_G(s, o, X, a, b))) <= 1e-12 * float(_G(s, o, X, a, b))
            start = e


def test_example1_keeps_its_order_under_any_weight(golden_dir):
    # Example 1 (Section 4): G(21 short requests) = 21 (alpha + 2) / 441 < G(long request) =
    # 63 alpha + 1 for every alpha >= 0, so the F-based order (total latency 45) stands.
    gold = read_golden(os.path.join(golden_dir, "example1.txt"))
    s1, o1, n1 = (int(x) for x in gold["type1"].split())
    s2, o2, n2 = (int(x) for x in gold["type2"].split())
    s = np.array([s1] * n1 + [s2] * n2, dtype=np.int32)
    o = np.array([o1] * n1 + [o2] * n2, dtype=np.int32)
    M = int(gold["M"])
    for a, b in ALPHAS + [(1000, 1)]:
        for order, ends, Gv in (oracle.sortedF(s, o, M, alpha=(a, b)), oracle.local_swap(s, o, M, alpha=(a, b))[:3],
                                oracle.exact_phase1(s, o, M, alpha=(a, b))):
            assert list(ends) == [21, 22]
            assert abs(Gv[0] - float(Fraction(21 * (a + 2 * b), 441 * b))) < 1e-12
            assert abs(Gv[1] - float(Fraction(63 * a + b, b))) < 1e-9
            assert oracle.simulate(s, o, M, order)[2] == int(gold["tel_sortedF"])


def test_heavy_prefill_weight_changes_the_batches():
    # with alpha large the metric is driven by the prompt lengths: on the mixed workload the
    # order differs from Sorted-F's and the batches cannot have a lower F than Sorted-F's own
    inst = workloads.instance(3, n=400)
    f = oracle.local_swap(inst.s, inst.o, inst.M, True)
    g = oracle.local_swap(inst.s, inst.o, inst.M, True, alpha=(5, 1))
    assert (f[0] != g[0]).any()
    assert sorted(g[0].tolist()) == list(range(inst.n))
