"""Pins of the exact Phase-1 oracle (Algorithm 2's dynamic programme used batch after batch)."""
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


def _first_batch(s, o, order, ends):
    X = [int(i) for i in order[: int(ends[0])]]
    return X, Fraction(sum(int(o[i]) for i in X), len(X) ** 2)


@pytest.mark.parametrize("feas_mode", [0, 1])
def test_first_batch_is_the_subset_optimum(feas_mode):
    # brute force over all subsets, feasibility written from the definition
    rng = np.random.default_rng(31 + feas_mode)
    cases = [workloads.instance(1)]
    for trial in range(40):
        n = int(rng.integers(1, 11))
        s = rng.integers(1, 9, n).astype(np.int32)
        o = rng.integers(1, 9, n).astype(np.int32)
        cases.append(workloads.Instance("rnd", s, o, int(rng.integers(16, 49))))
    for inst in cases:
        F_bf, ks_bf = exact.brute_best_batch(inst.s, inst.o, inst.M, profile=bool(feas_mode))
        for tie_rule in (0, 1):
            order, ends, F = oracle.exact_phase1(inst.s, inst.o, inst.M, feas_mode, tie_rule)
            X, F_X = _first_batch(inst.s, inst.o, order, ends)
            assert F_X == F_bf and F[0] == float(F_bf)
            assert len(X) == (max(ks_bf) if tie_rule == 0 else min(ks_bf))
            if feas_mode == 0:
                assert sum(int(inst.s[i]) + int(inst.o[i]) for i in X) <= inst.M
            else:
                assert exact.batch_profile_peak(inst.s, inst.o, X) <= inst.M


def test_agrees_with_the_dictionary_dp():
    # oracle/exact.py holds a separately written form of Algorithm 2 (sparse states)
    rng = np.random.default_rng(37)
    for trial in range(30):
        n = int(rng.integers(2, 14))
        s = rng.integers(1, 12, n).astype(np.int32)
        o = rng.integers(1, 12, n).astype(np.int32)
        M = int(rng.integers(24, 80))
        F_dp, ks, _ = exact.dp_best_batch(s, o, M)
        order, ends, F = oracle.exact_phase1(s, o, M, 0, 0)
        X, F_X = _first_batch(s, o, order, ends)
        assert F_X == F_dp and len(X) == max(ks)


def test_every_batch_is_optimal_for_what_remains_and_order_is_valid():
    rng = np.random.default_rng(41)
    for trial in range(25):
        n = int(rng.integers(3, 11))
        s = rng.integers(1, 9, n).astype(np.int32)
        o = rng.integers(1, 9, n).astype(np.int32)
        M = int(rng.integers(16, 40))
        for feas_mode in (0, 1):
            order, ends, F = oracle.exact_phase1(s, o, M, feas_mode, 0)
            assert sorted(order.tolist()) == list(range(n))
            remaining = list(range(n))
            start = 0
            for b, end in enumerate(ends):
                X = [int(i) for i in order[start:end]]
                sub_s, sub_o = s[remaining], o[remaining]
                F_bf, ks_bf = exact.brute_best_batch(sub_s, sub_o, M, profile=bool(feas_mode))
                assert Fraction(int(o[X].sum()), len(X) ** 2) == F_bf and len(X) == max(ks_bf)
                keys = [(int(o[i]), i) for i in X]
                assert keys == sorted(keys)  # nondecreasing o, ties by id
                remaining = [i for i in remaining if i not in X]
                start = end
            assert not remaining


def test_example1_of_the_paper(golden_dir):
    # Example 1 (Section 4): the exact batches are the 21 short requests (F = 42/441), then the long one.
    g = read_golden(os.path.join(golden_dir, "example1.txt"))
    s1, o1, n1 = _ints(g["type1"])
    s2, o2, n2 = _ints(g["type2"])
    s = np.array([s1] * n1 + [s2] * n2, dtype=np.int32)
    o = np.array([o1] * n1 + [o2] * n2, dtype=np.int32)
    M = int(g["M"])
    for feas_mode in (0, 1):
        order, ends, F = oracle.exact_phase1(s, o, M, feas_mode, 0)
        assert list(ends) == [21, 22] and order[21] == 0
        assert F[0] == float(Fraction(g["F_type2"])) and F[1] == float(Fraction(g["F_type1"]))
        assert oracle.simulate(s, o, M, order)[2] == int(g["tel_sortedF"])


def test_lemma1_output_balance():
    # Lemma 1 (Section 4): in an optimal batch the mean output length exceeds half the largest one.
    rng = np.random.default_rng(43)
    for trial in range(40):
        n = int(rng.integers(2, 40))
        s = rng.integers(1, 30, n).astype(np.int32)
        o = rng.integers(1, 30, n).astype(np.int32)
        M = int(rng.integers(60, 400))
        order, ends, _ = oracle.exact_phase1(s, o, M, 0, 0)
        start = 0
        for end in ends:
            oo = o[order[start:end]]
            assert oo.mean() > 0.5 * oo.max()
            start = end


def test_profile_feasibility_admits_at_least_the_sum_of_peaks_batches():
    # sum of peaks <= M implies the profile constraint, so the profile optimum is never worse
    rng = np.random.default_rng(47)
    for trial in range(30):
        n = int(rng.integers(2, 30))
        s = rng.integers(1, 20, n).astype(np.int32)
        o = rng.integers(1, 20, n).astype(np.int32)
        M = int(rng.integers(40, 200))
        Fs = oracle.exact_phase1(s, o, M, 0, 0)[2][0]
        Fp = oracle.exact_phase1(s, o, M, 1, 0)[2][0]
        assert Fp <= Fs


def test_heuristic_batches_never_beat_it():
    rng = np.random.default_rng(53)
    for trial in range(30):
        n = int(rng.integers(2, 60))
        s = rng.integers(1, 30, n).astype(np.int32)
        o = rng.integers(1, 30, n).astype(np.int32)
        M = int(rng.integers(60, 500))
        F_exact = oracle.exact_phase1(s, o, M, 0, 0)[2][0]
        assert F_exact <= oracle.sortedF(s, o, M)[2][0]
        assert F_exact <= oracle.local_swap(s, o, M)[2][0]
