"""The synthetic workload recipe (no GPU): sizes, ranges, determinism, candidate structure."""
import numpy as np

from paper_2508_06133_amd import workloads


def test_instances_shapes_and_ranges():
    expect = {1: (8, 48), 2: (200, 16384), 3: (2000, 131072), 4: (10000, 1048576), 5: (100000, 2097152)}
    for cfg, (n, M) in expect.items():
        inst = workloads.instance(cfg)
        assert inst.n == n and inst.M == M
        assert inst.s.dtype == np.int32 and inst.o.dtype == np.int32
        assert inst.s.min() >= 1 and inst.o.min() >= 1
        assert int((inst.s.astype(np.int64) + inst.o).max()) <= M
        again = workloads.instance(cfg)
        assert (again.s == inst.s).all() and (again.o == inst.o).all()
    c2 = workloads.instance(2)
    assert c2.s.min() >= 4 and c2.s.max() <= 2048 and c2.o.max() <= 2048
    c3 = workloads.instance(3)
    frac_long = float((c3.s > 2048).mean())
    assert 0.25 < frac_long < 0.35
    c5 = workloads.instance(5)
    assert set(np.unique(c5.s)) == {1, 4096} and set(np.unique(c5.o)) == {1, 4096}


def test_candidates_are_permutations():
    base = np.random.default_rng(0).permutation(50).astype(np.int32)
    for cfg, count in [(2, 64), (3, 128), (5, 8)]:
        rows = workloads.candidates(cfg, base, count=count)
        assert rows.shape == (count, 50) and rows.dtype == np.int32
        assert (rows[0] == base).all()
        assert (np.sort(rows, axis=1) == np.arange(50)).all()
    rows = workloads.candidates(2, base, count=64)
    assert ((rows[1:] != base).sum(axis=1) == 2).all()  # exactly one pair exchanged
    rows3 = workloads.candidates(3, base, count=128)
    diff = (rows3[1:126] != base).sum(axis=1)
    assert (diff == 2).all()
    assert len({tuple(np.nonzero(r != base)[0]) for r in rows3[1:126]}) == 125  # distinct pairs


def test_window_moves():
    rng = np.random.default_rng(1)
    mv = workloads.window_moves(rng, 100, 10, 42)
    assert tuple(mv[0]) == (0, 10, 10)
    assert ((mv[:, 1:] >= 10) & (mv[:, 1:] < 42)).all()
    assert set(np.unique(mv[:, 0])) == {0, 1}
    base = np.arange(64, dtype=np.int32)
    rows = workloads.orders_from_moves(base, mv)
    assert (np.sort(rows, axis=1) == base).all()
    assert (rows[:, :10] == base[:10]).all() and (rows[:, 42:] == base[42:]).all()
