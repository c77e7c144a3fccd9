"""GPU parity of kvsched_simulate_predicted (Phase 2 under predicted decode lengths: running
estimates, ordered eviction) with the CPU oracle: completion rounds, totals, eviction counts."""
import os

import numpy as np
import pytest

import oracle
from paper_2508_06133_amd import workloads
from conftest import read_golden

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import torch
    from paper_2508_06133_amd import kvsched

    assert torch.cuda.is_available()
    c = kvsched.Context(0)
    yield c
    c.close()


def _to_dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda:0")


def _gpu(ctx, s, o, est, M, rows):
    import torch

    tel, comp, ev = ctx.simulate_predicted(_to_dev(rows), _to_dev(s), _to_dev(o), _to_dev(est), M)
    torch.cuda.synchronize()
    return tel.cpu().numpy(), comp.cpu().numpy(), ev.cpu().numpy(), ctx.device_status()


def _check(ctx, s, o, est, M, rows, what):
    rows = np.asarray(rows, dtype=np.int32).reshape(-1, len(s))
    est = np.asarray(est, dtype=np.int32)
    print(f"predicted {what}: n={len(s)} C={rows.shape[0]} M={M} est rows {1 if est.ndim == 1 else est.shape[0]}", flush=True)
    tel_g, comp_g, ev_g, status = _gpu(ctx, s, o, est, M, rows)
    assert status == 0, what
    total_ev = 0
    for c in range(rows.shape[0]):
        e = est if est.ndim == 1 else est[c]
        p_o, c_o, tel_o, ev_o, _ = oracle.simulate_predicted(s, o, e, M, rows[c])
        assert tel_g[c] == tel_o and (comp_g[c] == c_o).all() and ev_g[c] == int(ev_o.sum()), (what, c)
        total_ev += int(ev_o.sum())
    return total_ev


def test_hand_worked_example(ctx, golden_dir):
    g = read_golden(os.path.join(golden_dir, "predicted_worked.txt"))
    ints = lambda k: [int(x) for x in g[k].split()]
    s, o, M, order = ints("s"), ints("o"), int(g["M"]), ints("order")
    tel, comp, ev, status = _gpu(ctx, s, o, ints("lower"), M, [order])
    assert list(comp[0]) == ints("amin_completion") and tel[0] == int(g["amin_tel"]) and ev[0] == 1 and status == 0
    tel, comp, ev, status = _gpu(ctx, s, o, ints("upper"), M, [order])
    assert list(comp[0]) == ints("amax_completion") and tel[0] == int(g["amax_tel"]) and ev[0] == 0 and status == 0


def test_random_small_instances_one_prediction_per_row(ctx):
    rng = np.random.default_rng(71)
    evictions = 0
    for trial in range(40):
        n = int(rng.integers(1, 90))
        smax, omax = int(rng.integers(1, 40)), int(rng.integers(1, 150))
        M = int(rng.integers(smax + omax, 6 * (smax + omax)))
        s = rng.integers(1, smax + 1, n).astype(np.int32)
        o = rng.integers(1, omax + 1, n).astype(np.int32)
        C = 24
        rows = np.stack([rng.permutation(n) for _ in range(C)]).astype(np.int32)
        est = np.empty((C, n), dtype=np.int32)
        for c in range(C):
            lower = np.array([int(rng.integers(1, x + 1)) for x in o])
            upper = np.array([int(rng.integers(x, M - sv + 1)) for sv, x in zip(s, o)])
            mode = c % 4
            est[c] = lower if mode == 0 else upper if mode == 1 else o if mode == 2 else np.where(rng.random(n) < 0.5, lower, upper)
        evictions += _check(ctx, s, o, est, M, rows, f"random {trial}")
    assert evictions > 200


@pytest.mark.parametrize("cfg,n,C,gamma", [(2, 200, 96, 0.5), (3, 500, 64, 0.25), (3, 2000, 12, 0.6), (5, 800, 16, 0.3)])
def test_configs_lower_and_upper_bounds(ctx, cfg, n, C, gamma):
    inst = workloads.instance(cfg, n=n)
    lower, upper = workloads.prediction_intervals(cfg, inst.s, inst.o, inst.M, gamma)
    base = oracle.sortedF(inst.s, lower, inst.M)[0]  # Phase 1 on the lower bounds, as the paper prescribes
    rows = workloads.candidates(3 if cfg != 2 else 2, base, count=C)
    ev = _check(ctx, inst.s, inst.o, lower, inst.M, rows, f"config {cfg} lower bounds")
    assert ev > 0
    assert _check(ctx, inst.s, inst.o, upper, inst.M, rows[: max(4, C // 4)], f"config {cfg} upper bounds") == 0


def test_exact_predictions_equal_kvsched_simulate(ctx):
    import torch

    inst = workloads.instance(3, n=700)
    base = oracle.sortedF(inst.s, inst.o, inst.M)[0]
    rows = workloads.candidates(3, base, count=256)
    s, o, r = _to_dev(inst.s), _to_dev(inst.o), _to_dev(rows)
    tel_p, comp_p, ev = ctx.simulate_predicted(r, s, o, o, inst.M)
    tel_s, comp_s = ctx.simulate(r, s, o, inst.M)
    torch.cuda.synchronize()
    assert torch.equal(tel_p, tel_s) and torch.equal(comp_p, comp_s) and int(ev.sum().item()) == 0


def test_faults(ctx):
    import torch
    from paper_2508_06133_amd import kvsched

    s, o, M = [3, 3, 3], [2, 2, 2], 10
    tel, comp, ev, status = _gpu(ctx, s, o, [2, 0, 2], M, [[0, 1, 2]])  # an estimate < 1
    assert tel[0] == -1 and status & kvsched.DEV_BAD_LENGTH
    tel, comp, ev, status = _gpu(ctx, s, o, [2, 8, 2], M, [[0, 1, 2]])  # s + estimate > M
    assert tel[0] == -1 and status & kvsched.DEV_BAD_LENGTH
    tel, comp, ev, status = _gpu(ctx, s, o, [2, 2, 2], M, [[0, 1, 2], [0, 0, 2]])  # second row no permutation
    assert tel[0] == 2 + 2 + 4 and tel[1] == -1 and status & kvsched.DEV_BAD_ORDER
    with pytest.raises(kvsched.KvschedError) as e:  # two prediction rows for three order rows
        ctx.simulate_predicted(_to_dev([[0, 1, 2]] * 3), _to_dev(s), _to_dev(o), _to_dev([[2, 2, 2]] * 2), M)
    assert e.value.code == -1
    with pytest.raises(kvsched.KvschedError) as e:  # per-candidate state beyond the LDS of a workgroup
        n = 12000
        ctx.simulate_predicted(_to_dev(np.arange(n)[None, :]), _to_dev(np.ones(n)), _to_dev(np.ones(n)),
                               _to_dev(np.ones(n)), 100)
    assert e.value.code == -2
