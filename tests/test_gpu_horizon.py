"""GPU parity of the receding-horizon step / driver (configuration 4) with the CPU oracle."""
import numpy as np
import pytest

import oracle
from oracle import horizon as ohorizon
from paper_2508_06133_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import torch
    from paper_2508_06133_amd import kvsched

    assert torch.cuda.is_available()
    c = kvsched.Context(0)
    yield c
    c.close()


def _dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda:0")


@pytest.mark.parametrize("cfg,n,window,every,K", [(4, 400, 32, 16, 256), (2, 150, 20, 7, 100), (5, 600, 64, 50, 64)])
def test_receding_horizon_scaled_full_parity(ctx, cfg, n, window, every, K):
    from paper_2508_06133_amd import horizon

    inst = workloads.instance(cfg, n=n)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    print(f"receding horizon config {cfg}: n={n} window={window} every={every} K={K}", flush=True)
    rng_o = np.random.default_rng(77)
    order_o, comp_o, log_o = ohorizon.receding_horizon(
        inst.s, inst.o, inst.M, base, lambda lo, hi: workloads.window_moves(rng_o, K, lo, hi), window, every)
    order_g, comp_g, log_g = horizon.receding_horizon(ctx, _dev(inst.s), _dev(inst.o), inst.M, _dev(base), window, every, K,
                                                      rng=np.random.default_rng(77), keep_tel=True)
    assert len(log_g) == len(log_o)
    for a, b in zip(log_g, log_o):
        for key in ("lo", "hi", "best", "best_tel", "base_tel", "committed", "completed", "T"):
            assert a[key] == b[key], (key, a[key], b[key])
        assert (a["tel"] == b["tel"]).all()
    assert (order_g.cpu().numpy() == order_o).all() and (comp_g.cpu().numpy() == comp_o).all()
    assert log_g[-1]["committed"] == n
    # every re-plan keeps the committed prefix and never makes the order worse
    tels = [r["best_tel"] for r in log_g]
    assert all(x >= y for x, y in zip(tels, tels[1:]))
    assert ctx.device_status() == 0


def test_horizon_step_literal_tiny(ctx):
    import torch

    inst = workloads.instance(1)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    moves = workloads.window_moves(np.random.default_rng(3), 40, 2, 8)
    order_o, comp_o, tel_o, res_o = ohorizon.horizon_step(inst.s, inst.o, inst.M, base, moves, 0, 3, literal=True)
    order = _dev(base)
    comp = torch.empty(8, dtype=torch.int32, device="cuda:0")
    tel, res = ctx.horizon_step(order, _dev(moves), _dev(inst.s), _dev(inst.o), inst.M, 0, 3, want_tel=True,
                                completion_out=comp)
    torch.cuda.synchronize()
    assert tuple(int(x) for x in res.cpu().numpy()) == res_o
    assert (tel.cpu().numpy() == tel_o).all() and (order.cpu().numpy() == order_o).all()
    assert (comp.cpu().numpy() == comp_o).all()


def test_hand_worked_example_on_gpu(ctx, golden_dir):
    # tests/golden/horizon_worked.txt: eight requests, three re-plans worked by hand (candidates'
    # latencies, chosen move, timeline, T / completed / committed of every step)
    import os
    import torch

    from conftest import read_golden
    from test_oracle_horizon import ints, worked_moves

    g = read_golden(os.path.join(golden_dir, "horizon_worked.txt"))
    s, o, M = _dev(ints(g["s"])), _dev(ints(g["o"])), int(g["M"])
    order = _dev(ints(g["base_order"]))
    comp = torch.empty(order.shape[0], dtype=torch.int32, device="cuda:0")
    completed = 0
    for k in (1, 2, 3):
        lo, hi = ints(g[f"step{k}_lo_hi"])
        tel, res = ctx.horizon_step(order, _dev(worked_moves(lo, hi)), s, o, M, completed, int(g["complete_every"]),
                                    want_tel=True, completion_out=comp)
        torch.cuda.synchronize()
        T, done, committed = ints(g[f"step{k}_T_completed_committed"])
        want = ints(g[f"step{k}_tel"])
        assert tel.cpu().tolist() == want
        assert res.cpu().tolist() == [int(g[f"step{k}_best"]), min(want), want[0], committed, done, T]
        assert order.cpu().tolist() == ints(g[f"step{k}_order"]) and comp.cpu().tolist() == ints(g[f"step{k}_completion"])
        completed = done
    assert ctx.device_status() == 0
