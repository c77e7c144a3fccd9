"""GPU parity of kvsched_local_swap (Phase 1 with Local Swap Search) with the CPU oracle."""
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


def _gpu(ctx, s, o, M):
    import torch

    order, ends, F, swaps, nb = ctx.local_swap(_to_dev(s), _to_dev(o), M)
    torch.cuda.synchronize()
    k = int(nb.item())
    return order.cpu().numpy(), ends.cpu().numpy()[:k], F.cpu().numpy()[:k], swaps.cpu().numpy()[:k]


def _check(ctx, s, o, M, what, literal=False):
    print(f"local_swap {what}: n={len(s)} M={M}", flush=True)
    order_o, ends_o, F_o, swaps_o = oracle.local_swap(s, o, M, early_exit=not literal)
    order_g, ends_g, F_g, swaps_g = _gpu(ctx, s, o, M)
    assert len(ends_g) == len(ends_o) and (ends_g == ends_o).all(), what
    assert (swaps_g == swaps_o).all(), what
    assert (order_g == order_o).all(), what
    assert np.allclose(F_g, F_o, rtol=1e-12, atol=0.0), what  # one IEEE division of exact integers
    assert ctx.device_status() == 0
    return int(swaps_o.sum())


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_local_swap_configs(ctx, cfg):
    inst = workloads.instance(cfg)
    _check(ctx, inst.s, inst.o, inst.M, f"config {cfg}", literal=cfg <= 3)


def test_hand_worked_example(ctx, golden_dir):
    g = read_golden(os.path.join(golden_dir, "local_swap_worked.txt"))
    ints = lambda k: [int(x) for x in g[k].split()]
    order, ends, F, swaps = _gpu(ctx, np.array(ints("s")), np.array(ints("o")), int(g["M"]))
    assert list(order) == ints("order") and list(ends) == ints("batch_end") and list(swaps) == ints("swaps")


@pytest.mark.parametrize("n,smax,omax,M", [(1, 3, 3, 6), (2, 1, 3, 100), (64, 20, 6, 90), (65, 20, 60, 2000),
                                           (1023, 50, 40, 3000), (1024, 50, 300, 5000), (1025, 3, 2, 40),
                                           (3000, 2, 2, 64), (3000, 4000, 4000, 90000), (2500, 1, 1, 1 << 20),
                                           (9000, 300, 300, 200000), (8193, 40, 40, 4000), (20000, 30, 30, 300000)])
def test_local_swap_random_and_tie_heavy(ctx, n, smax, omax, M):
    rng = np.random.default_rng(n * 11 + omax)
    s = rng.integers(1, smax + 1, n).astype(np.int32)
    o = rng.integers(1, omax + 1, n).astype(np.int32)
    swaps = _check(ctx, s, o, M, f"random n={n}")
    print(f"  exchanges: {swaps}", flush=True)


def test_many_small_instances(ctx):
    rng = np.random.default_rng(5)
    total = 0
    for trial in range(60):
        n = int(rng.integers(1, 300))
        smax, omax = int(rng.integers(1, 60)), int(rng.integers(1, 60))
        M = int(rng.integers(smax + omax, 12 * (smax + omax)))
        s = rng.integers(1, smax + 1, n).astype(np.int32)
        o = rng.integers(1, omax + 1, n).astype(np.int32)
        total += _check(ctx, s, o, M, f"small {trial}", literal=True)
    assert total > 0  # the instances must actually exercise exchanges


def test_bad_lengths_reported(ctx):
    from paper_2508_06133_amd import kvsched

    s = np.array([3, 4, 90, 2], dtype=np.int32)
    o = np.array([3, 4, 20, 2], dtype=np.int32)
    order, ends, F, swaps, nb = ctx.local_swap(_to_dev(s), _to_dev(o), 100)
    import torch

    torch.cuda.synchronize()
    assert int(nb.item()) == 0
    assert ctx.device_status() & kvsched.DEV_BAD_LENGTH


def test_order_feeds_simulate(ctx):
    # the order is a permutation the timeline kernels accept; its total latency equals the oracle's
    import torch

    inst = workloads.instance(3)
    s, o = _to_dev(inst.s), _to_dev(inst.o)
    order, ends, F, swaps, nb = ctx.local_swap(s, o, inst.M)
    tel, _ = ctx.simulate(order.reshape(1, -1), s, o, inst.M)
    torch.cuda.synchronize()
    order_o = oracle.local_swap(inst.s, inst.o, inst.M, True)[0]
    assert int(tel[0].item()) == oracle.simulate(inst.s, inst.o, inst.M, order_o, literal=False)[2]
