"""GPU parity of kvsched_exact_dp (Phase 1 with Algorithm 2's exact batches) with the CPU oracle."""
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


def _gpu(ctx, s, o, M, feas_mode, tie_rule):
    import torch

    order, ends, F, nb = ctx.exact_dp(_to_dev(s), _to_dev(o), M, feas_mode, tie_rule)
    torch.cuda.synchronize()
    k = int(nb.item())
    return order.cpu().numpy(), ends.cpu().numpy()[:k], F.cpu().numpy()[:k]


def _check(ctx, s, o, M, what, modes=(0, 1), ties=(0, 1)):
    for feas_mode in modes:
        for tie_rule in ties:
            print(f"exact_dp {what}: n={len(s)} M={M} feas={feas_mode} tie={tie_rule}", flush=True)
            order_o, ends_o, F_o = oracle.exact_phase1(s, o, M, feas_mode, tie_rule)
            order_g, ends_g, F_g = _gpu(ctx, s, o, M, feas_mode, tie_rule)
            assert len(ends_g) == len(ends_o) and (ends_g == ends_o).all(), what
            assert (order_g == order_o).all(), what
            assert np.allclose(F_g, F_o, rtol=1e-12, atol=0.0), what  # one IEEE division of exact integers
            assert ctx.device_status() == 0


def test_config1(ctx):
    inst = workloads.instance(1)
    _check(ctx, inst.s, inst.o, inst.M, "config 1")


def test_example1(ctx, golden_dir):
    g = read_golden(os.path.join(golden_dir, "example1.txt"))
    ints = lambda k: [int(x) for x in g[k].split()]
    s1, o1, n1 = ints("type1")
    s2, o2, n2 = ints("type2")
    s = np.array([s1] * n1 + [s2] * n2, dtype=np.int32)
    o = np.array([o1] * n1 + [o2] * n2, dtype=np.int32)
    for feas_mode in (0, 1):
        order, ends, F = _gpu(ctx, s, o, int(g["M"]), feas_mode, 0)
        assert list(ends) == [21, 22] and order[21] == 0


@pytest.mark.parametrize("n,smax,omax,M", [(1, 3, 3, 6), (2, 1, 3, 100), (13, 8, 8, 30), (64, 20, 6, 90),
                                           (100, 50, 50, 100), (100, 50, 50, 2000), (257, 30, 30, 1000),
                                           (64, 200, 300, 5000), (65, 3, 2, 255), (65, 3, 2, 256), (40, 5, 9, 1023)])
def test_random(ctx, n, smax, omax, M):
    rng = np.random.default_rng(n * 13 + omax)
    s = rng.integers(1, smax + 1, n).astype(np.int32)
    o = rng.integers(1, omax + 1, n).astype(np.int32)
    _check(ctx, s, o, M, f"random n={n}")


def test_many_tiny_instances(ctx):
    rng = np.random.default_rng(9)
    for trial in range(25):
        n = int(rng.integers(1, 30))
        smax, omax = int(rng.integers(1, 12)), int(rng.integers(1, 12))
        M = int(rng.integers(smax + omax, 8 * (smax + omax)))
        s = rng.integers(1, smax + 1, n).astype(np.int32)
        o = rng.integers(1, omax + 1, n).astype(np.int32)
        _check(ctx, s, o, M, f"tiny {trial}", ties=(trial % 2,))


def test_config2_chat_lengths(ctx):
    # config 2's length distributions at 100 requests (the size Algorithm 2 is meant for)
    inst = workloads.instance(2, n=100)
    _check(ctx, inst.s, inst.o, inst.M, "config 2, n=100", ties=(0,))


def test_config2_full_size(ctx):
    inst = workloads.instance(2)
    _check(ctx, inst.s, inst.o, inst.M, "config 2", ties=(0,))


def test_bad_lengths_and_limits(ctx):
    import torch
    from paper_2508_06133_amd import kvsched

    s = np.array([3, 4, 90, 2], dtype=np.int32)
    o = np.array([3, 4, 20, 2], dtype=np.int32)
    order, ends, F, nb = ctx.exact_dp(_to_dev(s), _to_dev(o), 100)
    torch.cuda.synchronize()
    assert int(nb.item()) == 0
    assert ctx.device_status() & kvsched.DEV_BAD_LENGTH
    big = np.ones(kvsched.EXACT_MAX_N + 1, dtype=np.int32)
    with pytest.raises(kvsched.KvschedError):
        ctx.exact_dp(_to_dev(big), _to_dev(big), 100)
    with pytest.raises(kvsched.KvschedError):
        ctx.exact_dp(_to_dev(s[:2]), _to_dev(o[:2]), 100, feas_mode=2)
