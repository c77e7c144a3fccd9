"""GPU parity of kvsched_phase1_G (Phase 1 under G = sum (alpha s + o) / |X|^2) with the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2508_06133_amd import workloads

pytestmark = pytest.mark.gpu

PREFIX, SWAP, EXACT = 0, 1, 2
ALPHAS = [(0, 1), (0, 7), (13, 1000), (1, 1), (5, 1), (1, 3)]


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


def _gpu(ctx, solver, s, o, M, alpha, tie_rule=0, feas_mode=0):
    import torch

    order, ends, G, swaps, nb = ctx.phase1_G(solver, _to_dev(s), _to_dev(o), M, alpha, tie_rule, feas_mode)
    torch.cuda.synchronize()
    k = int(nb.item())
    return order.cpu().numpy(), ends.cpu().numpy()[:k], G.cpu().numpy()[:k], swaps.cpu().numpy()[:k]


def _oracle(solver, s, o, M, alpha, tie_rule=0, feas_mode=0):
    if solver == PREFIX:
        order, ends, G = oracle.sortedF(s, o, M, tie_rule, feas_mode, alpha=alpha)
        return order, ends, G, None
    if solver == SWAP:
        return oracle.local_swap(s, o, M, True, alpha=alpha)
    order, ends, G = oracle.exact_phase1(s, o, M, feas_mode, tie_rule, alpha=alpha)
    return order, ends, G, None


def _check(ctx, solver, s, o, M, alpha, tie_rule=0, feas_mode=0, what=""):
    print(f"phase1_G solver {solver} alpha {alpha} tie {tie_rule} feas {feas_mode} n={len(s)} M={M} {what}", flush=True)
    order_o, ends_o, G_o, swaps_o = _oracle(solver, s, o, M, alpha, tie_rule, feas_mode)
    order_g, ends_g, G_g, swaps_g = _gpu(ctx, solver, s, o, M, alpha, tie_rule, feas_mode)
    assert len(ends_g) == len(ends_o) and (ends_g == ends_o).all(), what
    assert (order_g == order_o).all(), what
    assert np.allclose(G_g, G_o, rtol=1e-12, atol=0.0), what
    if swaps_o is not None:
        assert (swaps_g == swaps_o).all(), what
    assert ctx.device_status() == 0


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
@pytest.mark.parametrize("solver", [PREFIX, SWAP])
def test_configs_prefix_and_swap(ctx, cfg, solver):
    inst = workloads.instance(cfg)
    for alpha in ALPHAS:
        _check(ctx, solver, inst.s, inst.o, inst.M, alpha, what=f"config {cfg}")
    if solver == PREFIX:
        _check(ctx, solver, inst.s, inst.o, inst.M, (13, 1000), tie_rule=1, feas_mode=1, what=f"config {cfg} profile")


def test_config5_bimodal(ctx):
    inst = workloads.instance(5, n=30000)
    for alpha in [(13, 1000), (3, 1)]:
        _check(ctx, PREFIX, inst.s, inst.o, inst.M, alpha, what="config 5 scaled")
        _check(ctx, SWAP, inst.s, inst.o, inst.M, alpha, what="config 5 scaled")


@pytest.mark.parametrize("feas_mode", [0, 1])
def test_exact_dp(ctx, feas_mode):
    rng = np.random.default_rng(51)
    for trial in range(12):  # one-workgroup kernel
        n = int(rng.integers(2, 60))
        s = rng.integers(1, 12, n).astype(np.int32)
        o = rng.integers(1, 12, n).astype(np.int32)
        M = int(rng.integers(24, 100))
        _check(ctx, EXACT, s, o, M, ALPHAS[trial % len(ALPHAS)], trial % 2, feas_mode, what=f"small {trial}")
    inst = workloads.instance(2, n=60)  # per-request launches (tables in global memory)
    for alpha in [(13, 1000), (2, 1)]:
        _check(ctx, EXACT, inst.s, inst.o, 6000, alpha, 0, feas_mode, what="config 2 scaled")


def test_alpha_zero_is_the_f_metric_call(ctx):
    import torch

    inst = workloads.instance(3)
    s, o = _to_dev(inst.s), _to_dev(inst.o)
    order_f, ends_f, F_f, nb_f = ctx.sortedF(s, o, inst.M)
    order_g, ends_g, G_g, _, nb_g = ctx.phase1_G(PREFIX, s, o, inst.M, (0, 9))
    torch.cuda.synchronize()
    assert torch.equal(order_f, order_g) and torch.equal(ends_f, ends_g) and torch.equal(nb_f, nb_g)
    k = int(nb_f.item())
    assert torch.allclose(F_f[:k], G_g[:k], rtol=1e-12, atol=0.0)


def test_host_side_errors(ctx):
    from paper_2508_06133_amd import kvsched

    inst = workloads.instance(2)
    s, o = _to_dev(inst.s), _to_dev(inst.o)
    for bad in [dict(alpha=(-1, 1)), dict(alpha=(1, 0)), dict(solver=7), dict(solver=SWAP, feas_mode=1)]:
        args = dict(solver=PREFIX, alpha=(1, 1), feas_mode=0)
        args.update(bad)
        with pytest.raises(kvsched.KvschedError) as e:
            ctx.phase1_G(args["solver"], s, o, inst.M, args["alpha"], 0, args["feas_mode"])
        assert e.value.code == -1
    for solver, alpha, M in ((PREFIX, (1 << 16, 1), inst.M), (SWAP, (60000, 1), 1 << 16), (EXACT, (60000, 1), 1 << 15)):
        with pytest.raises(kvsched.KvschedError) as e:
            ctx.phase1_G(solver, s, o, M, alpha)  # effective lengths would overflow
        assert e.value.code == -2
