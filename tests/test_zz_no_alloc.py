"""kvsched_best_neighbor_static (the entry point that allocates nothing: its working memory is a fixed
array in the library's device image) against kvsched_best_neighbor, bit for bit, through the C ABI:
two calls in a row, the second on a smaller input, so that what the first left in the array is there
when the second runs; then a pair small enough for the oracle, compared with it as well.
"""
import numpy as np
import pytest

import oracle
from paper_2508_06133_amd import workloads

pytestmark = pytest.mark.gpu


def _to_dev(a, dtype=np.int32):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).to("cuda:0")


def _moves_anywhere(rng, K, n):
    """Identity first, then swaps and inserts over the whole order (so the timelines resume from the
    base order's saved states when there are enough of them)."""
    mv = np.zeros((K, 3), dtype=np.int32)
    mv[1:, 0] = rng.integers(0, 2, K - 1)
    mv[1:, 1] = rng.integers(0, n, K - 1)
    mv[1:, 2] = rng.integers(0, n, K - 1)
    return mv


def _both(ctx, ctx_ref, inst, base, mv, o_max):
    import torch

    s, o = _to_dev(inst.s), _to_dev(inst.o)
    d_base, d_mv = _to_dev(base), _to_dev(mv)
    tel_ref, res_ref = ctx_ref.best_neighbor(d_base, d_mv, s, o, inst.M)
    torch.cuda.synchronize()
    tel = torch.full((mv.shape[0],), -7, dtype=torch.int64, device="cuda:0")
    res = torch.full((3,), -7, dtype=torch.int64, device="cuda:0")
    ctx.best_neighbor_static(d_base, d_mv, s, o, inst.M, o_max, tel, res)
    torch.cuda.synchronize()
    assert ctx.device_status() == 0 and ctx_ref.device_status() == 0
    assert (tel.cpu().numpy() == tel_ref.cpu().numpy()).all()
    assert (res.cpu().numpy() == res_ref.cpu().numpy()).all()
    return tel.cpu().numpy(), res.cpu().numpy()


def test_static_entry_point_matches_best_neighbor_two_calls_in_a_row():
    import torch
    from paper_2508_06133_amd import kvsched

    assert torch.cuda.is_available()
    ctx, ctx_ref = kvsched.Context(0), kvsched.Context(0)
    try:
        # first call: enough moves and positions for the plan that resumes timelines from saved states
        big = workloads.instance(3, n=1400)
        base_big, _, _ = oracle.sortedF(big.s, big.o, big.M)
        mv_big = _moves_anywhere(np.random.default_rng(11), 6143, big.n)
        print(f"static best_neighbor: n={big.n} K={mv_big.shape[0]} o_max={int(big.o.max())}", flush=True)
        _both(ctx, ctx_ref, big, base_big, mv_big, int(big.o.max()))
        # second call, smaller, on the array as the first call left it; small enough for the oracle
        small = workloads.instance(2, n=150)
        base_small, _, _ = oracle.sortedF(small.s, small.o, small.M)
        mv_small = _moves_anywhere(np.random.default_rng(12), 300, small.n)
        print(f"static best_neighbor: n={small.n} K={mv_small.shape[0]} o_max=2048", flush=True)
        tel, res = _both(ctx, ctx_ref, small, base_small, mv_small, 2048)
        tel_o, res_o = oracle.best_neighbor(small.s, small.o, small.M, base_small, mv_small, literal=False)
        assert (tel == tel_o).all() and tuple(int(x) for x in res) == res_o
        # third: the larger one again after the small one
        print("static best_neighbor: first case again", flush=True)
        _both(ctx, ctx_ref, big, base_big, mv_big, 4096)
    finally:
        ctx.close()
        ctx_ref.close()


def test_static_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2508_06133_amd import kvsched

    ctx = kvsched.Context(0)
    try:
        n, K = 70000, 400000  # 20 (K + 1) + 17408 * 1093 bytes: far beyond the array
        z = torch.zeros(n, dtype=torch.int32, device="cuda:0")
        mv = torch.zeros((K, 3), dtype=torch.int32, device="cuda:0")
        res = torch.zeros(3, dtype=torch.int64, device="cuda:0")
        with pytest.raises(kvsched.KvschedError) as e:
            ctx.best_neighbor_static(z, mv, z, z, 1 << 20, 64, None, res)
        assert e.value.code == -2
        with pytest.raises(kvsched.KvschedError) as e:  # no bound on the decode lengths
            ctx.best_neighbor_static(z[:100], mv[:10], z[:100], z[:100], 1 << 20, 0, None, res)
        assert e.value.code == -1
    finally:
        ctx.close()
