"""GPU parity of kvsched_sortedF and kvsched_best_neighbor with the CPU oracle."""
import numpy as np
import pytest

import oracle
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


def _to_dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda:0")


def _gpu_sortedF(ctx, s, o, M, tie, feas_mode=0):
    import torch

    order, ends, F, nb = ctx.sortedF(_to_dev(s), _to_dev(o), M, tie, feas_mode)
    torch.cuda.synchronize()
    k = int(nb.item())
    return order.cpu().numpy(), ends.cpu().numpy()[:k], F.cpu().numpy()[:k]


def _check_sortedF(ctx, s, o, M, what, feas_mode=0):
    for tie in (0, 1):
        print(f"sortedF {what}: n={len(s)} M={M} tie={tie} feas={feas_mode}", flush=True)
        order_o, ends_o, F_o = oracle.sortedF(s, o, M, tie, feas_mode)
        order_g, ends_g, F_g = _gpu_sortedF(ctx, s, o, M, tie, feas_mode)
        assert len(ends_g) == len(ends_o) and (ends_g == ends_o).all(), what
        assert (order_g == order_o).all(), what
        assert np.allclose(F_g, F_o, rtol=1e-12, atol=0.0), what  # one IEEE division of exact integers
        assert ctx.device_status() == 0


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_sortedF_configs(ctx, cfg):
    inst = workloads.instance(cfg)
    _check_sortedF(ctx, inst.s, inst.o, inst.M, f"config {cfg}")


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_sortedF_profile_feasibility_configs(ctx, cfg):
    inst = workloads.instance(cfg)
    _check_sortedF(ctx, inst.s, inst.o, inst.M, f"config {cfg}", feas_mode=1)


def test_sortedF_profile_feasibility_config5_scaled(ctx):
    inst = workloads.instance(5, n=6000, M=131072)
    _check_sortedF(ctx, inst.s, inst.o, inst.M, "config 5 scaled", feas_mode=1)


@pytest.mark.parametrize("n,smax,omax,M", [(1, 3, 3, 6), (2, 1, 3, 100), (64, 20, 6, 90), (65, 20, 60, 2000),
                                           (1023, 50, 40, 3000), (1025, 3, 2, 40), (3000, 400, 400, 9000),
                                           (2500, 1, 1, 1 << 20), (5000, 2, 200, 640)])
def test_sortedF_profile_feasibility_random(ctx, n, smax, omax, M):
    rng = np.random.default_rng(n * 5 + omax)
    s = rng.integers(1, smax + 1, n).astype(np.int32)
    o = rng.integers(1, omax + 1, n).astype(np.int32)
    _check_sortedF(ctx, s, o, M, f"random n={n}", feas_mode=1)


@pytest.mark.parametrize("n,smax,omax,M", [(1, 3, 3, 6), (2, 1, 3, 100), (64, 20, 6, 90), (65, 20, 6, 2000),
                                           (1023, 50, 4, 300), (1024, 50, 300, 5000), (1025, 3, 2, 40),
                                           (5000, 2, 2, 64), (3000, 4000, 4000, 9000), (2500, 1, 1, 1 << 20)])
def test_sortedF_random_and_tie_heavy(ctx, n, smax, omax, M):
    rng = np.random.default_rng(n * 7 + omax)
    s = rng.integers(1, smax + 1, n).astype(np.int32)
    o = rng.integers(1, omax + 1, n).astype(np.int32)
    M = max(M, int((s.astype(np.int64) + o).max()))
    _check_sortedF(ctx, s, o, M, "random")


def test_sortedF_example1(ctx):
    s = np.array([63] + [1] * 21, dtype=np.int32)
    o = np.array([1] + [2] * 21, dtype=np.int32)
    order, ends, F = _gpu_sortedF(ctx, s, o, 64, 0)
    assert list(ends) == [21, 22] and order[21] == 0
    assert F[0] == 42 / 441 and F[1] == 1.0


def test_sortedF_bad_lengths(ctx):
    from paper_2508_06133_amd import kvsched

    s = np.array([3, 9], dtype=np.int32)
    o = np.array([2, 4], dtype=np.int32)
    order, ends, F = _gpu_sortedF(ctx, s, o, 12, 0)
    assert len(ends) == 0 and ctx.device_status() & kvsched.DEV_BAD_LENGTH


def _gpu_best(ctx, s, o, M, base, moves):
    import torch

    tel, res = ctx.best_neighbor(_to_dev(base), _to_dev(moves), _to_dev(s), _to_dev(o), M)
    torch.cuda.synchronize()
    return tel.cpu().numpy(), tuple(int(x) for x in res.cpu().numpy())


def test_best_neighbor_config1_every_move(ctx):
    inst = workloads.instance(1)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    moves = np.array([(k, i, j) for k in (0, 1) for i in range(8) for j in range(8)], dtype=np.int32)
    tel_o, res_o = oracle.best_neighbor(inst.s, inst.o, inst.M, base, moves, literal=True)
    tel_g, res_g = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
    assert (tel_g == tel_o).all() and res_g == res_o


@pytest.mark.parametrize("cfg,n,K", [(2, 200, 1500), (3, 450, 700), (5, 1000, 40)])
def test_best_neighbor_windows(ctx, cfg, n, K):
    inst = workloads.instance(cfg, n=n)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    rng = np.random.default_rng(cfg)
    lo = n // 5
    moves = workloads.window_moves(rng, K, lo, min(n, lo + 512))
    moves[-1] = (1, 0, n - 1)  # the longest shifts
    moves[-2] = (1, n - 1, 0)
    moves[-3] = (0, 0, n - 1)
    print(f"best_neighbor config {cfg}: n={n} K={K}", flush=True)
    tel_o, res_o = oracle.best_neighbor(inst.s, inst.o, inst.M, base, moves, literal=False)
    tel_g, res_g = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
    assert (tel_g == tel_o).all() and res_g == res_o
    assert ctx.device_status() == 0


def test_best_neighbor_ties_take_lowest_index(ctx):
    # identical requests: every move gives the same TEL, so move 0 must win
    s = np.full(10, 3, dtype=np.int32)
    o = np.full(10, 2, dtype=np.int32)
    moves = workloads.window_moves(np.random.default_rng(0), 50, 0, 10)[1:]
    tel_o, res_o = oracle.best_neighbor(s, o, 12, np.arange(10), moves, literal=True)
    tel_g, res_g = _gpu_best(ctx, s, o, 12, np.arange(10, dtype=np.int32), moves)
    assert res_o[0] == 0 and res_g == res_o and (tel_g == tel_o).all()


def test_best_neighbor_bad_moves(ctx):
    from paper_2508_06133_amd import kvsched

    inst = workloads.instance(2, n=40)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    moves = np.array([(0, 1, 2), (2, 1, 2), (0, -1, 3), (1, 5, 40), (1, 5, 39)], dtype=np.int32)
    tel_g, res_g = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
    assert ctx.device_status() == kvsched.DEV_BAD_MOVE
    assert list(tel_g[1:4]) == [-1, -1, -1]
    good = moves[[0, 4]]
    tel_o, res_o = oracle.best_neighbor(inst.s, inst.o, inst.M, base, good, literal=False)
    assert tel_g[0] == tel_o[0] and tel_g[4] == tel_o[1]
    assert res_g[0] == (0, 4)[res_o[0]] and res_g[1] == res_o[1] and res_g[2] == res_o[2]


@pytest.mark.parametrize("cfg,n,lo,width,K", [(3, 700, 300, 200, 500), (2, 200, 64, 100, 300), (4, 1500, 1333, 167, 256),
                                              (5, 2000, 1500, 400, 64)])
def test_best_neighbor_shared_prefix(ctx, cfg, n, lo, width, K):
    # every move lies at or beyond position lo >= 64: the library places the common prefix once and
    # resumes all neighbours from its state; results must not change
    inst = workloads.instance(cfg, n=n)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    moves = workloads.window_moves(np.random.default_rng(cfg + 10), K, lo, min(n, lo + width))
    print(f"best_neighbor shared prefix config {cfg}: n={n} window [{lo},{lo + width}) K={K}", flush=True)
    tel_o, res_o = oracle.best_neighbor(inst.s, inst.o, inst.M, base, moves, literal=False)
    tel_g, res_g = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
    assert (tel_g == tel_o).all() and res_g == res_o
    assert ctx.device_status() == 0


@pytest.mark.parametrize("cfg,n,K,min_rows", [(3, 2000, 4200, -1), (3, 700, 600, 256), (2, 330, 2300, 2048),
                                              (5, 1100, 500, 128)])
def test_best_neighbor_moves_anywhere_resume_from_the_base_order(ctx, cfg, n, K, min_rows):
    # swaps and insertions all over the order (no prefix common to all): each move's timeline starts
    # from the state the base order's timeline saved before the first position the move touches.
    # min_rows = -1: the library's own choice takes that path at this size; else forced for small cases.
    # Identity moves, moves at position 0 and at the last position, and malformed moves among them;
    # the same under the three hand-over settings and with resuming off
    from paper_2508_06133_amd import kvsched

    inst = workloads.instance(cfg) if n == 2000 else workloads.instance(cfg, n=n)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    moves = workloads.window_moves(np.random.default_rng(cfg + 40), K, 0, n)
    moves[5] = (0, 0, n - 1)
    moves[6] = (1, n - 1, 0)
    moves[7] = (1, 0, n - 1)
    moves[8] = (0, n - 1, n - 2)
    moves[9] = (1, 77, 77)
    print(f"best_neighbor over the whole order: config {cfg} n={n} K={K}", flush=True)
    tel_o, res_o = oracle.best_neighbor(inst.s, inst.o, inst.M, base, moves, literal=False)
    try:
        ctx.set_resume_min_rows(min_rows)
        for polls in (4096, 1, 0):
            ctx.set_resume_one_launch(polls)
            tel_g, res_g = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
            assert (tel_g == tel_o).all() and res_g == res_o, polls
            assert ctx.device_status() == 0
        ctx.set_resume_one_launch(4096)
        bad = moves.copy()
        bad[11] = (2, 1, 2)
        bad[12] = (0, -1, 3)
        bad[13] = (1, 5, n)
        tel_b, res_b = _gpu_best(ctx, inst.s, inst.o, inst.M, base, bad)
        assert ctx.device_status() == kvsched.DEV_BAD_MOVE
        keep = np.ones(K, dtype=bool)
        keep[11:14] = False
        assert list(tel_b[11:14]) == [-1, -1, -1] and (tel_b[keep] == tel_o[keep]).all()
        ctx.set_resume_min_rows(0)
        tel_p, res_p = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
        assert (tel_p == tel_o).all() and res_p == res_o
    finally:
        ctx.set_resume_min_rows(-1)
        ctx.set_resume_one_launch(4096)


@pytest.mark.parametrize("cfg,n", [(3, 1500), (4, 3000), (5, 1300)])
def test_moves_that_only_reorder_requests_started_together_are_not_placed(ctx, cfg, n):
    # A move that only reorders requests which the base order starts in one round changes no completion
    # round, and the library does not place such a move's timeline (at all, or beyond the 64-position
    # boundary behind the move): windows inside the base order's initial fill, across its end and behind
    # it, behind a common prefix (first position >= 64: the base order is placed once more through the
    # window to find its start rounds) and not (the moves' timelines start from the base order's saved
    # states and look at its start rounds as it goes).  Latencies and the best move as the oracle's,
    # which places every timeline in full; a timeline is cut short only where the condition holds.
    inst = workloads.instance(cfg, n=n)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    p0, _, _ = oracle.simulate(inst.s, inst.o, inst.M, base, literal=False)
    start0 = p0[base]
    fill = int((start0 == 0).sum())  # positions of the initial fill
    assert 200 < fill < n - 200, fill
    K = 700
    cut_short = placed_nothing = 0
    try:
        ctx.set_resume_min_rows(256)
        for lo, hi in ((0, 300), (80, fill - 20), (fill - 150, fill + 150), (fill + 100, min(n, fill + 500)), (64, n)):
            moves = workloads.window_moves(np.random.default_rng(cfg * 100 + lo), K, lo, hi)
            print(f"moves among requests started together: config {cfg} n={n} fill={fill} window [{lo},{hi})", flush=True)
            tel_o, res_o = oracle.best_neighbor(inst.s, inst.o, inst.M, base, moves, literal=False)
            tel_g, res_g = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
            assert (tel_g == tel_o).all() and res_g == res_o, (lo, hi)
            assert ctx.device_status() == 0
            import torch

            stop = ctx.neighbor_stop_positions(K, n).cpu().numpy()
            torch.cuda.synchronize()
            i = np.minimum(moves[:, 1], moves[:, 2])
            j = np.maximum(moves[:, 1], moves[:, 2])
            together = start0[j] == np.where(i > 0, start0[np.maximum(i - 1, 0)], 0)
            early = stop < n
            assert (together | (i == j))[early].all(), (lo, hi)
            assert ((stop[early] == 0) | ((stop[early] % 64 == 0) & (stop[early] > j[early]))).all()
            if lo >= 64 and hi <= fill:
                assert early.all(), (lo, hi)  # every move of a window inside the fill (behind a common prefix this does not depend on timing)
            cut_short += int(early.sum())
            placed_nothing += int((stop == 0).sum())
    finally:
        ctx.set_resume_min_rows(-1)
    assert cut_short > K and placed_nothing > K // 2, (cut_short, placed_nothing)


def test_best_neighbor_only_identity_moves(ctx):
    inst = workloads.instance(2, n=130)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    moves = np.array([(0, 5, 5), (1, 70, 70), (0, 129, 129)], dtype=np.int32)
    tel_o, res_o = oracle.best_neighbor(inst.s, inst.o, inst.M, base, moves, literal=False)
    tel_g, res_g = _gpu_best(ctx, inst.s, inst.o, inst.M, base, moves)
    assert (tel_g == tel_o).all() and res_g == res_o and res_g[0] == 0 and res_g[1] == res_g[2]
