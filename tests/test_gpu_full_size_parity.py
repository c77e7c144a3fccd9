"""Bit-exact parity of the timeline kernels with the CPU oracle at full size and on a fully occupied GPU.

* configuration 5 at its stated size (n = 100000, 1025 rows, the 65-row register file): every row;
* configuration 4 at its stated size (n = 10000, 65536 moves per 512-window): every candidate of the
  first window, and the whole receding-horizon run -- every 64th candidate of every window, every
  chosen move, every commit triple, the final order and timeline;
* every instantiation of the register kernel (9 / 33 / 65 / 129 / 225 profile rows; explicit rows or moves;
  from the start, resumed in one launch, resumed in two) with at least 8192 timelines in flight
  on an instance whose tight budget makes most requests wait, twice each, all rows compared.

The oracle runs its rows on several host threads (tests/oracle_pool.py).
"""
import numpy as np
import pytest

import oracle
import oracle_pool
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


def _dev(a, dtype=np.int32):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).to("cuda:0")


# ------------------------------------------------------------------ configuration 5, every row

C5_PARTS = 8


@pytest.fixture(scope="module")
def config5(ctx):
    """The 1025-row call at n = 100000, launched twice; results of both launches on the host."""
    import torch

    inst = workloads.instance(5)
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    rows = workloads.candidates(5, base)
    print(f"config 5: n={inst.n} C={rows.shape[0]} (two launches)", flush=True)
    s, o, d_rows = _dev(inst.s), _dev(inst.o), _dev(rows)
    out = []
    for _ in range(2):
        tel, comp = ctx.simulate(d_rows, s, o, inst.M)
        torch.cuda.synchronize()
        assert ctx.device_status() == 0
        out.append((tel.cpu().numpy(), comp.cpu().numpy()))
        del tel, comp
    return inst, rows, out


@pytest.mark.parametrize("part", range(C5_PARTS))
def test_config5_full_size_every_row(config5, part):
    inst, rows, out = config5
    pick = np.arange(part, rows.shape[0], C5_PARTS)
    print(f"config 5: rows {part}::{C5_PARTS} ({pick.size} rows) on {oracle_pool.workers()} host threads", flush=True)
    tel_o, comp_o = oracle_pool.simulate_many(inst.s, inst.o, inst.M, rows[pick], chunk=2)
    for launch, (tel_g, comp_g) in enumerate(out):
        bad = np.nonzero(tel_g[pick] != tel_o)[0]
        assert bad.size == 0, f"launch {launch}: total latency differs at rows {pick[bad][:8]}"
        assert (comp_g[pick] == comp_o).all(), f"launch {launch}: completion rounds differ"
    assert tel_o.max() > 2 ** 31  # needs the 64-bit accumulator


# ------------------------------------------- configuration 4, the whole receding-horizon run

def _check_window(inst, order, moves, rec, sample, step):
    """Latencies of the sampled moves of one window against the oracle (in chunks: a row is 40 KB);
    returns the oracle's latencies of the sample."""
    tel = rec["tel"]
    tel_o = np.empty(sample.size, dtype=np.int64)
    for lo in range(0, sample.size, 4096):
        rows = workloads.orders_from_moves(order, moves[sample[lo:lo + 4096]])
        tel_o[lo:lo + 4096], _ = oracle_pool.simulate_many(inst.s, inst.o, inst.M, rows, completions=False)
    bad = np.nonzero(tel[sample] != tel_o)[0]
    assert bad.size == 0, f"window {step}: latency differs at moves {sample[bad][:8]}"
    at_best = int(np.nonzero(sample == rec["best"])[0][0])
    # the chosen move: its latency is the oracle's, nothing compared lies below it and no equal one
    # lies before it
    assert rec["best_tel"] == int(tel_o[at_best]) == int(tel_o.min())
    assert sample[int(np.argmin(tel_o))] == rec["best"]
    assert rec["base_tel"] == int(tel_o[0])  # move 0 is the identity
    return tel_o


def test_config4_full_size_first_window_every_candidate(ctx):
    from paper_2508_06133_amd import horizon

    inst = workloads.instance(4)
    K = 65536
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    print(f"config 4: n={inst.n} M={inst.M}, first window, all {K} moves on {oracle_pool.workers()} host threads",
          flush=True)
    _, _, log = horizon.receding_horizon(ctx, _dev(inst.s), _dev(inst.o), inst.M, _dev(base), 512, 256, K,
                                         rng=np.random.default_rng(4), keep_tel=True, max_steps=1)
    assert ctx.device_status() == 0
    moves = workloads.window_moves(np.random.default_rng(4), K, 0, 512)
    _check_window(inst, base, moves, log[0], np.arange(K), 0)


def test_config4_full_size_whole_run(ctx):
    from paper_2508_06133_amd import horizon

    inst = workloads.instance(4)
    n, window, every, K = inst.n, 512, 256, 65536
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    print(f"config 4: n={n} M={inst.M}, whole run with {K} moves per window", flush=True)
    order_g, comp_g, log = horizon.receding_horizon(ctx, _dev(inst.s), _dev(inst.o), inst.M, _dev(base), window, every, K,
                                                    rng=np.random.default_rng(4), keep_tel=True)
    assert ctx.device_status() == 0
    print(f"config 4: {len(log)} re-plans; oracle on {oracle_pool.workers()} host threads", flush=True)
    rng_o = np.random.default_rng(4)
    order = base
    completed = committed = 0
    c = None
    for step, rec in enumerate(log):
        assert (rec["lo"], rec["hi"]) == (committed, min(n, committed + window))
        moves = workloads.window_moves(rng_o, K, rec["lo"], rec["hi"])
        # every 64th candidate, the chosen one, the first and the last
        sample = np.unique(np.concatenate([np.arange(0, K, 64), [rec["best"], 1, K - 1]]))
        _check_window(inst, order, moves, rec, sample, step)
        assert rec["best"] == int(np.argmin(rec["tel"]))  # and against the other latencies of the call itself
        order = workloads.apply_move(order, moves[rec["best"]])
        p, c, total = oracle.simulate(inst.s, inst.o, inst.M, order, literal=False)
        assert total == rec["best_tel"]
        k = min(n, completed + every)
        T = int(np.sort(c)[k - 1])
        assert (rec["T"], rec["completed"], rec["committed"]) == (T, int((c <= T).sum()), int((p[order] <= T).sum()))
        completed, committed = rec["completed"], rec["committed"]
        if step % 8 == 0:
            print(f"config 4: window {step} ok (committed {committed})", flush=True)
    assert committed == n
    assert (order_g.cpu().numpy() == order).all() and (comp_g.cpu().numpy() == c).all()


# --------------------------- every instantiation of the register kernel on a fully occupied GPU

# (profile rows, n, longest decode, share of long decodes)
OCCUPANCY_CASES = [(9, 320, 512, 0.25), (33, 256, 2048, 0.25), (65, 200, 4096, 0.25), (129, 136, 8192, 0.08),
                   (225, 132, 14336, 0.05)]
OCCUPANCY_ROWS = 8192 + 448  # eight wavefronts on each of the 1024 SIMDs, and a ragged rest


@pytest.fixture(scope="module", params=OCCUPANCY_CASES, ids=lambda c: f"NR{c[0]}")
def occupancy_case(request):
    nr, n, o_max, long_frac = request.param
    inst = workloads.tight_instance(o_max + n, n, o_max, long_frac=long_frac)
    assert (int(inst.o.max()) + 63) // 64 + 1 == nr
    base, _, _ = oracle.sortedF(inst.s, inst.o, inst.M)
    moves = workloads.moves_anywhere(np.random.default_rng(nr), OCCUPANCY_ROWS, n)
    rows = workloads.orders_from_moves(base, moves)
    print(f"occupancy case: {nr} profile rows, n={n} o_max={o_max} M={inst.M}, {OCCUPANCY_ROWS} timelines; "
          f"oracle on {oracle_pool.workers()} host threads", flush=True)
    tel_o, comp_o = oracle_pool.simulate_many(inst.s, inst.o, inst.M, rows)
    p, _, _ = oracle.simulate(inst.s, inst.o, inst.M, base, literal=False)
    assert (np.diff(p[base]) > 0).sum() >= n // 4  # most placements had to move the start round on
    return inst, base, moves, rows, tel_o, comp_o


@pytest.mark.parametrize("mode", ["from_start", "resumed_one_launch", "resumed_two_launches"])
def test_rows_on_a_full_gpu(ctx, occupancy_case, mode):
    import torch

    inst, base, moves, rows, tel_o, comp_o = occupancy_case
    s, o, d_rows = _dev(inst.s), _dev(inst.o), _dev(rows)
    try:
        ctx.set_resume_min_rows(0 if mode == "from_start" else 1)
        ctx.set_resume_one_launch(0 if mode == "resumed_two_launches" else 4096)
        for launch in range(2):
            print(f"rows, {mode}, launch {launch}: n={inst.n} C={rows.shape[0]}", flush=True)
            tel, comp = ctx.simulate(d_rows, s, o, inst.M)
            pos = ctx.simulate_resume_positions(rows.shape[0]).cpu().numpy()
            torch.cuda.synchronize()
            assert ctx.device_status() == 0
            bad = np.nonzero(tel.cpu().numpy() != tel_o)[0]
            assert bad.size == 0, f"{mode}, launch {launch}: total latency differs at rows {bad[:8]}"
            assert (comp.cpu().numpy() == comp_o).all(), f"{mode}, launch {launch}: completion rounds differ"
            assert (pos > 0).any() == (mode != "from_start")  # the path meant is the path taken
    finally:
        ctx.set_resume_min_rows(-1)
        ctx.set_resume_one_launch(4096)


@pytest.mark.parametrize("mode", ["from_start", "resumed_one_launch"])
def test_moves_on_a_full_gpu(ctx, occupancy_case, mode):
    import torch

    inst, base, moves, rows, tel_o, comp_o = occupancy_case
    s, o, d_base, d_moves = _dev(inst.s), _dev(inst.o), _dev(base), _dev(moves)
    best = int(np.argmin(tel_o))
    try:
        ctx.set_resume_min_rows(0 if mode == "from_start" else 1)
        for launch in range(2):
            print(f"moves, {mode}, launch {launch}: n={inst.n} K={moves.shape[0]}", flush=True)
            tel, res = ctx.best_neighbor(d_base, d_moves, s, o, inst.M)
            torch.cuda.synchronize()
            assert ctx.device_status() == 0
            bad = np.nonzero(tel.cpu().numpy() != tel_o)[0]
            assert bad.size == 0, f"{mode}, launch {launch}: total latency differs at moves {bad[:8]}"
            assert tuple(int(x) for x in res.cpu().numpy()) == (best, int(tel_o[best]), int(tel_o[0]))
    finally:
        ctx.set_resume_min_rows(-1)
