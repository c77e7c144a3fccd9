"""GPU parity of kvsched_online (scheduling under online arrivals) with the CPU oracle:
completion rounds and the four per-stream statistics, bit-exact."""
import os

import numpy as np
import pytest

import oracle
from paper_2508_06133_amd import workloads
from conftest import read_golden

pytestmark = pytest.mark.gpu

FCFS, MCSF, FOOT, SORTF = 0, 1, 2, 3


@pytest.fixture(scope="module")
def ctx():
    import torch
    from paper_2508_06133_amd import kvsched

    assert torch.cuda.is_available()
    c = kvsched.Context(0)
    yield c
    c.close()


def _to_dev(a, dtype=np.int32):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).to("cuda:0")


class Batch:
    """Streams to run in one call: request arrays are concatenated, a set of arrivals may be
    used by several streams (policies)."""

    def __init__(self):
        self.a, self.s, self.o, self.desc, self.cases = [], [], [], [], []
        self.N = 0
        self.out = 0

    def add_requests(self, a, s, o):
        begin = self.N
        self.a.append(np.asarray(a, dtype=np.int32))
        self.s.append(np.asarray(s, dtype=np.int32))
        self.o.append(np.asarray(o, dtype=np.int32))
        self.N += len(a)
        return begin, len(a)

    def add_stream(self, rng_, planner, period, window, refresh):
        begin, count = rng_
        self.desc.append([begin, count, planner, period, window, refresh[0], refresh[1], self.out])
        self.cases.append((begin, count, planner, period, window, refresh, self.out))
        self.out += count

    def run(self, ctx, M, what, cap=4096):
        import torch

        a, s, o = np.concatenate(self.a), np.concatenate(self.s), np.concatenate(self.o)
        print(f"online {what}: {len(self.desc)} streams, {self.N} requests, M={M}", flush=True)
        comp = torch.full((max(self.out, 1),), -7, dtype=torch.int32, device="cuda:0")
        comp, stats = ctx.online(_to_dev(np.array(self.desc)), _to_dev(a), _to_dev(s), _to_dev(o), M, comp,
                                 backlog_cap=cap)
        torch.cuda.synchronize()
        return a, s, o, comp.cpu().numpy(), stats.cpu().numpy()

    def check(self, ctx, M, what, cap=4096):
        a, s, o, comp, stats = self.run(ctx, M, what, cap)
        for k, (begin, count, planner, period, window, refresh, out) in enumerate(self.cases):
            sl = slice(begin, begin + count)
            p_o, c_o, st_o = oracle.online(a[sl], s[sl], o[sl], M, planner, period, window, refresh)
            assert tuple(int(x) for x in stats[k]) == st_o, (what, k, self.cases[k])
            assert (comp[out : out + count] == c_o).all(), (what, k, self.cases[k])
        assert ctx.device_status() == 0, what


def test_hand_worked_trace(ctx, golden_dir):
    g = read_golden(os.path.join(golden_dir, "online_worked.txt"))
    ints = lambda k: [int(x) for x in g[k].split()]
    b = Batch()
    r = b.add_requests(ints("a"), ints("s"), ints("o"))
    b.add_stream(r, SORTF, int(g["period"]), int(g["window"]), tuple(ints("refresh")))
    a, s, o, comp, stats = b.run(ctx, int(g["M"]), "hand-worked trace")
    assert list(comp) == [x + y for x, y in zip(ints("start"), ints("o"))]
    assert list(stats[0]) == [int(g["total_latency"]), int(g["refreshes"]), int(g["last_completion"]),
                              int(g["max_backlog"])]


def test_poisson_grid_three_policies(ctx):
    # the paper's online experiment: ten loads, arrivals over 4000 iterations, FCFS / shortest
    # decode first every iteration / Sorted-F-Online (refresh 10, window 300, 1/2)
    b = Batch()
    for rho in workloads.ONLINE_RHO:
        for seed in range(3):
            a, s, o, M = workloads.online_instance(seed, rho)
            r = b.add_requests(a, s, o)
            b.add_stream(r, FCFS, 1, 0, (0, 0))
            b.add_stream(r, MCSF, 1, 0, (0, 0))
            b.add_stream(r, SORTF, 10, 300, (1, 2))
    b.check(ctx, workloads.ONLINE_M, "Poisson grid", cap=512)


def test_policy_parameter_sweep(ctx):
    # one overloaded arrival sequence under many policy settings
    a, s, o, M = workloads.online_instance(7, 2.4)
    b = Batch()
    r = b.add_requests(a, s, o)
    for period in (1, 2, 5, 10, 50, 1000):
        for window in (0, 1, 16, 300, 1024):
            for refresh in ((1, 2), (0, 0), (3, 1), (1, 10)):
                b.add_stream(r, SORTF, period, window, refresh)
    for planner in (FCFS, MCSF, FOOT):
        for period in (1, 7, 100):
            b.add_stream(r, planner, period, 0, (1, 2))
    b.check(ctx, M, "parameter sweep", cap=1024)


def test_random_small_streams(ctx):
    rng = np.random.default_rng(21)
    for M_mode in range(3):
        b = Batch()
        M = (40, 120, 400)[M_mode]
        for k in range(150):
            n = int(rng.integers(1, 60))
            smax = int(rng.integers(1, M // 2))
            omax = int(rng.integers(1, M // 2))
            s = rng.integers(1, smax + 1, n)
            o = rng.integers(1, omax + 1, n)
            a = np.sort(rng.integers(0, int(rng.integers(1, 80)), n))
            r = b.add_requests(a, s, o)
            b.add_stream(r, int(rng.integers(0, 4)), int(rng.integers(1, 9)), int(rng.integers(0, 20)),
                         (int(rng.integers(0, 4)), int(rng.integers(0, 4))))
        b.check(ctx, M, f"random small streams, M={M}", cap=(64, 600, 4096)[M_mode])


def test_more_streams_than_run_at_once_are_taken_by_work(ctx):
    # beyond 1024 streams the library starts those with most work first (an order of its own over the
    # batch): results and their places in the outputs must not depend on it.  Streams of very
    # different sizes, and two with a malformed descriptor among them
    from paper_2508_06133_amd import kvsched

    rng = np.random.default_rng(23)
    b = Batch()
    M = 300
    for k in range(1300):
        n = int(rng.integers(1, 4)) if k % 3 else int(rng.integers(40, 160))
        s = rng.integers(1, 120, n)
        o = rng.integers(1, 120, n)
        a = np.sort(rng.integers(0, 50, n))
        r = b.add_requests(a, s, o)
        b.add_stream(r, int(rng.integers(0, 4)), int(rng.integers(1, 12)), int(rng.integers(0, 40)), (1, 2))
    b.check(ctx, M, "1300 streams", cap=512)
    bad = (17, 900)
    for k in bad:
        b.desc[k][3] = 0  # refresh period 0
    a, s, o, comp, stats = b.run(ctx, M, "1300 streams, two malformed", cap=512)
    assert ctx.device_status() == kvsched.DEV_BAD_STREAM
    for k, (begin, count, planner, period, window, refresh, out) in enumerate(b.cases):
        if k in bad:
            assert (stats[k] == -1).all()
        elif k % 50 == 0 or k in (16, 18, 899, 901):
            sl = slice(begin, begin + count)
            _, c_o, st_o = oracle.online(a[sl], s[sl], o[sl], M, planner, period, window, refresh)
            assert tuple(int(x) for x in stats[k]) == st_o and (comp[out : out + count] == c_o).all(), k


def test_bursts_deep_backlog_and_full_window(ctx):
    # everything arrives in a few large bursts: more than 256 arrivals per iteration (merged in
    # chunks), a backlog in the thousands, the largest window, batches of hundreds of requests
    rng = np.random.default_rng(22)
    b = Batch()
    n = 3500
    s = np.clip(np.rint(rng.lognormal(np.log(128.0), 0.8, n)), 4, 2048).astype(np.int32)
    o = np.clip(np.rint(rng.lognormal(np.log(200.0), 0.9, n)), 1, 2048).astype(np.int32)
    a = np.sort(rng.choice([0, 0, 0, 5, 40, 41, 300], n)).astype(np.int32)
    r = b.add_requests(a, s, o)
    b.add_stream(r, SORTF, 10, 1024, (1, 2))
    b.add_stream(r, SORTF, 3, 700, (0, 0))
    b.add_stream(r, FOOT, 10, 0, (1, 2))
    b.add_stream(r, MCSF, 1, 0, (0, 0))
    b.add_stream(r, FCFS, 1, 0, (0, 0))
    b.check(ctx, 131072, "bursts")


def test_longest_decode_and_idle_gaps(ctx):
    # decode lengths up to the limit (a ring slot per round of the longest decode, the slot of the
    # current round standing for the round one ring ahead), arrivals separated by gaps longer than the
    # ring, and a request that exactly fills the budget
    b = Batch()
    a = [0, 0, 3, 20000, 20000, 20001, 60000]
    s = [5, 1, 9, 1, 808, 2, 7]
    o = [8192, 8000, 1, 8192, 8191, 4000, 3]
    r = b.add_requests(a, s, o)
    for planner, period, window in ((FCFS, 1, 0), (MCSF, 1, 0), (FOOT, 4, 0), (SORTF, 10, 300), (SORTF, 1, 2)):
        b.add_stream(r, planner, period, window, (1, 2))
    b.check(ctx, 8999, "longest decode")
    # the same at a power-of-two limit of the smallest size class
    b = Batch()
    r = b.add_requests([0, 0, 1, 5000], [3, 1, 2, 1], [2048, 2048, 2047, 2048])
    for planner in (FCFS, MCSF, SORTF):
        b.add_stream(r, planner, 3, 4, (1, 2))
    b.check(ctx, 4100, "decode length = ring size", cap=16)


def test_long_waits_of_the_head_request(ctx):
    # the kernel passes the rounds at which the head of the list cannot start in one step: here the
    # head waits for hundreds of rounds behind a few long requests that nearly fill the budget, while
    # requests keep arriving, under every refresh rule (periods shorter and longer than the waits,
    # growth triggers that never / always / sometimes fire) -- refresh counts included
    rng = np.random.default_rng(77)
    for M, o_hi, n in ((600, 400, 60), (2000, 1500, 120), (300, 40, 200)):
        b = Batch()
        for rep in range(3):
            s = rng.integers(1, M // 4, n)
            o = rng.integers(max(1, o_hi // 3), o_hi + 1, n)
            short = rng.random(n) < 0.3
            o[short] = rng.integers(1, 6, int(short.sum()))
            a = np.sort(rng.integers(0, n * o_hi // 8, n))
            ok = s + o <= M
            s, o, a = s[ok], o[ok], a[ok]
            r = b.add_requests(a, s, o)
            for planner in (FCFS, MCSF, FOOT):
                for period in (1, 3, 1000):
                    for refresh in ((1, 2), (0, 0), (0, 1), (3, 1)):
                        b.add_stream(r, planner, period, 0, refresh)
            for period in (1, 7, 50, 1000):
                for window in (0, 2, 300):
                    for refresh in ((1, 2), (0, 0), (0, 3), (1, 10)):
                        b.add_stream(r, SORTF, period, window, refresh)
        b.check(ctx, M, f"long waits, M={M}", cap=256)


def test_all_present_at_round_zero_equals_offline(ctx):
    # arrivals all at round 0, one refresh, window over everything: the offline Sorted-F order
    # with Local Swap Search batches run through Phase 2
    import torch

    inst = workloads.instance(3, n=1000)
    b = Batch()
    r = b.add_requests(np.zeros(inst.n, dtype=np.int32), inst.s, inst.o)
    b.add_stream(r, SORTF, 1 << 30, 1024, (0, 0))
    a, s, o, comp, stats = b.run(ctx, inst.M, "all at round 0")
    order = oracle.local_swap(inst.s, inst.o, inst.M)[0]
    p0, c0, tel0 = oracle.simulate(inst.s, inst.o, inst.M, order, literal=False)
    assert (comp == c0).all() and int(stats[0, 0]) == tel0 and int(stats[0, 1]) == 1
    # and against the library's own offline path
    order_g = ctx.local_swap(_to_dev(inst.s), _to_dev(inst.o), inst.M)[0]
    tel_g, comp_g = ctx.simulate(order_g[None, :].contiguous(), _to_dev(inst.s), _to_dev(inst.o), inst.M)
    torch.cuda.synchronize()
    assert int(tel_g.item()) == tel0 and (comp_g.cpu().numpy()[0] == comp).all()


def test_size_classes_agree_and_the_bound_is_enforced(ctx):
    # the same streams under every backlog bound that holds them: identical results; under a bound
    # below the largest backlog the stream is faulted, whatever size class the bound falls in
    a, s, o, M = workloads.online_instance(3, 2.4)
    b = Batch()
    r = b.add_requests(a, s, o)
    b.add_stream(r, FCFS, 1, 0, (0, 0))
    b.add_stream(r, SORTF, 10, 300, (1, 2))
    ref = None
    for cap in (4096, 1024, 512, 400):
        _, _, _, comp, stats = b.run(ctx, M, f"size class for bound {cap}", cap)
        if ref is None:
            ref = (comp.copy(), stats.copy())
            worst = int(stats[0, 3])
            assert 100 < worst <= 400 and int(stats[1, 3]) < worst
        assert (comp == ref[0]).all() and (stats == ref[1]).all(), cap
        assert ctx.device_status() == 0
    _, _, _, comp, stats = b.run(ctx, M, "bound below the backlog", worst - 1)
    assert list(stats[0]) == [-1, -1, -1, -1] and (stats[1] == ref[1][1]).all()
    _, _, _, comp, stats = b.run(ctx, M, "bound at the backlog", worst)
    assert (stats == ref[1]).all()


def test_faults_are_reported_per_stream(ctx):
    import torch
    from paper_2508_06133_amd import kvsched

    M = 100
    b = Batch()
    good = b.add_requests([0, 1, 2], [3, 3, 3], [2, 2, 2])
    unsorted = b.add_requests([4, 2, 9], [3, 3, 3], [2, 2, 2])
    b.add_stream(good, FCFS, 1, 0, (0, 0))
    b.add_stream(unsorted, FCFS, 1, 0, (0, 0))
    b.add_stream(good, 9, 1, 0, (0, 0))                    # unknown planner
    b.add_stream(good, SORTF, 0, 10, (1, 2))               # period < 1
    b.add_stream(good, SORTF, 5, 2000, (1, 2))             # window above the limit
    b.add_stream((good[0], 50), FCFS, 1, 0, (0, 0))        # runs past the request arrays
    b.out = 64
    a, s, o, comp, stats = b.run(ctx, M, "faults")
    assert list(stats[0]) == [6, 3, 4, 1]
    for k in range(1, 6):
        assert list(stats[k]) == [-1, -1, -1, -1], k
    st = ctx.device_status()
    assert st & kvsched.DEV_BAD_ARRIVAL and st & kvsched.DEV_BAD_STREAM

    # a backlog beyond the limit
    n = kvsched.ONLINE_MAX_BACKLOG + 5
    b = Batch()
    r = b.add_requests(np.zeros(n, dtype=np.int32), np.full(n, 60), np.full(n, 30))
    b.add_stream(r, FCFS, 1, 0, (0, 0))
    a, s, o, comp, stats = b.run(ctx, M, "backlog overflow")
    assert list(stats[0]) == [-1, -1, -1, -1] and ctx.device_status() & kvsched.DEV_BACKLOG

    # a request that can never fit; a decode length above the limit is refused by the host
    b = Batch()
    r = b.add_requests([0, 0], [3, 90], [2, 20])
    b.add_stream(r, FCFS, 1, 0, (0, 0))
    a, s, o, comp, stats = b.run(ctx, M, "bad length")
    assert list(stats[0]) == [-1, -1, -1, -1] and ctx.device_status() & kvsched.DEV_BAD_LENGTH
    with pytest.raises(kvsched.KvschedError) as e:
        comp = torch.zeros(2, dtype=torch.int32, device="cuda:0")
        ctx.online(_to_dev(np.array([[0, 2, 0, 1, 0, 0, 0, 0]])), _to_dev([0, 0]), _to_dev([1, 1]),
                   _to_dev([5, kvsched.ONLINE_MAX_O + 1]), 1 << 20, comp)
    assert e.value.code == -2
    with pytest.raises(kvsched.KvschedError) as e:
        ctx.online(_to_dev(np.array([[0, 2, 0, 1, 0, 0, 0, 0]])), _to_dev([0, 0]), _to_dev([1, 1]), _to_dev([5, 5]),
                   1 << 20, comp, backlog_cap=kvsched.ONLINE_MAX_BACKLOG + 1)
    assert e.value.code == -2
