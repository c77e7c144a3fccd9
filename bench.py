#!/usr/bin/env python3
"""Benchmark of the schedule-evaluation hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input, everything already
resident in HBM: Sorted-F order construction (Phase 1), evaluation of the candidate orders (Phase 2:
timelines, total latency and completion rounds per candidate), argmin over the candidates.

Default workload: configuration 3 ("mixed chat + summarisation": n = 2000 requests, M = 131072
tokens, C = 16384 candidates = Sorted-F order, 16127 distinct 1-swap neighbours, 256 random
restarts).  --workload config1 | config2 | config5 run the same step on those configurations,
--workload config4 the receding-horizon run (one step = all re-plans of 65536 moves each until every
position is committed).

Prints ONE JSON line: candidate schedules evaluated per second, request-rounds per second, the
roofline object of the dominant kernel (integer-VALU bound; algorithmic lane-ops counted from the
outputs of the run, kernel time from HIP events on the kernel's stream) and the CPU oracle timed on
a sample of the same candidates on this host, on one thread and on all cores.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Peak plain-ALU rate of the chip: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one int32 op per
# lane per clock (the fp32 vector peak of 157.3 TFLOP/s counts an FMA as two and packs two).
PEAK_INT32_LANE_OPS = 256 * 4 * 16 * 2.4e9
PEAK_HBM_BYTES = 8.0e12
# Lane-ops no dense-profile kernel on this instruction set can do without.  A visit is one future
# round of one request's window, inspected (the admission check, including the rounds that enter the
# window while the request waits) or updated (the admitted request's memory added to the profile).
#   * an inspected round has to be an operand of some vector instruction at least once, and an
#     instruction takes at most two new operands next to its accumulator (v_max3_i32): 1/2 lane-op;
#   * an updated round has to be written back by some vector instruction: 1 lane-op.
# The kernel's row chains come to 1/2 and 3/2 (the ramp shared by two rows costs a step).  Everything
# else it issues (the masked last row, dead lanes of partial rows, per-request bookkeeping, the second
# pass with the rows' limits, moving the register file) is overhead and is not credited, so the
# fraction below cannot exceed the share of issue slots the kernel uses.
OPS_PER_INSPECTED = 0.5
OPS_PER_UPDATED = 1.0
# The credit in use before the admission check became a plain maximum over the rows (add, min per row
# and a three-way maximum per two rows, two adds and a ramp step per two rows: 2 per visit); kept as
# a second figure so that the kernels can be compared across that change.
OPS_PER_VISIT_BEFORE = 2
CFG = 3

# What rocprofv3 counters measured for the dominant kernel of a workload (summaries and commands in
# profiles/): HBM bytes per launch (FETCH_SIZE, WRITE_SIZE scaled by what a plain 256 MiB copy reads
# on the same counters), share of the vector / scalar issue slots in use, vector lane-slots issued
# per credited visit.  Valid only for the kernel sources they were taken on (hash below); reported as
# null once those change.
PROFILED = {
    # profiles/timeline_kernel_config3_traffic.md, timeline_kernel_config3_counters.md
    "config3": {"traffic_bytes": int((42913.8 * 1.99974 + 77268.3 * 1.0) * 1024),
                "issue": {"valu": 0.895, "scalar_and_branch": 0.760, "lane_slots_per_visit": 3.27,
                          "source": "profiles/timeline_kernel_config3_counters.md"}},
    # profiles/timeline_kernel_config5_rows65.md (one wavefront per SIMD)
    "config5": {"traffic_bytes": None,
                "issue": {"valu": 0.362, "scalar_and_branch": 0.089, "lane_slots_per_visit": 1.05,
                          "source": "profiles/timeline_kernel_config5_rows65.md"}},
    # profiles/timeline_kernel_config4_moves.md (candidates' launches; the counters give 1.07 vector
    # instructions per SIMD and four nominal clocks: saturated)
    "config4": {"traffic_bytes": None,
                "issue": {"valu": 1.0, "scalar_and_branch": 0.91, "lane_slots_per_visit": 2.84,
                          "source": "profiles/timeline_kernel_config4_moves.md"}},
}
PROFILED_SOURCES = ("timeline_reg.hip", "device_util.h")
PROFILED_SOURCES_SHA256 = "4ba068fa5037d160"


def _kernel_sources_hash() -> str:
    import hashlib

    h = hashlib.sha256()
    for f in PROFILED_SOURCES:
        with open(os.path.join(ROOT, "paper_2508_06133_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def profiled(workload: str):
    """(traffic bytes per launch, issue figures) from the committed counter summaries, or (None, None)."""
    rec = PROFILED.get(workload)
    if rec is None or _kernel_sources_hash() != PROFILED_SOURCES_SHA256:
        return None, None
    return rec.get("traffic_bytes"), rec.get("issue")


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def host_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))  # a one-GPU machine's share of the host is 16 cores


def cpu_baseline_rows(inst, make_rows, C: int, tel_gpu, what: str):
    """The oracle (oracle_simulate_profile, as it stands) on a bounded sample of the candidates:
    one thread, then every host thread at once (one ordinary single-threaded call per chunk of rows;
    ctypes releases the interpreter lock).  make_rows(lo, hi) -> order rows [hi - lo, n] of candidates
    lo..hi-1.  Returns the cpu_baseline object, or None when GPU and oracle disagree."""
    import oracle  # test infrastructure; only this baseline leg uses it

    def run(rows):
        return oracle.simulate_many(inst.s, inst.o, inst.M, rows, literal=False, completions=True)[0]

    t0 = time.perf_counter()
    probe = run(make_rows(0, min(2, C)))
    per_row = max((time.perf_counter() - t0) / min(2, C), 1e-6)
    if not (probe == tel_gpu[: len(probe)]).all():
        return None
    threads = host_threads()
    n1 = int(min(C, max(2, 6.0 / per_row)))
    rows1 = make_rows(0, n1)
    t0 = time.perf_counter()
    tel1 = run(rows1)
    s1 = time.perf_counter() - t0
    if not (tel1 == tel_gpu[:n1]).all():
        return None
    nA = int(min(C, max(threads, 6.0 * threads / per_row)))
    rowsA = rows1 if nA == n1 else make_rows(0, nA)
    chunk = max(1, min(64, -(-nA // (4 * threads))))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(lambda lo: run(rowsA[lo:lo + chunk]), range(0, nA, chunk)))
    sA = time.perf_counter() - t0
    if not (np.concatenate(parts) == tel_gpu[:nA]).all():
        return None
    return {
        "value": nA / sA,
        "unit": "candidates/s",
        "cores": threads,
        "kind": "oracle",
        "cpu_model": cpu_model(),
        "host_cores": os.cpu_count(),
        "single_thread": {"value": n1 / s1, "unit": "candidates/s", "cores": 1, "sample_rows": n1, "seconds": round(s1, 2)},
        "sample": f"first {nA} of the {C} {what} on {threads} threads ({sA:.1f} s), first {n1} on one thread "
                  f"({s1:.1f} s); array-profile oracle (oracle_simulate_profile), plain C, one row after the other per thread",
    }


def roofline_object(kernel: str, inspected: int, updated: int, kernel_ms_total: float, launches: int, workload: str,
                    hbm_bytes: int, extra: dict | None = None):
    """Integer-VALU roofline of the timeline kernel: credited lane-ops = inspected / 2 + updated."""
    secs = kernel_ms_total * 1e-3
    visits = inspected + updated
    ops = OPS_PER_INSPECTED * inspected + OPS_PER_UPDATED * updated
    achieved = ops / secs
    traffic, issue = profiled(workload)
    obj = {
        "bound": "alu",
        "kernel": kernel,
        "launches": launches,
        "avg_launch_ms": kernel_ms_total / launches,
        "achieved": achieved / 1e12,
        "peak": PEAK_INT32_LANE_OPS / 1e12,
        "unit": "Tlane-op/s (int32)",
        "frac": achieved / PEAK_INT32_LANE_OPS,
        "traffic": traffic,
        "visits": visits,
        "inspected": inspected,
        "updated": updated,
        "ops_per_visit": ops / visits,
        "frac_at_two_ops_per_visit": OPS_PER_VISIT_BEFORE * visits / secs / PEAK_INT32_LANE_OPS,
        "issue_measured": issue,
        "hbm": {"algorithmic_bytes": hbm_bytes, "achieved_GBps": hbm_bytes / secs / 1e9,
                "frac_of_8TBps": hbm_bytes / secs / PEAK_HBM_BYTES},
    }
    if extra:
        obj.update(extra)
    return obj


def reg_rows(o_max: int) -> int:
    rows = (o_max + 63) // 64 + 1
    return 9 if rows <= 9 else 33 if rows <= 33 else 65


def bench_online(args, ctx, dev) -> int:
    """One step = every stream of the Poisson grid run to completion: 10 load levels x
    `online_seeds` arrival sequences x 3 policies (arrival order, shortest decode first every
    iteration, Sorted-F-Online with refresh 10 / window 300 / growth trigger 1/2)."""
    import torch

    from paper_2508_06133_amd import kvsched, workloads

    A, S, O, desc = [], [], [], []
    N = out = 0
    policies = ((kvsched.PLANNER_ARRIVAL, 1, 0, 0, 0), (kvsched.PLANNER_SHORTEST_DECODE, 1, 0, 0, 0),
                (kvsched.PLANNER_SORTED_F, 10, 300, 1, 2))
    for rho in workloads.ONLINE_RHO:
        for seed in range(args.online_seeds):
            a, s, o, M = workloads.online_instance(seed, rho)
            A.append(a), S.append(s), O.append(o)
            for pl, per, win, num, den in policies:
                desc.append([N, len(a), pl, per, win, num, den, out])
                out += len(a)
            N += len(a)
    a, s, o = np.concatenate(A), np.concatenate(S), np.concatenate(O)
    a_d, s_d, o_d = (torch.from_numpy(x).to(dev) for x in (a, s, o))
    desc_d = torch.tensor(desc, dtype=torch.int32, device=dev)
    comp = torch.zeros(out, dtype=torch.int32, device=dev)
    stats = torch.zeros((len(desc), 4), dtype=torch.int64, device=dev)
    ctx.set_o_max(2048)  # the generator clips decode lengths there; makes the call asynchronous
    cap = 512

    def step():
        ctx.online(desc_d, a_d, s_d, o_d, M, comp, stats_out=stats, backlog_cap=cap)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if ctx.device_status() != 0:
        print("bench.py: device status", ctx.device_status(), file=sys.stderr)
        return 1
    st = stats.cpu().numpy()
    B = len(desc)
    iterations = int(st[:, 2].sum())  # rounds up to the last completion, summed over streams
    result = {
        "metric": "online request streams evaluated/s (Poisson arrivals, 3 policies)",
        "value": B * args.steps / wall,
        "unit": "streams/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": f"online Poisson arrivals: {len(workloads.ONLINE_RHO)} loads x {args.online_seeds} "
                               f"sequences x 3 policies, T={workloads.ONLINE_T}, M={M}",
                   "streams": B, "requests": int(N), "backlog_cap": cap},
        "requests_per_s": out * args.steps / wall,
        "rounds_per_s": iterations * args.steps / wall,
        "roofline": None,  # a stream is a chain of dependent steps: latency-bound, no throughput roofline applies
    }
    if not args.no_cpu_baseline:
        import oracle  # test infrastructure; only this baseline leg uses it

        pick = list(range(0, B, max(1, B // 150)))
        t0 = time.perf_counter()
        for k in pick:
            b0, cnt, pl, per, win, num, den, _ = desc[k]
            _, _, so = oracle.online(a[b0:b0 + cnt], s[b0:b0 + cnt], o[b0:b0 + cnt], M, pl, per, win, (num, den))
            if so != tuple(int(x) for x in st[k]):
                print("bench.py: GPU and oracle disagree on stream", k, file=sys.stderr)
                return 1
        cpu_s = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": len(pick) / cpu_s, "unit": "streams/s", "cores": 1, "kind": "oracle",
                                  "sample": f"every {max(1, B // 150)}th of the {B} streams (oracle_online, "
                                            f"array-profile form), single thread, {cpu_s:.1f} s"}
    print(json.dumps(result))
    ctx.close()
    return 0


def bench_phase1(args, ctx, dev) -> int:
    """One step = the Phase-1 constructions of the library on resident inputs: the sorted-prefix
    order under both feasibility tests and Local Swap Search on configs 3, 4 and 5 (n = 2000, 10000,
    100000), the exact batches of Algorithm 2 on the first 100 requests of config 2."""
    import torch

    from paper_2508_06133_amd import kvsched, workloads

    cases = []
    for cfg in (3, 4, 5):
        inst = workloads.instance(cfg)
        cases.append((cfg, inst, torch.from_numpy(inst.s).to(dev), torch.from_numpy(inst.o).to(dev)))
    small = workloads.instance(2, n=100)
    s_small, o_small = torch.from_numpy(small.s).to(dev), torch.from_numpy(small.o).to(dev)
    out = {}

    def step():
        for cfg, inst, s, o in cases:
            out[cfg, "prefix"] = ctx.sortedF(s, o, inst.M, kvsched.TIE_LARGER, kvsched.FEAS_SUM_OF_PEAKS)
            out[cfg, "prefix_profile"] = ctx.sortedF(s, o, inst.M, kvsched.TIE_LARGER, kvsched.FEAS_PROFILE)
            out[cfg, "swap"] = ctx.local_swap(s, o, inst.M)
        out[2, "exact"] = ctx.exact_dp(s_small, o_small, small.M)

    calls = 3 * len(cases) + 1
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if ctx.device_status() != 0:
        print("bench.py: device status", ctx.device_status(), file=sys.stderr)
        return 1
    requests = sum(3 * inst.n for _, inst, _, _ in cases) + small.n
    result = {
        "metric": "Phase-1 orders constructed/s (sorted prefix, Local Swap Search, exact batches)",
        "value": calls * args.steps / wall,
        "unit": "orders/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int64",
        "data": "synthetic",
        "config": {"workload": "Phase 1: sorted prefix (sum of peaks, profile) and Local Swap Search on configs 3, 4, 5 "
                               "(n = 2000, 10000, 100000); Algorithm 2 on 100 requests of config 2",
                   "calls_per_step": calls, "requests_per_step": requests},
        "batches": {f"config{cfg}_{k}": int(v[-1].item()) for (cfg, k), v in out.items()},
        "roofline": None,  # one workgroup per construction, a chain of short dependent steps: latency-bound
    }
    if not args.no_cpu_baseline:
        import oracle  # test infrastructure; only this baseline leg uses it

        t0 = time.perf_counter()
        n_cpu = 0
        for cfg, inst, _, _ in cases[:2]:  # config 5 takes the oracle's quadratic Local Swap Search minutes
            ref = {"prefix": oracle.sortedF(inst.s, inst.o, inst.M, feas_mode=0),  # sum of peaks
                   "prefix_profile": oracle.sortedF(inst.s, inst.o, inst.M, feas_mode=1),  # profile
                   "swap": oracle.local_swap(inst.s, inst.o, inst.M)}
            n_cpu += 3
            for k, r in ref.items():
                if not (np.asarray(r[0]) == out[cfg, k][0].cpu().numpy()).all():
                    print(f"bench.py: GPU and oracle disagree on config {cfg} {k}", file=sys.stderr)
                    return 1
        cpu_s = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": n_cpu / cpu_s, "unit": "orders/s", "cores": 1, "kind": "oracle",
                                  "sample": f"the {n_cpu} constructions on configs 3 and 4 (oracle_sortedF, "
                                            f"oracle_local_swap), single thread, {cpu_s:.1f} s"}
    print(json.dumps(result))
    ctx.close()
    return 0


def bench_predicted(args, ctx, dev) -> int:
    """One step = Phase 1 on the lower bounds + the 16384 config-3 candidate orders run under
    predicted decode lengths (running estimates from the lower bounds, ordered eviction) + argmin."""
    import torch

    from paper_2508_06133_amd import workloads

    inst = workloads.instance(CFG)
    n, M = inst.n, inst.M
    lower, upper = workloads.prediction_intervals(CFG, inst.s, inst.o, M, args.gamma)
    s = torch.from_numpy(inst.s).to(dev)
    o = torch.from_numpy(inst.o).to(dev)
    lo = torch.from_numpy(lower).to(dev)
    order_d, _, _, nb_d = ctx.sortedF(s, lo, M)  # the scheduler sees only the predictions
    torch.cuda.synchronize()
    rows_h = workloads.candidates(CFG, order_d.cpu().numpy())
    C = rows_h.shape[0]
    orders = torch.from_numpy(rows_h).to(dev)
    ctx.set_o_max(int(max(inst.o.max(), lower.max())))
    best = torch.empty(2, dtype=torch.int64, device=dev)
    out = {}

    def step():
        ctx.sortedF(s, lo, M)
        out["r"] = ctx.simulate_predicted(orders, s, o, lo, M)
        ctx.argmin(out["r"][0], result_out=best)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if ctx.device_status() != 0:
        print("bench.py: device status", ctx.device_status(), file=sys.stderr)
        return 1
    tel, comp, ev = out["r"]
    tel_h = tel.cpu().numpy()
    result = {
        "metric": "candidate schedules evaluated/s under predicted decode lengths (n=2000 mixed)",
        "value": C * args.steps / wall,
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": f"config 3 candidates (n={n}, M={M}, C={C}) under interval predictions, gamma={args.gamma}, "
                               "estimates started from the lower bounds", "n": n, "M": M, "C": C},
        "mean_evictions_per_candidate": float(ev.float().mean().item()),
        "best_candidate": {"index": int(best[0].item()), "tel": int(best[1].item()), "base_tel": int(tel_h[0])},
        "roofline": None,  # a round-by-round event loop per candidate: latency- and LDS-capacity-bound
    }
    if not args.no_cpu_baseline:
        import oracle  # test infrastructure; only this baseline leg uses it

        rows_cpu = min(args.cpu_rows, 128)
        t0 = time.perf_counter()
        for c in range(rows_cpu):
            _, c_o, tel_o, ev_o, _ = oracle.simulate_predicted(inst.s, inst.o, lower, M, rows_h[c])
            if tel_o != tel_h[c]:
                print("bench.py: GPU and oracle disagree on row", c, file=sys.stderr)
                return 1
        cpu_s = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": rows_cpu / cpu_s, "unit": "candidates/s", "cores": 1, "kind": "oracle",
                                  "sample": f"first {rows_cpu} of the {C} candidate rows (oracle_simulate_predicted, "
                                            f"array form), single thread, {cpu_s:.1f} s"}
    print(json.dumps(result))
    ctx.close()
    return 0


def bench_rows(args, ctx, dev, cfg: int) -> int:
    """Configurations 1, 2, 3, 5: one step = Sorted-F order (sorted-prefix scoring, or Local Swap
    Search with --phase1 local_swap) + timelines of all candidate rows + argmin."""
    import torch

    from paper_2508_06133_amd import workloads

    inst = workloads.instance(cfg)
    scale = int(args.decode_scale)
    if scale > 1:  # the same instance with decode lengths and budget scaled: the larger register files
        inst = dataclasses.replace(inst, o=np.minimum(inst.o.astype(np.int64) * scale, 14336).astype(np.int32),
                                   M=int(inst.M) * scale)
    n, M = inst.n, inst.M
    s = torch.from_numpy(inst.s).to(dev)
    o = torch.from_numpy(inst.o).to(dev)

    # The candidate set is built around the Sorted-F order; that order comes from the library.
    order_d, ends_d, F_d, nb_d = ctx.sortedF(s, o, M)
    torch.cuda.synchronize()
    base = order_d.cpu().numpy()
    rows_h = workloads.candidates(cfg, base)
    C = rows_h.shape[0]
    orders = torch.from_numpy(rows_h).to(dev)
    tel = torch.empty(C, dtype=torch.int64, device=dev)
    comp = torch.empty((C, n), dtype=torch.int32, device=dev)
    best = torch.empty(2, dtype=torch.int64, device=dev)

    p1_out = (order_d, ends_d, F_d, nb_d)  # Phase 1 writes into the same tensors every step
    o_max = int(inst.o.max())
    ctx.set_o_max(o_max)  # the caller's bound on decode lengths: no read-back inside the step
    ctx.reserve(C, n, 0)  # scratch sized once: no call of the loop allocates
    ctx.enable_timing(True)
    stream = torch.cuda.current_stream()

    def step():
        if args.phase1 == "local_swap":
            ctx.local_swap(s, o, M)
        else:
            ctx.sortedF(s, o, M, out=p1_out)
        ctx.simulate(orders, s, o, M, tel_out=tel, completion_out=comp)
        ctx.argmin(tel, result_out=best)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    kernel_ms = []
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
        kernel_ms.append(ctx.last_timeline_ms())  # events on the stream the kernel ran on
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = ev0.elapsed_time(ev1)
    status = ctx.device_status()
    if status != 0:
        print(f"bench.py: device status {status}", file=sys.stderr)
        return 1

    if args.calibrate_copy:  # 2^26 int32 = 256 MiB read + 256 MiB written by one elementwise kernel
        src = torch.arange(1 << 26, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- accounting from the outputs of the run (outside the timed region)
    tel_h = tel.cpu().numpy()
    o64 = o.to(torch.int64)
    sum_o = int(o64.sum().item())
    last_req = orders[:, -1].to(torch.int64)
    p_last = comp.gather(1, last_req[:, None]).squeeze(1).to(torch.int64) - o64[last_req]
    # Rows that share leading positions with row 0 start from row 0's saved state; only what
    # they place themselves is counted: rounds waited through since the resume point + window
    # checked + window updated for the positions from there on.
    resume = ctx.simulate_resume_positions(C).to(torch.int64)
    order0 = orders[0].to(torch.int64)
    o_row0 = o64[order0]
    start0 = comp[0].to(torch.int64)[order0] - o_row0  # start rounds of row 0 by position
    cum0 = torch.cat([torch.zeros(1, dtype=torch.int64, device=dev), torch.cumsum(o_row0, 0)])
    t_res = torch.where(resume > 0, start0[(resume - 1).clamp(min=0)], torch.zeros_like(resume))
    # ... and a row whose timeline became row 0's again stopped placing there: positions [resume, stop)
    stop = torch.maximum(ctx.simulate_stop_positions(C, n).to(torch.int64), resume)
    rejoined = stop < n
    p_end = torch.where(rejoined, torch.where(stop > resume, start0[(stop - 1).clamp(min=0)], t_res), p_last)
    updated = int((cum0[stop] - cum0[resume]).sum().item())
    inspected = int((p_end - t_res).sum().item()) + updated
    visits_from_scratch = int((p_last + 2 * sum_o).sum().item())
    resumed_rows = int((resume > 0).sum().item())
    rejoined_rows = int(rejoined.sum().item())
    hbm_bytes = int((8 * (stop - resume) + 8).sum().item()) + 8 * n  # order entries read, completion rounds written, for the positions placed
    kernel = f"timeline_reg_kernel<{reg_rows(o_max)},{'1,false,true,true' if resumed_rows else '4,false,false,false'}>"
    names = {1: "config 1: tiny exact, n=8, M=48, all 8! orders + the Sorted-F order",
             2: "config 2: short conversation, n=200, M=16384, Sorted-F order + 4095 random pairwise swaps",
             3: "config 3: mixed chat+summarization, n=2000, M=131072, C=16384 "
                "(Sorted-F order + 16127 1-swap neighbours + 256 random restarts)",
             5: "config 5: adversarial bimodal, n=100000, M=2097152, Sorted-F order (prefix scoring of every batch) "
                "+ 1024 rows of 64 random swaps"}
    result = {
        "metric": f"candidate schedules evaluated/s (config {cfg}, n={n}, decode lengths x {scale})" if scale > 1
                  else "candidate schedules evaluated/s (n=2000 mixed)" if cfg == 3
                  else f"candidate schedules evaluated/s (config {cfg}, n={n})",
        "value": C * args.steps / wall,
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": names[cfg] + (f"; decode lengths and budget x {scale} (o_max {o_max})" if scale > 1 else ""),
                   "n": n, "M": M, "C": C, "sortedF_batches": int(nb_d.item()), "phase1": args.phase1},
        "request_rounds_per_s": C * sum_o * args.steps / wall,
        "gpu_ms_per_step": gpu_ms / args.steps,
        "timeline_kernel_ms": float(np.mean(kernel_ms)),
        "best_candidate": {"index": int(best[0].item()), "tel": int(best[1].item()), "base_tel": int(tel_h[0])},
        "roofline": roofline_object(kernel, inspected * args.steps, updated * args.steps, float(np.sum(kernel_ms)), args.steps,
                                    f"config{cfg}" if scale == 1 else "scaled",
                                    hbm_bytes * args.steps,
                                    {"resumed_rows": resumed_rows, "rejoined_rows": rejoined_rows,
                                     "visits_without_resume": visits_from_scratch}),
    }
    if not args.no_cpu_baseline:
        base_line = cpu_baseline_rows(inst, lambda lo, hi: rows_h[lo:hi], C, tel_h, "candidate rows")
        if base_line is None:
            print("bench.py: GPU and oracle disagree on the sampled rows", file=sys.stderr)
            return 1
        result["cpu_baseline"] = base_line
    print(json.dumps(result))
    ctx.close()
    return 0


def bench_horizon(args, ctx, dev) -> int:
    """Configuration 4: one step = the whole receding-horizon run (n = 10000, windows of 512 positions,
    65536 swap / insert moves per window, a new plan after every 256 completions, every timeline run
    to completion), through kvsched_horizon_step; the host loop draws each window's moves and reads
    48 bytes back per re-plan."""
    import torch

    from paper_2508_06133_amd import horizon, workloads

    inst = workloads.instance(4)
    n, M = inst.n, inst.M
    window, every, K = 512, 256, 65536
    s = torch.from_numpy(inst.s).to(dev)
    o = torch.from_numpy(inst.o).to(dev)
    order_d, _, _, nb_d = ctx.sortedF(s, o, M)
    torch.cuda.synchronize()
    o_max = int(inst.o.max())
    ctx.reserve(0, n, K)  # scratch sized once: no call of the loop allocates
    ctx.enable_timing(True)

    class Timed:  # the context, recording the candidates' launch time of every re-plan
        def __init__(self):
            self.ms = []

        def horizon_step(self, *a, **kw):
            out = ctx.horizon_step(*a, **kw)
            self.ms.append(ctx.last_timeline_ms())
            return out

    p1_out = ctx.sortedF(s, o, M)

    def run(keep_tel=False, max_steps=None, timed=None, keep_completion=False):
        ctx.sortedF(s, o, M, out=p1_out)  # Phase 1 is part of the step (the order itself is order_d, computed above)
        return horizon.receding_horizon(timed or ctx, s, o, M, order_d, window, every, K, rng=np.random.default_rng(4),
                                        keep_tel=keep_tel, max_steps=max_steps, keep_completion=keep_completion)

    for _ in range(min(args.warmup, 1)):
        run()
    torch.cuda.synchronize()
    timed = Timed()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        order_g, comp_g, log = run(timed=timed)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    class Accounted:  # the context, recording where the library stopped placing each move's timeline
        def __init__(self):
            self.stops = []

        def horizon_step(self, *a, **kw):
            out = ctx.horizon_step(*a, **kw)
            self.stops.append(ctx.neighbor_stop_positions(K, n).cpu().numpy().astype(np.int64))
            return out

    accounted = Accounted()
    _, _, log = run(keep_completion=True, timed=accounted)  # the same run once more, untimed, keeping every chosen timeline for the accounts
    status = ctx.device_status()
    if status != 0:
        print(f"bench.py: device status {status}", file=sys.stderr)
        return 1
    replans = len(log)
    timelines = replans * (K + 2)  # the moves, the order as it stands, the chosen order again for its completion rounds

    # ---- accounting (outside the timed region).  Every candidate of a window repeats the order up to
    # the first position a move touches: the library places that prefix once (windows behind position 64)
    # or starts each move from the state saved at its 64-position block (first window).  Credited per
    # candidate: rounds waited through from its start point on + windows checked and updated for the
    # positions from there on, with the start rounds of the chosen timeline of that re-plan standing in
    # for the candidates' own (they differ inside the window only; 2 sum(o) dominates).
    o_h = inst.o.astype(np.int64)
    rng = np.random.default_rng(4)
    order = order_d.cpu().numpy()
    waited = 0   # rounds that entered a window while its request waited
    window = 0   # rounds of the windows themselves: each inspected once and updated once
    hbm_bytes = 0
    kept_prefix = 0
    stops_seen = []  # per re-plan: moves not placed to their end
    for rec in log:
        moves = workloads.window_moves(rng, K, rec["lo"], rec["hi"])
        touched = np.minimum(moves[:, 1], moves[:, 2])
        ident = moves[:, 1] == moves[:, 2]
        order = workloads.apply_move(order, moves[rec["best"]])
        start = (rec["completion"].astype(np.int64) - o_h)[order]  # start rounds of the chosen order, by position
        cum = np.concatenate([[0], np.cumsum(o_h[order])])
        lowest = int(touched[~ident].min()) if (~ident).any() else n
        if lowest >= 64:  # common prefix placed once, every candidate starts behind it
            first = np.full(K + 1, lowest, dtype=np.int64)
            # the prefix itself: continued from the state the step before left behind its own prefix
            kept = kept_prefix if 64 <= kept_prefix <= lowest else 0
            waited += int(start[lowest - 1] - (start[kept - 1] if kept > 0 else 0))
            window += int(cum[lowest] - cum[kept])
            kept_prefix = lowest
        else:  # from the saved state of the move's block (identity moves: of the last block)
            kept_prefix = 0
            first = np.where(ident, (n - 1) // 64 * 64, touched // 64 * 64).astype(np.int64)
            first = np.concatenate([first, [0]])  # the order as it stands runs from the start and saves the states
        t_first = np.where(first > 0, start[np.maximum(first - 1, 0)], 0)
        # a move whose timeline became the order's own again was placed up to there only, or not at all
        stop = np.maximum(np.concatenate([accounted.stops[len(stops_seen)], [n]]), first)
        stops_seen.append(int((stop < n).sum()))
        t_end = np.where(stop < n, np.where(stop > first, start[np.maximum(stop - 1, 0)], t_first), start[-1])
        waited += int((t_end - t_first).sum())
        window += int((cum[stop] - cum[first]).sum())
        # ... and the chosen order once more, from the common prefix's state on where there is one
        chosen_first = lowest if lowest >= 64 else 0
        waited += int(start[-1] - (start[chosen_first - 1] if chosen_first > 0 else 0))
        window += int(cum[n] - cum[chosen_first])
        hbm_bytes += 12 * K + 8 * (K + 1) + 12 * n
    kernel_ms_total = float(np.sum(timed.ms))
    launches = len(timed.ms)
    sum_o = int(o_h.sum())
    result = {
        "metric": "candidate schedules evaluated/s (config 4, receding horizon, n=10000)",
        "value": timelines * args.steps / wall,
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": min(args.warmup, 1),
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": "config 4: receding horizon, n=10000 (config-3 mixture), M=1048576, windows of 512 positions "
                               "re-planned every 256 completions, 65536 swap/insert moves per window, every timeline to completion",
                   "n": n, "M": M, "moves_per_window": K, "replans_per_step": replans, "sortedF_batches": int(nb_d.item())},
        "request_rounds_per_s": timelines * sum_o * args.steps / wall,
        "ms_per_replan": wall * 1e3 / args.steps / replans,
        "candidate_launch_ms_per_replan": kernel_ms_total / launches,
        "final_tel": int(log[-1]["best_tel"]), "start_tel": int(log[0]["base_tel"]),
        "roofline": roofline_object(f"timeline_reg_kernel<{reg_rows(o_max)},4,true,...> (the candidates' launch of each re-plan)",
                                    (waited + window) * args.steps, window * args.steps, kernel_ms_total, launches,
                                    "config4", hbm_bytes * args.steps,
                                    {"moves_stopped_early": int(sum(stops_seen)),
                                     "note": "visits credited from each candidate's start point (common prefix or saved "
                                             "state of its block) on; the chosen timeline's start rounds stand in for the "
                                             "candidates' own"}),
    }
    if not args.no_cpu_baseline:
        # the first window's candidates through the oracle
        _, _, log1 = run(keep_tel=True, max_steps=1)
        torch.cuda.synchronize()
        base = order_d.cpu().numpy()
        moves = workloads.window_moves(np.random.default_rng(4), K, 0, min(n, window))
        base_line = cpu_baseline_rows(inst, lambda lo, hi: workloads.orders_from_moves(base, moves[lo:hi]), K, log1[0]["tel"],
                                      "moves of the first window")
        if base_line is None:
            print("bench.py: GPU and oracle disagree on the sampled moves", file=sys.stderr)
            return 1
        result["cpu_baseline"] = base_line
    print(json.dumps(result))
    ctx.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cpu-rows", type=int, default=128, help="candidate rows the CPU oracle is timed on (--workload predicted)")
    ap.add_argument("--phase1", choices=("sorted_prefix", "local_swap"), default="sorted_prefix",
                    help="Phase-1 solver run inside the step (the candidate set is always built around the sorted-prefix order)")
    ap.add_argument("--workload", choices=("config1", "config2", "config3", "config4", "config5", "online", "predicted",
                                           "phase1"), default="config3",
                    help="config3: the headline workload; config1 / config2 / config5: the same step on those "
                         "configurations; config4: the receding-horizon run (65536 moves per 512-window); online: the paper's Poisson-arrival experiment "
                         "(Section 7) as a batch of independent streams through kvsched_online; predicted: the "
                         "config-3 candidates run under interval predictions of the decode lengths "
                         "(kvsched_simulate_predicted, estimates started from the lower bounds); phase1: the "
                         "Phase-1 constructions (sorted prefix, Local Swap Search, exact batches) on configs 3, 4, 5")
    ap.add_argument("--decode-scale", type=int, default=1,
                    help="configs 1, 2, 3, 5: multiply decode lengths (capped at 14336) and the budget by this factor")
    ap.add_argument("--gamma", type=float, default=0.6, help="prediction confidence inf l_i / u_i of --workload predicted")
    ap.add_argument("--online-seeds", type=int, default=200,
                    help="arrival sequences per load level of the online workload (10 loads x 3 policies each)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy, the yardstick for FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: libkvsched evaluates schedules on ONE GPU; --gpus must be 1 "
              "(candidates are independent and would shard across GPUs; that is not built)", file=sys.stderr)
        return 2

    import torch

    from paper_2508_06133_amd import kvsched, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libkvsched has no CPU path", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ctx = kvsched.Context(0)
    if args.workload == "online":
        return bench_online(args, ctx, dev)
    if args.workload == "phase1":
        return bench_phase1(args, ctx, dev)
    if args.workload == "predicted":
        return bench_predicted(args, ctx, dev)

    if args.workload == "config4":
        return bench_horizon(args, ctx, dev)
    return bench_rows(args, ctx, dev, int(args.workload[-1]))


if __name__ == "__main__":
    sys.exit(main())
