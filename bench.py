#!/usr/bin/env python3
"""Benchmark of the schedule-evaluation hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input, everything already
resident in HBM: Sorted-F order construction (Phase 1), evaluation of the C candidate orders
(Phase 2: timelines, total latency and completion rounds per candidate), argmin over the
candidates.  Workload: configuration 3 ("mixed chat + summarisation": n = 2000 requests,
M = 131072 tokens, C = 16384 candidates = Sorted-F order, 16127 distinct 1-swap neighbours,
256 random restarts).

Prints ONE JSON line:  candidate schedules evaluated per second, the roofline object of the
dominant kernel (integer-VALU bound; algorithmic lane-ops from the outputs of the run) and the
CPU oracle timed on the same rows on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Peak plain-ALU rate of the chip: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one int32 op per
# lane per clock (the fp32 vector peak of 157.3 TFLOP/s counts an FMA as two and packs two).
PEAK_INT32_LANE_OPS = 256 * 4 * 16 * 2.4e9
PEAK_HBM_BYTES = 8.0e12
OPS_PER_VISIT = 6  # int32 lane-ops to inspect or update one future round for one request
CFG = 3

# HBM traffic of the dominant kernel per launch (one per step) on this workload, from rocprofv3
# counters (profiles/timeline_kernel_config3_traffic.md): FETCH_SIZE 46963 KiB x 1.9997 (what a
# plain 256 MiB copy reads per KiB moved) + WRITE_SIZE 89485 KiB x 1.0.  Valid only for the kernel
# sources it was measured on; reported as null once they change.
TRAFFIC_BYTES = int((46963 * 1.9997 + 89485 * 1.0) * 1024)
TRAFFIC_SOURCES = ("timeline_reg.hip", "device_util.h")
TRAFFIC_SOURCES_SHA256 = "35d75c7b25cb13ed"


# Issue slots the same kernel really used on this workload (profiles/timeline_kernel_config3_counters.md):
# SQ_INSTS_VALU 1.185e9 x 4 cycles / (1024 SIMDs x 4.94e6 cycles) and (SQ_INSTS_SALU 8.763e8 +
# SQ_INSTS_BRANCH 2.252e8) / (256 scalar units x 4.94e6 cycles), cycles from GRBM_GUI_ACTIVE / 8 XCDs.
# The accounting above credits 6 lane-ops per visit where the kernel issues 4.9, so the physical
# utilisation is this, not roofline.frac.
ISSUE_SLOTS = {"valu": 0.937, "scalar_and_branch": 0.871}


def _kernel_sources_unchanged() -> bool:
    import hashlib

    h = hashlib.sha256()
    for f in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, "paper_2508_06133_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16] == TRAFFIC_SOURCES_SHA256


def measured_traffic():
    return TRAFFIC_BYTES if _kernel_sources_unchanged() else None


def measured_issue_slots():
    return ISSUE_SLOTS if _kernel_sources_unchanged() else None


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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cpu-rows", type=int, default=16384, help="candidate rows the CPU oracle is timed on")
    ap.add_argument("--phase1", choices=("sorted_prefix", "local_swap"), default="sorted_prefix",
                    help="Phase-1 solver run inside the step (the candidate set is always built around the sorted-prefix order)")
    ap.add_argument("--workload", choices=("config3", "online", "predicted", "phase1"), default="config3",
                    help="config3: the headline workload; online: the paper's Poisson-arrival experiment "
                         "(Section 7) as a batch of independent streams through kvsched_online; predicted: the "
                         "config-3 candidates run under interval predictions of the decode lengths "
                         "(kvsched_simulate_predicted, estimates started from the lower bounds); phase1: the "
                         "Phase-1 constructions (sorted prefix, Local Swap Search, exact batches) on configs 3, 4, 5")
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

    inst = workloads.instance(CFG)
    n, M = inst.n, inst.M
    s = torch.from_numpy(inst.s).to(dev)
    o = torch.from_numpy(inst.o).to(dev)

    # The candidate set is built around the Sorted-F order; that order comes from the library.
    order_d, ends_d, F_d, nb_d = ctx.sortedF(s, o, M)
    torch.cuda.synchronize()
    base = order_d.cpu().numpy()
    rows_h = workloads.candidates(CFG, base)
    C = rows_h.shape[0]
    orders = torch.from_numpy(rows_h).to(dev)
    tel = torch.empty(C, dtype=torch.int64, device=dev)
    comp = torch.empty((C, n), dtype=torch.int32, device=dev)
    best = torch.empty(2, dtype=torch.int64, device=dev)

    p1_out = (order_d, ends_d, F_d, nb_d)  # Phase 1 writes into the same tensors every step
    ctx.set_o_max(int(inst.o.max()))  # the caller's bound on decode lengths: no read-back inside the step

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
    ms_per_step = wall * 1e3 / args.steps
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
    visits = int(((p_last - t_res) + 2 * (sum_o - cum0[resume])).sum().item())
    visits_from_scratch = int((p_last + 2 * sum_o).sum().item())
    lane_ops = OPS_PER_VISIT * visits
    k_ms = float(np.mean(kernel_ms))
    achieved = lane_ops / (k_ms * 1e-3)
    hbm_bytes = int((8 * (n - resume) + 8).sum().item()) + 8 * n  # order entries read, completion rounds written, from the resume point on
    result = {
        "metric": "candidate schedules evaluated/s (n=2000 mixed)",
        "value": C * args.steps / wall,
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": "config 3: mixed chat+summarization, n=2000, M=131072, C=16384 "
                               "(Sorted-F order + 16127 1-swap neighbours + 256 random restarts)",
                   "n": n, "M": M, "C": C, "sortedF_batches": int(nb_d.item()), "phase1": args.phase1},
        "request_rounds_per_s": C * sum_o * args.steps / wall,
        "gpu_ms_per_step": gpu_ms / args.steps,
        "timeline_kernel_ms": k_ms,
        "best_candidate": {"index": int(best[0].item()), "tel": int(best[1].item()), "base_tel": int(tel_h[0])},
        "roofline": {
            "bound": "alu",
            "kernel": "timeline_reg_kernel<33,4,false,true,true>",
            "launches_per_step": 1,  # row 0 saves its state every 64 positions; the rows that share them wait for theirs
            "resumed_rows": int((resume > 0).sum().item()),
            "visits_without_resume": visits_from_scratch,
            "achieved": achieved / 1e12,
            "peak": PEAK_INT32_LANE_OPS / 1e12,
            "unit": "Tlane-op/s (int32)",
            "frac": achieved / PEAK_INT32_LANE_OPS,
            "traffic": measured_traffic(),
            "issue_slots_measured": measured_issue_slots(),
            "visits_per_step": visits,  # from each row's resume point on
            "ops_per_visit": OPS_PER_VISIT,
            "hbm": {"algorithmic_bytes": hbm_bytes, "achieved_GBps": hbm_bytes / (k_ms * 1e-3) / 1e9,
                    "frac_of_8TBps": hbm_bytes / (k_ms * 1e-3) / PEAK_HBM_BYTES},
        },
    }

    if not args.no_cpu_baseline:
        import oracle  # test infrastructure; only this baseline leg uses it

        rows_cpu = rows_h[: max(1, min(args.cpu_rows, C))]
        t0 = time.perf_counter()
        tel_o, _ = oracle.simulate_many(inst.s, inst.o, M, rows_cpu, literal=False, completions=True)
        cpu_s = time.perf_counter() - t0
        if not (tel_o == tel_h[: rows_cpu.shape[0]]).all():
            print("bench.py: GPU and oracle disagree on the sampled rows", file=sys.stderr)
            return 1
        result["cpu_baseline"] = {
            "value": rows_cpu.shape[0] / cpu_s,
            "unit": "candidates/s",
            "cores": 1,
            "kind": "oracle",
            "sample": f"first {rows_cpu.shape[0]} of the {C} candidate rows, array-profile oracle "
                      f"(oracle_simulate_profile), single thread, {cpu_s:.1f} s",
        }
    print(json.dumps(result))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
