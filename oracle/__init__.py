"""CPU oracle for the schedule-evaluation path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, single-threaded reference written from the paper.  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may import this package; the GPU
library and its Python binding never do, and share no code with it.

  kvsched_oracle.c : Phase 2 of Algorithm 1 (literal and array-profile forms), sorted-prefix
                     Phase 1 with the F-metric, Phase 1 with Local Swap Search, Phase 1 with exact
                     batches (Algorithm 2), the same under the G metric, position moves, best neighbour,
                     Phase 2 under predicted decode lengths (running estimates, ordered eviction).
  online_oracle.c  : scheduling under online arrivals (cached priority list, refresh triggers,
                     look-ahead window; FCFS / shortest-decode-first / footprint / Sorted-F-Online).
  exact.py         : Algorithm 2 (exact DP), subset / permutation / start-time brute force,
                     lower bound -- tiny instances only.
  check.py         : direct-definition schedule checker (memory per round, greedy-earliest).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "kvsched_oracle.c"), os.path.join(_HERE, "online_oracle.c")]
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (a second or so)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", *_SRCS, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f64p = ctypes.POINTER(ctypes.c_double)


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a, typ):
    return a.ctypes.data_as(typ) if a is not None else None


class OracleError(ValueError):
    pass


def _check(rc):
    if rc != 0:
        raise OracleError(f"oracle rejected the input (code {rc})")


def check_instance(s, o, M) -> bool:
    s, o = _i32(s), _i32(o)
    return _load().oracle_check_instance(ctypes.c_int32(len(s)), _ptr(s, _i32p), _ptr(o, _i32p), ctypes.c_int64(int(M))) == 0


def simulate(s, o, M, order, literal: bool = True):
    """One order -> (start rounds p[n], completion rounds c[n], TEL); indexed by request id."""
    s, o, order = _i32(s), _i32(o), _i32(order)
    n = len(s)
    if len(o) != n or len(order) != n:
        raise OracleError("length mismatch")
    p = np.zeros(n, dtype=np.int32)
    c = np.zeros(n, dtype=np.int32)
    tel = ctypes.c_int64(0)
    fn = _load().oracle_simulate_literal if literal else _load().oracle_simulate_profile
    _check(fn(ctypes.c_int32(n), _ptr(s, _i32p), _ptr(o, _i32p), ctypes.c_int64(int(M)), _ptr(order, _i32p),
              _ptr(p, _i32p), _ptr(c, _i32p), ctypes.byref(tel)))
    return p, c, int(tel.value)


def simulate_many(s, o, M, orders, literal: bool = False, completions: bool = True):
    """Rows of `orders` [C, n] -> (tel[C] int64, completion[C, n] int32 or None)."""
    s, o, orders = _i32(s), _i32(o), _i32(orders)
    C, n = orders.shape
    if len(s) != n or len(o) != n:
        raise OracleError("length mismatch")
    tel = np.zeros(C, dtype=np.int64)
    comp = np.zeros((C, n), dtype=np.int32) if completions else None
    _check(_load().oracle_simulate_many(ctypes.c_int32(n), _ptr(s, _i32p), _ptr(o, _i32p), ctypes.c_int64(int(M)),
                                        _ptr(orders, _i32p), ctypes.c_int32(C), ctypes.c_int32(1 if literal else 0),
                                        _ptr(tel, _i64p), _ptr(comp, _i32p)))
    return tel, comp


def sortedF(s, o, M, tie_rule: int = 0, feas_mode: int = 0, alpha=(0, 1)):
    """-> (order[n], batch_end[num_batches], F[num_batches]).  feas_mode as exact_phase1.
    alpha = (a, b): the metric is G = sum (a s_i + b o_i) / (b |X|^2); (0, 1) is the F-metric."""
    s, o = _i32(s), _i32(o)
    n = len(s)
    order = np.zeros(n, dtype=np.int32)
    ends = np.zeros(max(n, 1), dtype=np.int32)
    F = np.zeros(max(n, 1), dtype=np.float64)
    nb = ctypes.c_int32(0)
    _check(_load().oracle_sortedG(ctypes.c_int32(n), _ptr(s, _i32p), _ptr(o, _i32p), ctypes.c_int64(int(M)),
                                  ctypes.c_int32(int(alpha[0])), ctypes.c_int32(int(alpha[1])),
                                  ctypes.c_int32(tie_rule), ctypes.c_int32(feas_mode), _ptr(order, _i32p),
                                  _ptr(ends, _i32p), _ptr(F, _f64p), ctypes.byref(nb)))
    return order, ends[: nb.value].copy(), F[: nb.value].copy()


def local_swap(s, o, M, early_exit: bool = False, alpha=(0, 1)):
    """Phase 1 with Local Swap Search -> (order[n], batch_end[nb], F[nb], swaps[nb]).  alpha as sortedF."""
    s, o = _i32(s), _i32(o)
    n = len(s)
    order = np.zeros(n, dtype=np.int32)
    ends = np.zeros(max(n, 1), dtype=np.int32)
    F = np.zeros(max(n, 1), dtype=np.float64)
    swaps = np.zeros(max(n, 1), dtype=np.int32)
    nb = ctypes.c_int32(0)
    _check(_load().oracle_local_swap_G(ctypes.c_int32(n), _ptr(s, _i32p), _ptr(o, _i32p), ctypes.c_int64(int(M)),
                                     ctypes.c_int32(int(alpha[0])), ctypes.c_int32(int(alpha[1])),
                                     ctypes.c_int32(1 if early_exit else 0), _ptr(order, _i32p), _ptr(ends, _i32p),
                                     _ptr(F, _f64p), _ptr(swaps, _i32p), ctypes.byref(nb)))
    return order, ends[: nb.value].copy(), F[: nb.value].copy(), swaps[: nb.value].copy()


def exact_phase1(s, o, M, feas_mode: int = 0, tie_rule: int = 0, alpha=(0, 1)):
    """Phase 1 with exact batches (Algorithm 2) -> (order[n], batch_end[nb], F[nb]).
    feas_mode 0: sum of peaks <= M; 1: simultaneous-start memory profile <= M.  alpha as sortedF."""
    s, o = _i32(s), _i32(o)
    n = len(s)
    order = np.zeros(n, dtype=np.int32)
    ends = np.zeros(max(n, 1), dtype=np.int32)
    F = np.zeros(max(n, 1), dtype=np.float64)
    nb = ctypes.c_int32(0)
    _check(_load().oracle_exact_phase1_G(ctypes.c_int32(n), _ptr(s, _i32p), _ptr(o, _i32p), ctypes.c_int64(int(M)),
                                       ctypes.c_int32(int(alpha[0])), ctypes.c_int32(int(alpha[1])),
                                       ctypes.c_int32(feas_mode), ctypes.c_int32(tie_rule), _ptr(order, _i32p),
                                       _ptr(ends, _i32p), _ptr(F, _f64p), ctypes.byref(nb)))
    return order, ends[: nb.value].copy(), F[: nb.value].copy()


def apply_move(base, move):
    base = _i32(base)
    out = np.zeros_like(base)
    _check(_load().oracle_apply_move(ctypes.c_int32(len(base)), _ptr(base, _i32p), ctypes.c_int32(int(move[0])),
                                     ctypes.c_int32(int(move[1])), ctypes.c_int32(int(move[2])), _ptr(out, _i32p)))
    return out


def best_neighbor(s, o, M, base, moves, literal: bool = False):
    """-> (tel[K], (best_move_index, best_tel, base_tel)); ties -> lowest move index."""
    s, o, base = _i32(s), _i32(o), _i32(base)
    moves = _i32(moves).reshape(-1, 3)
    K = moves.shape[0]
    tel = np.zeros(K, dtype=np.int64)
    res = np.zeros(3, dtype=np.int64)
    _check(_load().oracle_best_neighbor(ctypes.c_int32(len(s)), _ptr(s, _i32p), _ptr(o, _i32p), ctypes.c_int64(int(M)),
                                        _ptr(base, _i32p), _ptr(moves, _i32p), ctypes.c_int32(K),
                                        ctypes.c_int32(1 if literal else 0), _ptr(tel, _i64p), _ptr(res, _i64p)))
    return tel, (int(res[0]), int(res[1]), int(res[2]))


def simulate_predicted(s, o, est0, M, order, literal: bool = False, max_runs: int = 0):
    """Phase 2 under predicted decode lengths (running estimates, ordered eviction).
    -> (p[n], c[n], TEL, evictions[n], runs[k, 4] = {request, start, end, 0 completed | 1 stopped})."""
    s, o, est0, order = _i32(s), _i32(o), _i32(est0), _i32(order)
    n = len(s)
    if len(o) != n or len(est0) != n or len(order) != n:
        raise OracleError("length mismatch")
    p = np.zeros(n, dtype=np.int32)
    c = np.zeros(n, dtype=np.int32)
    ev = np.zeros(n, dtype=np.int32)
    runs = np.zeros((max(max_runs, 1), 4), dtype=np.int32)
    tel = ctypes.c_int64(0)
    nr = ctypes.c_int32(0)
    _check(_load().oracle_simulate_predicted(ctypes.c_int32(n), _ptr(s, _i32p), _ptr(o, _i32p), _ptr(est0, _i32p),
                                             ctypes.c_int64(int(M)), _ptr(order, _i32p),
                                             ctypes.c_int32(1 if literal else 0), _ptr(p, _i32p), _ptr(c, _i32p),
                                             ctypes.byref(tel), _ptr(ev, _i32p), _ptr(runs, _i32p) if max_runs else None,
                                             ctypes.c_int32(max_runs), ctypes.byref(nr)))
    if max_runs and nr.value > max_runs:
        raise OracleError("run log too small")
    return p, c, int(tel.value), ev, runs[: nr.value].copy() if max_runs else None


PLANNER_ARRIVAL, PLANNER_SHORTEST_DECODE, PLANNER_FOOTPRINT, PLANNER_SORTED_F = 0, 1, 2, 3


def online(a, s, o, M, planner: int, period: int = 10, window: int = 300, refresh=(1, 2), literal: bool = False):
    """Scheduling under online arrivals (a[] nondecreasing) -> (p[n], c[n], stats) with
    stats = (sum of c_i - a_i, refreshes of the cached order, last completion round, largest backlog).
    refresh = (num, den): early refresh once the waiting newcomers reach num/den of the backlog
    at the last refresh; den = 0 switches that trigger off."""
    a, s, o = _i32(a), _i32(s), _i32(o)
    n = len(s)
    if len(o) != n or len(a) != n:
        raise OracleError("length mismatch")
    p = np.zeros(n, dtype=np.int32)
    c = np.zeros(n, dtype=np.int32)
    stats = np.zeros(4, dtype=np.int64)
    _check(_load().oracle_online(ctypes.c_int32(n), _ptr(a, _i32p), _ptr(s, _i32p), _ptr(o, _i32p),
                                 ctypes.c_int64(int(M)), ctypes.c_int32(planner), ctypes.c_int32(period),
                                 ctypes.c_int32(window), ctypes.c_int32(int(refresh[0])), ctypes.c_int32(int(refresh[1])),
                                 ctypes.c_int32(1 if literal else 0), _ptr(p, _i32p), _ptr(c, _i32p), _ptr(stats, _i64p)))
    return p, c, tuple(int(x) for x in stats)
