"""ctypes binding over libkvsched.so -- argument marshalling only.

Same names as the C ABI (see include/kvsched.h).  Inputs and outputs are torch tensors on
the context's GPU; torch is used for device memory and the current stream, nothing else.
Importing this module loads the shared library and raises if it has not been built:
there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

OK = 0
TIE_LARGER, TIE_SMALLER = 0, 1
MOVE_SWAP, MOVE_INSERT = 0, 1
DEV_BAD_LENGTH, DEV_BAD_ORDER, DEV_BAD_MOVE, DEV_O_MAX = 1, 2, 4, 8
DEV_BAD_ARRIVAL, DEV_BACKLOG, DEV_BAD_STREAM, DEV_ROUND_LIMIT = 16, 32, 64, 128
PLANNER_ARRIVAL, PLANNER_SHORTEST_DECODE, PLANNER_FOOTPRINT, PLANNER_SORTED_F = 0, 1, 2, 3
ONLINE_MAX_BACKLOG, ONLINE_MAX_WINDOW, ONLINE_MAX_O = 4096, 1024, 8192
FEAS_SUM_OF_PEAKS, FEAS_PROFILE = 0, 1
EXACT_MAX_N = 4096
SOLVER_SORTED_PREFIX, SOLVER_LOCAL_SWAP, SOLVER_EXACT_DP = 0, 1, 2
RESUME_AUTO = -1


class KvschedError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what} failed: {code} ({strerror(code)})")
        self.code = code


def _load() -> ctypes.CDLL:
    path = _build.lib_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_2508_06133_amd.build` "
            "(hipcc, gfx950); libkvsched has no CPU fallback"
        )
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.kvsched_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.kvsched_destroy.argtypes = [vp]
    lib.kvsched_destroy.restype = None
    lib.kvsched_strerror.argtypes = [ctypes.c_int]
    lib.kvsched_strerror.restype = ctypes.c_char_p
    lib.kvsched_set_o_max.argtypes = [vp, i32]
    lib.kvsched_reserve.argtypes = [vp, i32, i32, i32]
    lib.kvsched_device_status.argtypes = [vp, vp, ctypes.POINTER(i32)]
    lib.kvsched_enable_timing.argtypes = [vp, ctypes.c_int]
    lib.kvsched_last_timeline_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.kvsched_argmin.argtypes = [vp, vp, i32, vp, vp]
    lib.kvsched_simulate.argtypes = [vp, vp, i32, i32, vp, vp, i64, vp, vp, i32, vp]
    lib.kvsched_simulate_resume_positions.argtypes = [vp, i32, vp, vp]
    lib.kvsched_simulate_stop_positions.argtypes = [vp, i32, i32, vp, vp]
    lib.kvsched_neighbor_stop_positions.argtypes = [vp, i32, i32, vp, vp]
    lib.kvsched_set_resume_min_rows.argtypes = [vp, i32]
    lib.kvsched_set_resume_one_launch.argtypes = [vp, i32]
    lib.kvsched_sortedF.argtypes = [vp, i32, vp, vp, i64, i32, i32, vp, vp, vp, vp, vp]
    lib.kvsched_local_swap.argtypes = [vp, i32, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.kvsched_exact_dp.argtypes = [vp, i32, vp, vp, i64, i32, i32, vp, vp, vp, vp, vp]
    lib.kvsched_simulate_predicted.argtypes = [vp, vp, i32, i32, vp, vp, vp, i32, i64, vp, vp, vp, vp]
    lib.kvsched_phase1_G.argtypes = [vp, i32, i32, vp, vp, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.kvsched_best_neighbor.argtypes = [vp, vp, i32, vp, i32, vp, vp, i64, vp, vp, vp]
    lib.kvsched_best_neighbor_static.argtypes = [vp, vp, i32, vp, i32, vp, vp, i64, i32, vp, vp, vp]
    lib.kvsched_horizon_step.argtypes = [vp, vp, i32, vp, i32, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.kvsched_online.argtypes = [vp, i32, vp, i32, vp, vp, vp, i64, i32, vp, i32, vp, vp]
    return lib


_lib = _load()


def strerror(code: int) -> str:
    return _lib.kvsched_strerror(int(code)).decode()


def _dev(t: torch.Tensor, dtype, what: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what}: expected a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Context:
    """Owns a kvsched_ctx on one device; methods mirror the C entry points."""

    def __init__(self, device: int = 0):
        self._h = ctypes.c_void_p()
        self.device = int(device)
        rc = _lib.kvsched_create(ctypes.byref(self._h), self.device)
        if rc != OK:
            raise KvschedError(rc, "kvsched_create")

    def close(self):
        if getattr(self, "_h", None) and self._h.value and _lib is not None:
            _lib.kvsched_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):  # at interpreter exit the module globals may already be gone
        try:
            self.close()
        except Exception:
            pass

    def reserve(self, rows: int, n: int, moves: int = 0):
        """Size the context's scratch once for calls of up to `rows` rows / `moves` moves of `n` positions."""
        rc = _lib.kvsched_reserve(self._h, int(rows), int(n), int(moves))
        if rc != OK:
            raise KvschedError(rc, "kvsched_reserve")

    def set_o_max(self, bound: int):
        rc = _lib.kvsched_set_o_max(self._h, int(bound))
        if rc != OK:
            raise KvschedError(rc, "kvsched_set_o_max")

    def enable_timing(self, on: bool = True):
        rc = _lib.kvsched_enable_timing(self._h, 1 if on else 0)
        if rc != OK:
            raise KvschedError(rc, "kvsched_enable_timing")

    def last_timeline_ms(self) -> float:
        out = ctypes.c_float(0.0)
        rc = _lib.kvsched_last_timeline_ms(self._h, ctypes.byref(out))
        if rc != OK:
            raise KvschedError(rc, "kvsched_last_timeline_ms")
        return float(out.value)

    def argmin(self, tel, result_out=None):
        """tel [C] int64 -> result [2] int64 = {index of the least valid entry, its value}."""
        res = torch.empty(2, dtype=torch.int64, device=tel.device) if result_out is None else result_out
        rc = _lib.kvsched_argmin(self._h, _dev(tel, torch.int64, "tel"), tel.shape[0], _dev(res, torch.int64, "result"),
                                 _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_argmin")
        return res

    def device_status(self) -> int:
        out = ctypes.c_int32(0)
        rc = _lib.kvsched_device_status(self._h, _stream(), ctypes.byref(out))
        if rc != OK:
            raise KvschedError(rc, "kvsched_device_status")
        return int(out.value)

    def simulate(self, orders, s, o, M, completions: bool = True, common_prefix: int = 0, tel_out=None,
                 completion_out=None):
        """orders [C, n] -> (tel [C] int64, completion [C, n] int32 by request id or None)."""
        C, n = orders.shape
        dev = orders.device
        tel = torch.empty(C, dtype=torch.int64, device=dev) if tel_out is None else tel_out
        comp = None
        if completions:
            comp = torch.empty((C, n), dtype=torch.int32, device=dev) if completion_out is None else completion_out
        rc = _lib.kvsched_simulate(self._h, _dev(orders, torch.int32, "orders"), C, n, _dev(s, torch.int32, "s"),
                                   _dev(o, torch.int32, "o"), int(M), _dev(tel, torch.int64, "tel_out"),
                                   _dev(comp, torch.int32, "completion_out") if comp is not None else None,
                                   int(common_prefix), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_simulate")
        return tel, comp

    def set_resume_one_launch(self, wait_polls: int):
        rc = _lib.kvsched_set_resume_one_launch(self._h, int(wait_polls))
        if rc != 0:
            raise KvschedError(rc, "kvsched_set_resume_one_launch")

    def set_resume_min_rows(self, rows: int):
        rc = _lib.kvsched_set_resume_min_rows(self._h, int(rows))
        if rc != OK:
            raise KvschedError(rc, "kvsched_set_resume_min_rows")

    def simulate_resume_positions(self, C: int, device="cuda:0"):
        """-> [C] int32: position from which each row of the last simulate() call was placed."""
        out = torch.empty(int(C), dtype=torch.int32, device=device)
        rc = _lib.kvsched_simulate_resume_positions(self._h, int(C), out.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_simulate_resume_positions")
        return out

    def simulate_stop_positions(self, C: int, n: int, device="cuda:0"):
        """-> [C] int32: position before which each row of the last simulate() call stopped placing
        (n: it placed its last position itself)."""
        out = torch.empty(int(C), dtype=torch.int32, device=device)
        rc = _lib.kvsched_simulate_stop_positions(self._h, int(C), int(n), out.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_simulate_stop_positions")
        return out

    def neighbor_stop_positions(self, K: int, n: int, device="cuda:0"):
        """-> [K] int32: position before which the timeline of each move of the last best_neighbor() /
        horizon_step() call stopped being placed (n: placed to its end, 0: not placed at all)."""
        out = torch.empty(int(K), dtype=torch.int32, device=device)
        rc = _lib.kvsched_neighbor_stop_positions(self._h, int(K), int(n), out.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_neighbor_stop_positions")
        return out

    def sortedF(self, s, o, M, tie_rule: int = TIE_LARGER, feas_mode: int = FEAS_SUM_OF_PEAKS, out=None):
        """-> (order [n] int32, batch_end [n] int32, F [n] float64, num_batches [1] int32); the first
        num_batches entries of batch_end / F are meaningful.  out: the four tensors to write into
        (a caller in a loop keeps them; otherwise they are allocated, batch_end and F zero-filled)."""
        n = s.shape[0]
        dev = s.device
        if out is None:
            order = torch.empty(n, dtype=torch.int32, device=dev)
            ends = torch.zeros(n, dtype=torch.int32, device=dev)
            F = torch.zeros(n, dtype=torch.float64, device=dev)
            nb = torch.zeros(1, dtype=torch.int32, device=dev)
        else:
            order, ends, F, nb = out
            _dev(order, torch.int32, "order"), _dev(ends, torch.int32, "batch_end")
            _dev(F, torch.float64, "F"), _dev(nb, torch.int32, "num_batches")
            if order.shape[0] < n or ends.shape[0] < n or F.shape[0] < n or nb.shape[0] < 1:
                raise ValueError("sortedF: output tensors too short")
        rc = _lib.kvsched_sortedF(self._h, n, _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"), int(M),
                                  int(tie_rule), int(feas_mode), order.data_ptr(), ends.data_ptr(), F.data_ptr(),
                                  nb.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_sortedF")
        return order, ends, F, nb

    def local_swap(self, s, o, M):
        """Phase 1 with Local Swap Search -> (order [n], batch_end [n], F [n], swaps [n], num_batches [1])."""
        n = s.shape[0]
        dev = s.device
        order = torch.empty(n, dtype=torch.int32, device=dev)
        ends = torch.zeros(n, dtype=torch.int32, device=dev)
        F = torch.zeros(n, dtype=torch.float64, device=dev)
        swaps = torch.zeros(n, dtype=torch.int32, device=dev)
        nb = torch.zeros(1, dtype=torch.int32, device=dev)
        rc = _lib.kvsched_local_swap(self._h, n, _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"), int(M),
                                     order.data_ptr(), ends.data_ptr(), F.data_ptr(), swaps.data_ptr(),
                                     nb.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_local_swap")
        return order, ends, F, swaps, nb

    def exact_dp(self, s, o, M, feas_mode: int = FEAS_SUM_OF_PEAKS, tie_rule: int = TIE_LARGER):
        """Phase 1 with exact batches (Algorithm 2) -> (order [n], batch_end [n], F [n], num_batches [1])."""
        n = s.shape[0]
        dev = s.device
        order = torch.empty(n, dtype=torch.int32, device=dev)
        ends = torch.zeros(n, dtype=torch.int32, device=dev)
        F = torch.zeros(n, dtype=torch.float64, device=dev)
        nb = torch.zeros(1, dtype=torch.int32, device=dev)
        rc = _lib.kvsched_exact_dp(self._h, n, _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"), int(M),
                                   int(feas_mode), int(tie_rule), order.data_ptr(), ends.data_ptr(), F.data_ptr(),
                                   nb.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_exact_dp")
        return order, ends, F, nb

    def simulate_predicted(self, orders, s, o, est0, M, completions: bool = True):
        """Phase 2 under predicted decode lengths.  orders [C, n]; est0 [n] or [C, n] initial estimates
        -> (tel [C] int64, completion [C, n] int32 or None, evictions [C] int32)."""
        C, n = orders.shape
        dev = orders.device
        E = 1 if est0.dim() == 1 else est0.shape[0]
        tel = torch.empty(C, dtype=torch.int64, device=dev)
        comp = torch.empty((C, n), dtype=torch.int32, device=dev) if completions else None
        ev = torch.empty(C, dtype=torch.int32, device=dev)
        rc = _lib.kvsched_simulate_predicted(self._h, _dev(orders, torch.int32, "orders"), C, n,
                                             _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"),
                                             _dev(est0, torch.int32, "est0"), E, int(M), tel.data_ptr(),
                                             comp.data_ptr() if comp is not None else None, ev.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_simulate_predicted")
        return tel, comp, ev

    def phase1_G(self, solver: int, s, o, M, alpha, tie_rule: int = TIE_LARGER, feas_mode: int = FEAS_SUM_OF_PEAKS):
        """Phase 1 under G = sum (alpha s + o) / |X|^2, alpha = (num, den)
        -> (order [n], batch_end [n], G [n], swaps [n], num_batches [1])."""
        n = s.shape[0]
        dev = s.device
        order = torch.empty(n, dtype=torch.int32, device=dev)
        ends = torch.zeros(n, dtype=torch.int32, device=dev)
        G = torch.zeros(n, dtype=torch.float64, device=dev)
        swaps = torch.zeros(n, dtype=torch.int32, device=dev)
        nb = torch.zeros(1, dtype=torch.int32, device=dev)
        rc = _lib.kvsched_phase1_G(self._h, int(solver), n, _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"), int(M),
                                   int(alpha[0]), int(alpha[1]), int(tie_rule), int(feas_mode), order.data_ptr(),
                                   ends.data_ptr(), G.data_ptr(), swaps.data_ptr(), nb.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_phase1_G")
        return order, ends, G, swaps, nb

    def best_neighbor(self, base_order, moves, s, o, M, want_tel: bool = True):
        """-> (tel [K] int64 or None, result [3] int64 = {best move, its TEL, TEL of base})."""
        n = base_order.shape[0]
        K = moves.shape[0]
        dev = base_order.device
        tel = torch.empty(K, dtype=torch.int64, device=dev) if want_tel else None
        res = torch.empty(3, dtype=torch.int64, device=dev)
        rc = _lib.kvsched_best_neighbor(self._h, _dev(base_order, torch.int32, "base_order"), n,
                                        _dev(moves, torch.int32, "moves"), K, _dev(s, torch.int32, "s"),
                                        _dev(o, torch.int32, "o"), int(M),
                                        tel.data_ptr() if tel is not None else None, res.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_best_neighbor")
        return tel, res

    def best_neighbor_static(self, base_order, moves, s, o, M, o_max_bound: int, tel_out, result_out):
        """kvsched_best_neighbor on the library's fixed working array: the caller passes every output
        tensor (tel_out [K] int64 or None, result_out [3] int64); nothing is allocated."""
        rc = _lib.kvsched_best_neighbor_static(self._h, _dev(base_order, torch.int32, "base_order"),
                                               base_order.shape[0], _dev(moves, torch.int32, "moves"), moves.shape[0],
                                               _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"), int(M),
                                               int(o_max_bound),
                                               _dev(tel_out, torch.int64, "tel_out") if tel_out is not None else None,
                                               _dev(result_out, torch.int64, "result_out"), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_best_neighbor_static")
        return tel_out, result_out

    def horizon_step(self, order, moves, s, o, M, completed_in: int, complete_every: int, want_tel: bool = False,
                     completion_out=None):
        """One re-planning step; `order` [n] is updated in place.
        -> (tel [K] or None, result [6] int64 = {best move, its TEL, TEL before, committed positions,
        requests completed by T, T})."""
        n = order.shape[0]
        K = moves.shape[0]
        dev = order.device
        tel = torch.empty(K, dtype=torch.int64, device=dev) if want_tel else None
        res = torch.empty(6, dtype=torch.int64, device=dev)
        rc = _lib.kvsched_horizon_step(self._h, _dev(order, torch.int32, "order"), n, _dev(moves, torch.int32, "moves"),
                                       K, _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"), int(M),
                                       int(completed_in), int(complete_every),
                                       tel.data_ptr() if tel is not None else None,
                                       _dev(completion_out, torch.int32, "completion_out")
                                       if completion_out is not None else None,
                                       res.data_ptr(), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_horizon_step")
        return tel, res

    def online(self, streams, a, s, o, M, completion_out, stats_out=None, backlog_cap: int = ONLINE_MAX_BACKLOG):
        """streams [B, 8] int32 descriptors {first request, count, planner, period, window,
        refresh_num, refresh_den, first output slot}; a, s, o [N] int32; completion_out [out_len]
        int32 is the tensor the descriptors' output slots refer to; backlog_cap bounds the requests
        of one stream that may wait at once (smaller bounds let more streams run side by side).
        -> (completion_out, stats [B, 4] int64 = {sum of c_i - a_i, refreshes, last completion
        round, largest backlog})."""
        B = streams.shape[0]
        stats = torch.empty((B, 4), dtype=torch.int64, device=a.device) if stats_out is None else stats_out
        rc = _lib.kvsched_online(self._h, B, _dev(streams, torch.int32, "streams"), a.shape[0],
                                 _dev(a, torch.int32, "a"), _dev(s, torch.int32, "s"), _dev(o, torch.int32, "o"),
                                 int(M), int(backlog_cap), _dev(completion_out, torch.int32, "completion_out"),
                                 completion_out.shape[0],
                                 _dev(stats, torch.int64, "stats_out"), _stream())
        if rc != OK:
            raise KvschedError(rc, "kvsched_online")
        return completion_out, stats
