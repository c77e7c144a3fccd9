"""Receding-horizon driver over libkvsched (offline form: every request present at round 0).

The loop only draws the window's moves and reads back six numbers per re-plan; the planning,
the move, the timeline and the commit point are computed by kvsched_horizon_step on the GPU.
"""
from __future__ import annotations

import numpy as np
import torch

from . import workloads


def receding_horizon(ctx, s, o, M, base_order, window: int = 512, complete_every: int = 256, moves_per_window: int = 65536,
                     rng: np.random.Generator | None = None, keep_tel: bool = False, max_steps: int | None = None,
                     keep_completion: bool = False):
    """-> (final order tensor, completion rounds tensor, list of per-step records).

    Each record: dict(lo, hi, best, best_tel, base_tel, committed, completed, T[, tel][, completion])."""
    rng = np.random.default_rng(0) if rng is None else rng
    n = int(base_order.shape[0])
    dev = base_order.device
    order = base_order.clone()
    completion = torch.empty(n, dtype=torch.int32, device=dev)
    committed, completed, log = 0, 0, []
    while committed < n and (max_steps is None or len(log) < max_steps):
        lo, hi = committed, min(n, committed + window)
        moves = workloads.window_moves(rng, moves_per_window, lo, hi)
        tel, res = ctx.horizon_step(order, torch.from_numpy(moves).to(dev), s, o, M, completed, complete_every,
                                    want_tel=keep_tel, completion_out=completion)
        r = [int(x) for x in res.cpu().numpy()]  # synchronises
        rec = dict(lo=lo, hi=hi, best=r[0], best_tel=r[1], base_tel=r[2], committed=r[3], completed=r[4], T=r[5])
        if keep_tel:
            rec["tel"] = tel.cpu().numpy()
        if keep_completion:  # completion rounds of the chosen order, by request id
            rec["completion"] = completion.cpu().numpy()
        log.append(rec)
        if r[0] < 0:
            raise RuntimeError("receding_horizon: the order or the instance is malformed (see device_status)")
        committed, completed = r[3], r[4]
    return order, completion, log
