"""Seeded synthetic instances and candidate-order sets.

The paper evaluates on LMSYS-Chat-1M conversations mixed with Arxiv long-document
summarisation (Section 7, "Dataset Overview"); neither is available offline, so these
generators stand in for them with the same structure: many short chat requests plus a
minority of long-prompt requests, one KV budget M, all requests present at round 0.

Nothing in this module computes anything of the scheduling method itself: it draws
request lengths and builds candidate orders from a *given* base order by index moves.
Both the CPU oracle's tests and the GPU path's tests/bench use it.
"""
from __future__ import annotations

import functools
import itertools
from dataclasses import dataclass

import numpy as np

SEED0 = 20250806

MOVE_SWAP = 0
MOVE_INSERT = 1


@dataclass(frozen=True)
class Instance:
    name: str
    s: np.ndarray  # int32 [n] prompt lengths
    o: np.ndarray  # int32 [n] decode lengths
    M: int  # KV budget in tokens

    @property
    def n(self) -> int:
        return int(self.s.shape[0])


def _rng(cfg: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng(SEED0 + cfg + 1000 * stream)


def _chat_lengths(rng: np.random.Generator, n: int):
    s = np.clip(np.rint(rng.lognormal(np.log(128.0), 0.8, n)), 4, 2048)
    o = np.clip(np.rint(rng.lognormal(np.log(200.0), 0.9, n)), 1, 2048)
    return s.astype(np.int32), o.astype(np.int32)


def _mixed_lengths(rng: np.random.Generator, n: int):
    s, o = _chat_lengths(rng, n)
    is_long = rng.random(n) < 0.3
    s_long = rng.integers(2048, 8193, n).astype(np.int32)
    o_long = rng.integers(100, 501, n).astype(np.int32)
    return np.where(is_long, s_long, s).astype(np.int32), np.where(is_long, o_long, o).astype(np.int32)


def instance(cfg: int, n: int | None = None, M: int | None = None) -> Instance:
    """The five workload configurations; `n` / `M` override the size for scaled-down tests."""
    rng = _rng(cfg)
    if cfg == 1:  # tiny exact
        n = 8 if n is None else n
        s = rng.integers(1, 9, n).astype(np.int32)
        o = rng.integers(1, 9, n).astype(np.int32)
        return Instance("tiny-exact", s, o, 48 if M is None else M)
    if cfg == 2:  # short conversations
        n = 200 if n is None else n
        s, o = _chat_lengths(rng, n)
        return Instance("short-conversation", s, o, 16384 if M is None else M)
    if cfg == 3:  # mixed chat + long-document summarisation
        n = 2000 if n is None else n
        s, o = _mixed_lengths(rng, n)
        return Instance("mixed-chat-summarization", s, o, 131072 if M is None else M)
    if cfg == 4:  # receding-horizon scale
        n = 10000 if n is None else n
        s, o = _mixed_lengths(rng, n)
        return Instance("receding-horizon", s, o, 1048576 if M is None else M)
    if cfg == 5:  # adversarial bimodal
        n = 100000 if n is None else n
        s = np.where(rng.random(n) < 0.5, 1, 4096).astype(np.int32)
        o = np.where(rng.random(n) < 0.5, 4096, 1).astype(np.int32)
        return Instance("adversarial-bimodal", s, o, 2097152 if M is None else M)
    raise ValueError(f"unknown config {cfg}")


# ----------------------------------------------------------------------------- moves

def apply_move(order: np.ndarray, move) -> np.ndarray:
    """Position-level neighbour of a priority order.

    swap(i, j): exchange the entries at positions i and j.
    insert(i, j): take the entry at position i out and put it back so that it ends up at
    position j; the entries in between shift by one.  i == j is the identity for both.
    """
    kind, i, j = int(move[0]), int(move[1]), int(move[2])
    out = np.array(order, dtype=np.int32, copy=True)
    if kind == MOVE_SWAP:
        out[i], out[j] = order[j], order[i]
    elif kind == MOVE_INSERT:
        out = np.insert(np.delete(out, i), j, order[i]).astype(np.int32)
    else:
        raise ValueError("move type must be 0 (swap) or 1 (insert)")
    return out


def random_swap_moves(rng: np.random.Generator, count: int, lo: int, hi: int, distinct: bool = False) -> np.ndarray:
    """`count` swap moves with both positions in [lo, hi), i != j; optionally distinct pairs."""
    moves = np.zeros((count, 3), dtype=np.int32)
    seen = set()
    k = 0
    while k < count:
        i, j = (int(x) for x in rng.integers(lo, hi, 2))
        if i == j:
            continue
        a, b = min(i, j), max(i, j)
        if distinct:
            if (a, b) in seen:
                continue
            seen.add((a, b))
        moves[k] = (MOVE_SWAP, a, b)
        k += 1
    return moves


def window_moves(rng: np.random.Generator, count: int, lo: int, hi: int) -> np.ndarray:
    """Move 0 is the identity; the rest alternate swaps (odd index) and inserts (even index) on two
    different positions drawn uniformly inside [lo, hi)."""
    moves = np.zeros((count, 3), dtype=np.int32)
    moves[:, 1] = lo
    moves[:, 2] = lo
    if hi - lo < 2 or count < 2:
        return moves
    i = rng.integers(lo, hi, count - 1)
    j = rng.integers(lo, hi - 1, count - 1)
    j = j + (j >= i)  # uniform over the positions other than i
    moves[1:, 0] = np.where(np.arange(1, count) % 2 == 1, MOVE_SWAP, MOVE_INSERT)
    moves[1:, 1] = i
    moves[1:, 2] = j
    return moves


def moves_anywhere(rng: np.random.Generator, count: int, n: int) -> np.ndarray:
    """Move 0 is the identity; the rest are swaps and inserts (a coin each) on two positions drawn
    uniformly over the whole order (they may coincide: the identity again)."""
    moves = np.zeros((count, 3), dtype=np.int32)
    if count > 1:
        moves[1:, 0] = rng.integers(0, 2, count - 1)
        moves[1:, 1] = rng.integers(0, n, count - 1)
        moves[1:, 2] = rng.integers(0, n, count - 1)
    return moves


def tight_instance(seed: int, n: int, o_max: int, long_frac: float = 0.25, width: float = 3.0) -> Instance:
    """A small instance under a tight budget, for parity cases in which most requests have to wait:
    decode lengths uniform in [1, o_max // 16] or, with probability long_frac, in (o_max // 2, o_max]
    (one request has exactly o_max), prompts uniform in [1, o_max // 4], and a budget of `width` times
    the largest s + o."""
    rng = np.random.default_rng(SEED0 + 7000 + seed)
    short = rng.integers(1, max(1, o_max // 16) + 1, n)
    long_ = rng.integers(o_max // 2 + 1, o_max + 1, n)
    o = np.where(rng.random(n) < long_frac, long_, short).astype(np.int32)
    o[int(rng.integers(0, n))] = o_max
    s = rng.integers(1, max(1, o_max // 4) + 1, n).astype(np.int32)
    M = int(width * int((s.astype(np.int64) + o).max()))
    return Instance(f"tight{seed}", s, o, M)


def orders_from_moves(base: np.ndarray, moves: np.ndarray) -> np.ndarray:
    rows = np.empty((moves.shape[0], base.shape[0]), dtype=np.int32)
    for k in range(moves.shape[0]):
        rows[k] = apply_move(base, moves[k])
    return rows


# ------------------------------------------------------------------------ candidates

def all_permutations(n: int) -> np.ndarray:
    """All n! orders in lexicographic order, int32 [n!, n]."""
    return np.array(list(itertools.permutations(range(n))), dtype=np.int32)


def candidates(cfg: int, base: np.ndarray, count: int | None = None) -> np.ndarray:
    """Candidate order matrix [C, n] for configurations 1, 2, 3 and 5 given the base order.

    cfg 1: every permutation of the n requests (lexicographic) followed by the base order.
    cfg 2: row 0 = base; the rest = base with one random position pair exchanged.
    cfg 3: row 0 = base; then distinct random 1-swap neighbours; the last 256 rows
           (count // 64 when scaled down) are uniform random permutations (restarts).
    cfg 5: row 0 = base; the rest = base with 64 random position pairs exchanged in turn.
    """
    base = np.asarray(base, dtype=np.int32)
    n = base.shape[0]
    rng = _rng(cfg, stream=1)
    if cfg == 1:
        return np.concatenate([all_permutations(n), base[None, :]], axis=0)
    if cfg == 2:
        C = 4096 if count is None else count
        moves = random_swap_moves(rng, C - 1, 0, n)
        return np.concatenate([base[None, :], orders_from_moves(base, moves)], axis=0)
    if cfg == 3:
        C = 16384 if count is None else count
        restarts = 256 if count is None else max(1, C // 64)
        moves = random_swap_moves(rng, C - 1 - restarts, 0, n, distinct=True)
        rows = np.empty((C, n), dtype=np.int32)
        rows[0] = base
        rows[1 : C - restarts] = np.broadcast_to(base, (C - 1 - restarts, n))
        idx = np.arange(C - 1 - restarts)
        a, b = moves[:, 1], moves[:, 2]
        rows[1 + idx, a] = base[b]
        rows[1 + idx, b] = base[a]
        for k in range(restarts):
            rows[C - restarts + k] = rng.permutation(n).astype(np.int32)
        return rows
    if cfg == 5:
        C = 1025 if count is None else count
        rows = np.broadcast_to(base, (C, n)).copy()
        for k in range(1, C):
            for _ in range(64):
                i, j = (int(x) for x in rng.integers(0, n, 2))
                rows[k, i], rows[k, j] = rows[k, j], rows[k, i]
        return rows
    raise ValueError("config 4 draws its candidates per re-planning window; see window_moves()")


# ------------------------------------------------------------------- online arrivals

# Normalised loads rho = lambda / lambda* of the paper's Poisson experiment (Section 7,
# "Experiment under Online Poisson Arrivals": lambda = 0.05 .. 0.30 against lambda* = 0.104).
ONLINE_RHO = (0.48, 0.67, 0.87, 1.06, 1.25, 1.44, 1.73, 2.02, 2.40, 2.88)
ONLINE_M = 16492  # the KV budget the paper derives for its serving setup
ONLINE_T = 4000  # iterations during which requests arrive


def _online_lengths(rng: np.random.Generator, n: int, long_frac: float):
    s, o = _chat_lengths(rng, n)
    is_long = rng.random(n) < long_frac
    s_long = rng.integers(2048, 8193, n).astype(np.int32)
    o_long = rng.integers(100, 501, n).astype(np.int32)
    return np.where(is_long, s_long, s).astype(np.int32), np.where(is_long, o_long, o).astype(np.int32)


@functools.lru_cache(maxsize=None)
def online_lambda_star(M: int = ONLINE_M, long_frac: float = 0.2) -> float:
    """Arrival rate at which the offered token-rounds equal the budget: M over the mean
    memory-time area sum_{j=1..o}(s + j) of one request, estimated on a fixed seeded sample."""
    s, o = _online_lengths(np.random.default_rng(SEED0 + 777), 200_000, long_frac)
    area = s.astype(np.float64) * o + o.astype(np.float64) * (o + 1) / 2
    return float(M / area.mean())


def online_instance(seed: int, rho: float, T: int = ONLINE_T, M: int = ONLINE_M, long_frac: float = 0.2):
    """Poisson arrivals of rate rho * lambda* per iteration over T iterations, lengths from the
    short/long mixture (80/20 by default, as in the paper's online experiment; chat lengths and
    long-document lengths as in configurations 2 and 3).  -> (a, s, o, M), a nondecreasing int32."""
    rng = np.random.default_rng(SEED0 + 5000 + seed)
    lam = rho * online_lambda_star(M, long_frac)
    counts = rng.poisson(lam, T)
    a = np.repeat(np.arange(T, dtype=np.int32), counts).astype(np.int32)
    s, o = _online_lengths(rng, a.shape[0], long_frac)
    return a, s, o, M


# ------------------------------------------------------------- predicted decode lengths

def prediction_intervals(seed: int, s: np.ndarray, o: np.ndarray, M: int, gamma: float):
    """Interval predictions [lower_i, upper_i] around the true decode lengths (Section 5,
    "Prediction Model": o_i in [l_i, u_i], gamma = inf l_i / u_i): l_i = ceil(a_i o_i) and
    u_i = floor(o_i / b_i) with a_i, b_i uniform in [sqrt(gamma), 1], u_i capped so that
    s_i + u_i <= M.  -> (lower, upper) int32."""
    rng = np.random.default_rng(SEED0 + 9000 + seed)
    g = float(np.sqrt(gamma))
    a = rng.uniform(g, 1.0, o.shape[0])
    b = rng.uniform(g, 1.0, o.shape[0])
    lower = np.maximum(1, np.ceil(a * o)).astype(np.int64)
    upper = np.minimum(np.floor(o / b), np.asarray(M, dtype=np.int64) - s).astype(np.int64)
    return np.minimum(lower, o).astype(np.int32), np.maximum(upper, o).astype(np.int32)
