"""Many rows through the CPU oracle on several host cores -- TEST INFRASTRUCTURE ONLY.

The oracle itself stays what it is: plain single-threaded C, one row after the other.  Here the rows
are cut into chunks and every chunk is one ordinary call of oracle.simulate_many from a Python
thread of its own (ctypes releases the interpreter lock for the duration of a foreign call and the
C code keeps no state between calls), so that a full-size comparison finishes in minutes.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle


def workers() -> int:
    """Host threads to use: the machine's cores, at most 16 (a one-GPU machine's share)."""
    return max(1, min(16, os.cpu_count() or 1))


def simulate_many(s, o, M, rows, completions: bool = True, literal: bool = False, chunk: int | None = None,
                  threads: int | None = None):
    """oracle.simulate_many over `rows` [C, n], chunks of rows on `threads` host threads.
    -> (tel [C] int64, completion [C, n] int32 or None), the same arrays one call would give."""
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    C = rows.shape[0]
    threads = workers() if threads is None else threads
    if chunk is None:
        chunk = max(1, min(256, -(-C // (4 * threads))))
    cuts = list(range(0, C, chunk))

    def one(lo):
        return oracle.simulate_many(s, o, M, rows[lo:lo + chunk], literal=literal, completions=completions)

    if threads == 1 or len(cuts) == 1:
        parts = [one(lo) for lo in cuts]
    else:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            parts = list(pool.map(one, cuts))
    tel = np.concatenate([p[0] for p in parts])
    comp = np.concatenate([p[1] for p in parts]) if completions else None
    return tel, comp
