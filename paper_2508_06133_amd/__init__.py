"""libkvsched: batched evaluation of candidate schedules for KV-cache-constrained
LLM serving (offline, backlogged model), hand-written HIP for gfx950.

Sub-modules:
  kvsched   -- thin ctypes binding over the C-ABI shared library (loads it on import
               and raises if it is missing; there is no CPU fallback).
  workloads -- seeded synthetic instance / candidate generators (no scheduling
               arithmetic in there).
  build     -- compiles the shared library with hipcc for gfx950.
"""

__all__ = ["kvsched", "workloads", "build"]
