"""Explicit allocator event lists (signed raw bytes, CSR offsets).

`generate` produces the seeded ~10^4-event iterations of the explicit-timeline
grid through the small C generator next to this file (built on first use with
gcc); `from_lists` packs hand-written lists for tests.  No estimator arithmetic.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "events_gen.c")
_LIB = os.path.join(_HERE, "_events_gen.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64p = ctypes.POINTER(ctypes.c_int64)
        lib.llmem_events_count.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, i64p, ctypes.c_int]
        lib.llmem_events_count.restype = None
        lib.llmem_events_fill.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, i64p, i64p, ctypes.c_int]
        lib.llmem_events_fill.restype = None
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def counts(n: int, seed: int = 0, first: int = 0, threads: int = 1) -> np.ndarray:
    c = np.empty(n, dtype=np.int64)
    if n:
        _load().llmem_events_count(seed, first, n, _p(c), threads)
    return c


def generate(n: int, seed: int = 0, first: int = 0, threads: int = 1) -> Tuple[np.ndarray, np.ndarray]:
    """Events and offsets of configurations [first, first + n)."""
    c = counts(n, seed, first, threads)
    offsets = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(c, out=offsets[1:])
    events = np.empty(int(offsets[-1]), dtype=np.int64)
    if n:
        _load().llmem_events_fill(seed, first, n, _p(offsets), _p(events), threads)
    return events, offsets


def from_lists(lists: Sequence[Sequence[int]]) -> Tuple[np.ndarray, np.ndarray]:
    offsets = np.zeros(len(lists) + 1, dtype=np.int64)
    np.cumsum([len(x) for x in lists], out=offsets[1:])
    events = np.asarray([v for x in lists for v in x], dtype=np.int64).reshape(-1)
    return events, offsets
