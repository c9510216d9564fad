"""ctypes front end of CPU oracle B (llmem_oracle.c).  TEST INFRASTRUCTURE ONLY.

Packs the table objects into the oracle's own C structs (this packing is the
oracle's and is not shared with the HIP binding), builds the library with gcc on
first use, and returns numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "llmem_oracle.c")
_LIB = os.path.join(_HERE, "_llmem_oracle.so")
_lib = None

NDETAIL = 12
_DIMS = ("one", "bs", "sl", "sl_m1", "h", "ffn", "n_heads", "n_kv", "head_dim", "kv_dim",
         "V", "P", "L", "B_logits", "d")
_CLS = {"E": 0, "L": 1, "B": 2, "N": 3}
_ROLE = {"EMBED_TOK": 0, "LM_HEAD": 1, "OTHER": 2}
_SEG = {"A": 0, "F": 1, "H": 2, "B": 3, "Z": 4}
_SCALE = {"none": 0, "tp_gather": 1}


class _Param(ctypes.Structure):
    _fields_ = [("coef", ctypes.c_int64), ("ndims", ctypes.c_int32), ("dims", ctypes.c_int32 * 4),
                ("cls", ctypes.c_int32), ("role", ctypes.c_int32), ("per_layer", ctypes.c_int32)]


class _Event(ctypes.Structure):
    _fields_ = [("coef", ctypes.c_int64), ("ndims", ctypes.c_int32), ("dims", ctypes.c_int32 * 4),
                ("elem_bytes", ctypes.c_int32), ("seg", ctypes.c_int32), ("sign", ctypes.c_int32),
                ("method_mask", ctypes.c_int32), ("scale", ctypes.c_int32), ("times_L", ctypes.c_int32)]


class _Table(ctypes.Structure):
    _fields_ = [("n_params", ctypes.c_int32), ("n_events", ctypes.c_int32),
                ("params", ctypes.POINTER(_Param)), ("events", ctypes.POINTER(_Event))]


_CFG_FIELDS = (("arch_id", np.uint8), ("h", np.uint32), ("L", np.uint16), ("n_heads", np.uint16),
               ("n_kv", np.uint16), ("ffn", np.uint32), ("V", np.uint32), ("P", np.uint32),
               ("bs", np.uint16), ("sl", np.uint16), ("method", np.uint8), ("d", np.uint8),
               ("chunk_k", np.int8), ("flags", np.uint8))


class _Configs(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name, _ in _CFG_FIELDS]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.llmem_oracle_estimate.restype = ctypes.c_int
        lib.llmem_oracle_estimate.argtypes = [
            ctypes.POINTER(_Configs), ctypes.c_int64, ctypes.POINTER(_Table), ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.llmem_oracle_event_lists.restype = ctypes.c_int
        lib.llmem_oracle_event_lists.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                                 ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.llmem_oracle_methods.restype = ctypes.c_int
        lib.llmem_oracle_methods.argtypes = [
            ctypes.POINTER(_Configs), ctypes.c_void_p, ctypes.c_int64, ctypes.POINTER(_Table), ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.llmem_oracle_decide.restype = ctypes.c_int
        lib.llmem_oracle_decide.argtypes = [
            ctypes.POINTER(_Configs), ctypes.c_void_p, ctypes.c_int64, ctypes.POINTER(_Table), ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int]
        lib.llmem_oracle_sweep.restype = ctypes.c_int
        lib.llmem_oracle_sweep.argtypes = [ctypes.POINTER(_Configs), ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        _lib = lib
    return _lib


def _pack_tables(tables: Sequence):
    keep = []
    arr = (_Table * max(len(tables), 1))()
    for a, t in enumerate(tables):
        ps = (_Param * max(len(t.params), 1))()
        for j, p in enumerate(t.params):
            ps[j].coef, ps[j].ndims = p.coef, len(p.dims)
            for q, name in enumerate(p.dims):
                ps[j].dims[q] = _DIMS.index(name)
            ps[j].cls, ps[j].role, ps[j].per_layer = _CLS[p.cls], _ROLE[p.role], int(p.per_layer)
        es = (_Event * max(len(t.events), 1))()
        for j, e in enumerate(t.events):
            es[j].coef, es[j].ndims = e.coef, len(e.dims)
            for q, name in enumerate(e.dims):
                es[j].dims[q] = _DIMS.index(name)
            es[j].elem_bytes, es[j].seg, es[j].sign = e.elem_bytes, _SEG[e.seg], e.sign
            es[j].method_mask = sum(1 << m for m in e.methods)
            es[j].scale, es[j].times_L = _SCALE[e.scale], int(e.times_L)
        arr[a].n_params, arr[a].n_events = len(t.params), len(t.events)
        arr[a].params, arr[a].events = ps, es
        keep += [ps, es]
    return arr, keep


def estimate(cfg: Dict[str, np.ndarray], tables: Sequence, const, timeline: bool = True,
             threads: int = 1, want_detail: bool = True):
    """Returns (peaks[n], detail[n, 12] or None).  Raises on int64 overflow."""
    lib = _load()
    cols = {name: np.ascontiguousarray(cfg[name], dtype=dt) for name, dt in _CFG_FIELDS}
    n = len(cols["h"])
    c = _Configs(**{name: cols[name].ctypes.data for name, _ in _CFG_FIELDS})
    arr, keep = _pack_tables(tables)
    peaks = np.empty(n, dtype=np.int64)
    detail = np.empty((n, NDETAIL), dtype=np.int64) if want_detail else None
    rc = lib.llmem_oracle_estimate(ctypes.byref(c), n, arr, len(tables), const.m_base, const.cu_p,
                                   const.align, int(timeline), peaks.ctypes.data,
                                   detail.ctypes.data if want_detail else None, threads)
    if rc == 1:
        raise OverflowError("an intermediate value does not fit int64")
    if rc:
        raise ValueError("malformed table")
    del keep
    return peaks, detail


def _raise(rc):
    if rc == 1:
        raise OverflowError("an intermediate value does not fit int64")
    if rc:
        raise ValueError("malformed table")


def method_peaks(cfg: Dict[str, np.ndarray], tp_n: np.ndarray, tables: Sequence, const, threads: int = 1):
    """Returns (peaks[n, 4], flags[n]): CDP, ZeRO-3, TP, DP+TP estimates of every configuration."""
    lib = _load()
    cols = {name: np.ascontiguousarray(cfg[name], dtype=dt) for name, dt in _CFG_FIELDS}
    tp = np.ascontiguousarray(tp_n, dtype=np.uint8)
    n = len(cols["h"])
    c = _Configs(**{name: cols[name].ctypes.data for name, _ in _CFG_FIELDS})
    arr, keep = _pack_tables(tables)
    peaks = np.empty((n, 4), dtype=np.int64)
    flags = np.empty(n, dtype=np.int64)
    _raise(lib.llmem_oracle_methods(ctypes.byref(c), tp.ctypes.data, n, arr, len(tables), const.m_base,
                                    const.cu_p, const.align, peaks.ctypes.data, flags.ctypes.data, threads))
    del keep
    return peaks, flags


NDECIDE = 12


def decide(cfg: Dict[str, np.ndarray], tp_n: np.ndarray, tables: Sequence, const, m_total: int,
           threads: int = 1):
    """Algorithm 1 for every query; returns rows[n, NDECIDE]."""
    lib = _load()
    cols = {name: np.ascontiguousarray(cfg[name], dtype=dt) for name, dt in _CFG_FIELDS}
    tp = np.ascontiguousarray(tp_n, dtype=np.uint8)
    n = len(cols["h"])
    c = _Configs(**{name: cols[name].ctypes.data for name, _ in _CFG_FIELDS})
    arr, keep = _pack_tables(tables)
    rows = np.empty((n, NDECIDE), dtype=np.int64)
    _raise(lib.llmem_oracle_decide(ctypes.byref(c), tp.ctypes.data, n, arr, len(tables), const.m_base,
                                   const.cu_p, const.align, int(m_total), rows.ctypes.data, threads))
    del keep
    return rows


NSWEEP, SWEEP_GROUPS = 8, 48


def sweep(cfg: Dict[str, np.ndarray], first: int, tables: Sequence, const, m_total: int, threads: int = 1):
    """Statistics per (method, gpu_n) of the configurations `cfg`, whose indices in their grid
    start at `first`; returns stats[NSWEEP, SWEEP_GROUPS]."""
    lib = _load()
    _, detail = estimate(cfg, tables, const, threads=threads)
    cols = {name: np.ascontiguousarray(cfg[name], dtype=dt) for name, dt in _CFG_FIELDS}
    c = _Configs(**{name: cols[name].ctypes.data for name, _ in _CFG_FIELDS})
    stats = np.empty((NSWEEP, SWEEP_GROUPS), dtype=np.int64)
    _raise(lib.llmem_oracle_sweep(ctypes.byref(c), len(cols["h"]), int(first), detail.ctypes.data,
                                  int(m_total), stats.ctypes.data))
    return stats


def event_lists_peaks(events: np.ndarray, offsets: np.ndarray, threads: int = 1):
    lib = _load()
    events = np.ascontiguousarray(events, dtype=np.int64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    n = len(offsets) - 1
    alloc = np.empty(n, dtype=np.int64)
    resv = np.empty(n, dtype=np.int64)
    rc = lib.llmem_oracle_event_lists(events.ctypes.data, offsets.ctypes.data, n,
                                      alloc.ctypes.data, resv.ctypes.data, threads)
    if rc:
        raise OverflowError("an intermediate value does not fit int64")
    return alloc, resv
