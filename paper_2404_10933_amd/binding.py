"""ctypes binding of libllmem.so: argument marshalling only.

Function names mirror the C entry points of include/llmem.h.  PyTorch supplies
device memory (tensors) and streams; no estimator arithmetic happens here, and
there is no fallback: if the shared library is missing every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libllmem.so")
_lib = None

MAX_ARCH = 8
(KERNEL_AUTO, KERNEL_WAVE, KERNEL_LANE, KERNEL_LANE_EVENTS, KERNEL_LANE_COMPILED, KERNEL_LANE_SPECIALIZED,
 KERNEL_LANE_RUNTIME, KERNEL_LANE_DIRECT) = range(8)
PROGRAM_WORDS = 704
NDETAIL = 12
DETAIL_COLUMNS = ("m_peak", "param_bytes_gpu", "grad_bytes_gpu", "os_bytes_gpu", "m_out", "m_lm",
                  "m_back", "k_chosen", "peak_live", "n_params", "t_max", "flags")

NDECIDE = 12
DECISION_COLUMNS = ("method", "bs", "bs_cdp", "bs_adp", "bs_tp", "bs_hybrid", "score2_cdp", "score2_adp",
                    "score2_tp", "score2_hybrid", "m_peak", "flags")
METHOD_CDP, METHOD_ZERO3, METHOD_TP, METHOD_HYBRID, METHOD_OFFLOAD = range(5)

NSWEEP, SWEEP_GROUPS = 8, 48
SWEEP_COLUMNS = ("count", "fit", "max_peak", "min_peak", "max_live", "best", "k_sum", "max_nparams_fit")

# column name -> (numpy dtype, torch dtype); order = struct llmem_configs
CONFIG_COLUMNS = (
    ("arch_id", np.uint8, torch.uint8), ("h", np.uint32, torch.uint32), ("L", np.uint16, torch.uint16),
    ("n_heads", np.uint16, torch.uint16), ("n_kv", np.uint16, torch.uint16), ("ffn", np.uint32, torch.uint32),
    ("V", np.uint32, torch.uint32), ("P", np.uint32, torch.uint32), ("bs", np.uint16, torch.uint16),
    ("sl", np.uint16, torch.uint16), ("method", np.uint8, torch.uint8), ("d", np.uint8, torch.uint8),
    ("chunk_k", np.int8, torch.int8), ("flags", np.uint8, torch.uint8),
)

_DIMS = ("one", "bs", "sl", "sl_m1", "h", "ffn", "n_heads", "n_kv", "head_dim", "kv_dim", "V", "P", "L",
         "B_logits", "d")
_CLS = {"E": 0, "L": 1, "B": 2, "N": 3}
_ROLE = {"EMBED_TOK": 0, "LM_HEAD": 1, "OTHER": 2}
_SEG = {"A": 0, "F": 1, "H": 2, "B": 3, "Z": 4}
_EV_FREE, _EV_TIMES_L, _EV_TP_GATHER = 1, 2, 4

PARAM_DTYPE = np.dtype([("coef", "<u4"), ("dim", "u1", (4,)), ("cls", "u1"), ("role", "u1"),
                        ("per_layer", "u1"), ("reserved", "u1", (5,))])
EVENT_DTYPE = np.dtype([("coef", "<u4"), ("dim", "u1", (4,)), ("elem_bytes", "u1"), ("seg", "u1"),
                        ("flags", "u1"), ("method_mask", "u1"), ("reserved", "<u4")])
assert PARAM_DTYPE.itemsize == 16 and EVENT_DTYPE.itemsize == 16


class LlmemError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"llmem error {code}: {text}")
        self.code = code


class _Configs(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name, _, _ in CONFIG_COLUMNS]


class _ArchDesc(ctypes.Structure):
    _fields_ = [("param_first", ctypes.c_int32), ("n_param", ctypes.c_int32),
                ("event_first", ctypes.c_int32), ("n_event", ctypes.c_int32)]


class _Tables(ctypes.Structure):
    _fields_ = [("m_base", ctypes.c_int64), ("cu_p", ctypes.c_int64), ("align", ctypes.c_int64),
                ("n_arch", ctypes.c_int32), ("n_param_total", ctypes.c_int32),
                ("n_event_total", ctypes.c_int32), ("kernel", ctypes.c_int32),
                ("arch", _ArchDesc * MAX_ARCH),
                ("params_host", ctypes.c_void_p), ("events_host", ctypes.c_void_p),
                ("params_dev", ctypes.c_void_p), ("events_dev", ctypes.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libllmem.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2404_10933_amd.build` "
            "(hipcc, gfx950); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, u64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
    lib.llmem_estimate.argtypes = [ctypes.POINTER(_Configs), i64, ctypes.POINTER(_Tables), vp]
    lib.llmem_estimate_ex.argtypes = [ctypes.POINTER(_Configs), i64, ctypes.POINTER(_Tables), vp, vp, vp]
    lib.llmem_timeline_peaks.argtypes = [vp, vp, i64, vp, vp, vp]
    lib.llmem_grid_generate.argtypes = [ci, u64, i64, i64, ctypes.POINTER(_Configs), vp]
    lib.llmem_events_count.argtypes = [u64, i64, i64, vp, vp]
    lib.llmem_events_generate.argtypes = [u64, i64, i64, vp, vp, vp]
    lib.llmem_estimate_methods.argtypes = [ctypes.POINTER(_Configs), vp, i64, ctypes.POINTER(_Tables), vp, vp, vp]
    lib.llmem_decide.argtypes = [ctypes.POINTER(_Configs), vp, i64, ctypes.POINTER(_Tables), i64, vp, vp, vp, vp]
    lib.llmem_queries_generate.argtypes = [u64, i64, i64, ctypes.POINTER(_Configs), vp, vp]
    lib.llmem_sweep.argtypes = [ci, u64, i64, i64, ctypes.POINTER(_Tables), i64, vp, vp]
    lib.llmem_sweep_reset.argtypes = [vp, vp]
    for f in (lib.llmem_estimate, lib.llmem_estimate_ex, lib.llmem_timeline_peaks, lib.llmem_grid_generate,
              lib.llmem_events_count, lib.llmem_events_generate, lib.llmem_abi_version,
              lib.llmem_estimate_methods, lib.llmem_decide, lib.llmem_queries_generate, lib.llmem_sweep,
              lib.llmem_sweep_reset):
        f.restype = ci
    lib.llmem_config_bytes.argtypes = [i64]
    lib.llmem_config_bytes.restype = ctypes.c_size_t
    lib.llmem_events_bytes.argtypes = [i64]
    lib.llmem_events_bytes.restype = ctypes.c_size_t
    lib.llmem_strerror.argtypes = [ci]
    lib.llmem_strerror.restype = ctypes.c_char_p
    lib.llmem_kernel_forms.argtypes = [ctypes.POINTER(_Tables), ctypes.POINTER(ctypes.c_int32)]
    lib.llmem_kernel_forms.restype = ci
    lib.llmem_compiled_tables.argtypes = [ctypes.POINTER(_Tables), ctypes.POINTER(ctypes.c_uint32), ctypes.c_int32,
                                          ctypes.POINTER(ctypes.c_int32)]
    lib.llmem_compiled_tables.restype = ci
    lib.llmem_kernels_release.argtypes = []
    lib.llmem_kernels_release.restype = ci
    lib.llmem_selftest_divide.argtypes = [u64, ctypes.c_uint32]
    lib.llmem_selftest_divide.restype = u64
    _lib = lib
    return lib


def _check(code: int):
    if code != 0:
        raise LlmemError(code, load_library().llmem_strerror(code).decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream) -> Optional[ctypes.c_void_p]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class DeviceConfigs:
    """n configurations as 14 device columns plus the matching C struct."""

    def __init__(self, columns: Dict[str, torch.Tensor]):
        self.columns = columns
        self.n = int(columns["h"].numel())
        for name, _, tdt in CONFIG_COLUMNS:
            t = columns[name]
            if t.dtype != tdt or t.numel() != self.n or not t.is_contiguous():
                raise ValueError(f"column {name}: need contiguous {tdt} of {self.n} values")
        self.struct = _Configs(**{name: columns[name].data_ptr() for name, _, _ in CONFIG_COLUMNS})

    @classmethod
    def from_numpy(cls, cfg: Dict[str, np.ndarray], device="cuda"):
        cols = {}
        for name, ndt, _ in CONFIG_COLUMNS:
            cols[name] = torch.from_numpy(np.ascontiguousarray(cfg[name], dtype=ndt)).to(device)
        return cls(cols)

    @classmethod
    def empty(cls, n: int, device="cuda"):
        return cls({name: torch.empty(n, dtype=tdt, device=device) for name, _, tdt in CONFIG_COLUMNS})

    def to_numpy(self) -> Dict[str, np.ndarray]:
        return {name: self.columns[name].cpu().numpy() for name, _, _ in CONFIG_COLUMNS}


class Tables:
    """Architecture tables packed into the library's 16-byte entries: a host copy
    (validated by the library on every call) and the same bytes on the device."""

    def __init__(self, tables: Sequence, m_base: int = 0, cu_p: int = 2 * 1024 * 1024, align: int = 512,
                 device="cuda", kernel: int = 0):
        if len(tables) > MAX_ARCH:
            raise ValueError("too many architecture tables")
        params, events = [], []
        self.struct = _Tables()
        self.struct.m_base, self.struct.cu_p, self.struct.align = m_base, cu_p, align
        self.struct.n_arch = len(tables)
        self.struct.kernel = kernel
        for a, t in enumerate(tables):
            self.struct.arch[a] = _ArchDesc(len(params), len(t.params), len(events), len(t.events))
            for p in t.params:
                params.append(self._param(p))
            for e in t.events:
                events.append(self._event(e))
        self.params_host = np.array(params, dtype=PARAM_DTYPE) if params else np.zeros(0, dtype=PARAM_DTYPE)
        self.events_host = np.array(events, dtype=EVENT_DTYPE) if events else np.zeros(0, dtype=EVENT_DTYPE)
        self.struct.n_param_total, self.struct.n_event_total = len(params), len(events)
        self.struct.params_host = self.params_host.ctypes.data if len(params) else None
        self.struct.events_host = self.events_host.ctypes.data if len(events) else None
        if device is None:
            # host-only tables: good for llmem_kernel_forms, not for launching (the device
            # pointers are placeholders that are never dereferenced on the host)
            self.params_dev = self.events_dev = None
            self.struct.params_dev = 16 if len(params) else None
            self.struct.events_dev = 16 if len(events) else None
        else:
            self.params_dev = torch.from_numpy(self.params_host.view(np.uint8).reshape(-1).copy()).to(device)
            self.events_dev = torch.from_numpy(self.events_host.view(np.uint8).reshape(-1).copy()).to(device)
            self.struct.params_dev = self.params_dev.data_ptr() if len(params) else None
            self.struct.events_dev = self.events_dev.data_ptr() if len(events) else None

    @staticmethod
    def _dims(names):
        if len(names) > 4:
            raise ValueError("a size is a product of at most 4 dimensions")
        idx = [_DIMS.index(n) for n in names]
        return tuple(idx + [0] * (4 - len(idx)))

    @classmethod
    def _param(cls, p):
        if not 0 <= p.coef < 2 ** 32:
            raise ValueError("coef must fit 32 bits")
        return (p.coef, cls._dims(p.dims), _CLS[p.cls], _ROLE[p.role], int(p.per_layer), (0,) * 5)

    @classmethod
    def _event(cls, e):
        if not 0 <= e.coef < 2 ** 32 or not 0 <= e.elem_bytes < 256:
            raise ValueError("coef must fit 32 bits and elem_bytes 8 bits")
        flags = (_EV_FREE if e.sign < 0 else 0) | (_EV_TIMES_L if e.times_L else 0) \
            | (_EV_TP_GATHER if e.scale == "tp_gather" else 0)
        return (e.coef, cls._dims(e.dims), e.elem_bytes, _SEG[e.seg], flags, sum(1 << m for m in e.methods), 0)


# ---------------------------------------------------------------------------
# entry points (same names as the C ABI)
# ---------------------------------------------------------------------------
def llmem_estimate(cfg: DeviceConfigs, tables: Tables, out_peaks: torch.Tensor) -> None:
    _check(load_library().llmem_estimate(ctypes.byref(cfg.struct), cfg.n, ctypes.byref(tables.struct),
                                         _ptr(out_peaks)))


def llmem_estimate_ex(cfg: DeviceConfigs, tables: Tables, out_peaks: Optional[torch.Tensor],
                      out_detail: Optional[torch.Tensor], stream=None, n: Optional[int] = None) -> None:
    """out_detail: int64 tensor of shape (NDETAIL, n) or None."""
    n = cfg.n if n is None else n
    if out_peaks is not None and (out_peaks.dtype != torch.int64 or out_peaks.numel() < n):
        raise ValueError("out_peaks: need int64 of n values")
    if out_detail is not None and (out_detail.dtype != torch.int64 or out_detail.numel() < NDETAIL * n
                                   or not out_detail.is_contiguous()):
        raise ValueError("out_detail: need contiguous int64 of NDETAIL * n values")
    _check(load_library().llmem_estimate_ex(ctypes.byref(cfg.struct), n, ctypes.byref(tables.struct),
                                            _ptr(out_peaks), _ptr(out_detail), _stream_handle(stream)))


def _check_tp(tp_n: Optional[torch.Tensor], n: int):
    if tp_n is not None and (tp_n.dtype != torch.uint8 or tp_n.numel() < n or not tp_n.is_contiguous()):
        raise ValueError("tp_n: need contiguous uint8 of n values")


def llmem_estimate_methods(cfg: DeviceConfigs, tp_n: Optional[torch.Tensor], tables: Tables,
                           out_peaks: torch.Tensor, out_flags: Optional[torch.Tensor] = None, stream=None,
                           n: Optional[int] = None) -> None:
    """out_peaks: int64 tensor of shape (4, n); out_flags: int64 of n values or None."""
    n = cfg.n if n is None else n
    _check_tp(tp_n, n)
    if out_peaks.dtype != torch.int64 or out_peaks.numel() < 4 * n or not out_peaks.is_contiguous():
        raise ValueError("out_peaks: need contiguous int64 of 4 * n values")
    if out_flags is not None and (out_flags.dtype != torch.int64 or out_flags.numel() < n):
        raise ValueError("out_flags: need int64 of n values")
    _check(load_library().llmem_estimate_methods(ctypes.byref(cfg.struct), _ptr(tp_n), n, ctypes.byref(tables.struct),
                                                 _ptr(out_peaks), _ptr(out_flags), _stream_handle(stream)))


def llmem_decide(queries: DeviceConfigs, tp_n: Optional[torch.Tensor], tables: Tables, m_total: int,
                 out_method: Optional[torch.Tensor], out_bs: Optional[torch.Tensor],
                 out_detail: Optional[torch.Tensor] = None, stream=None, n: Optional[int] = None) -> None:
    """out_method, out_bs: int32 of n values; out_detail: int64 of shape (NDECIDE, n) or None."""
    n = queries.n if n is None else n
    _check_tp(tp_n, n)
    for t in (out_method, out_bs):
        if t is not None and (t.dtype != torch.int32 or t.numel() < n or not t.is_contiguous()):
            raise ValueError("out_method / out_bs: need contiguous int32 of n values")
    if out_detail is not None and (out_detail.dtype != torch.int64 or out_detail.numel() < NDECIDE * n
                                   or not out_detail.is_contiguous()):
        raise ValueError("out_detail: need contiguous int64 of NDECIDE * n values")
    _check(load_library().llmem_decide(ctypes.byref(queries.struct), _ptr(tp_n), n, ctypes.byref(tables.struct),
                                       int(m_total), _ptr(out_method), _ptr(out_bs), _ptr(out_detail),
                                       _stream_handle(stream)))


def llmem_queries_generate(seed: int, first: int, n: int, cfg_out: DeviceConfigs, tp_n_out: torch.Tensor,
                           stream=None) -> None:
    if cfg_out.n < n:
        raise ValueError("cfg_out too small")
    _check_tp(tp_n_out, n)
    _check(load_library().llmem_queries_generate(seed, first, n, ctypes.byref(cfg_out.struct), _ptr(tp_n_out),
                                                 _stream_handle(stream)))


def _check_stats(stats: torch.Tensor) -> None:
    if stats.dtype != torch.int64 or stats.numel() < NSWEEP * SWEEP_GROUPS or not stats.is_contiguous():
        raise ValueError("stats: need contiguous int64 of NSWEEP * SWEEP_GROUPS values")


def llmem_sweep_reset(stats: torch.Tensor, stream=None) -> None:
    _check_stats(stats)
    _check(load_library().llmem_sweep_reset(_ptr(stats), _stream_handle(stream)))


def llmem_sweep(grid_id: int, seed: int, first: int, n: int, tables: Tables, m_total: int, stats: torch.Tensor,
                stream=None) -> None:
    """stats: int64 of shape (NSWEEP, SWEEP_GROUPS), added to (see llmem_sweep_reset)."""
    _check_stats(stats)
    _check(load_library().llmem_sweep(grid_id, seed, first, n, ctypes.byref(tables.struct), int(m_total),
                                      _ptr(stats), _stream_handle(stream)))


def llmem_timeline_peaks(events: torch.Tensor, offsets: torch.Tensor, out_allocated: torch.Tensor,
                         out_reserved: torch.Tensor, stream=None) -> None:
    n = offsets.numel() - 1
    for t in (events, offsets, out_allocated, out_reserved):
        if t.dtype != torch.int64 or not t.is_contiguous():
            raise ValueError("need contiguous int64 tensors")
    if out_allocated.numel() < n or out_reserved.numel() < n:
        raise ValueError("outputs too small")
    _check(load_library().llmem_timeline_peaks(_ptr(events), _ptr(offsets), n, _ptr(out_allocated),
                                               _ptr(out_reserved), _stream_handle(stream)))


def llmem_grid_generate(grid_id: int, seed: int, first: int, n: int, cfg_out: DeviceConfigs, stream=None) -> None:
    if cfg_out.n < n:
        raise ValueError("cfg_out too small")
    _check(load_library().llmem_grid_generate(grid_id, seed, first, n, ctypes.byref(cfg_out.struct),
                                              _stream_handle(stream)))


def llmem_events_count(seed: int, first: int, n: int, counts: torch.Tensor, stream=None) -> None:
    if counts.dtype != torch.int64 or counts.numel() < n:
        raise ValueError("counts: need int64 of n values")
    _check(load_library().llmem_events_count(seed, first, n, _ptr(counts), _stream_handle(stream)))


def llmem_events_generate(seed: int, first: int, n: int, offsets: torch.Tensor, events: torch.Tensor,
                          stream=None) -> None:
    if offsets.dtype != torch.int64 or events.dtype != torch.int64 or offsets.numel() < n + 1:
        raise ValueError("offsets: need int64 of n + 1 values; events int64")
    _check(load_library().llmem_events_generate(seed, first, n, _ptr(offsets), _ptr(events),
                                                _stream_handle(stream)))


def llmem_kernel_forms(tables: "Tables") -> Dict[str, int]:
    info = (ctypes.c_int32 * 8)()
    _check(load_library().llmem_kernel_forms(ctypes.byref(tables.struct), info))
    return {"allowed": [k for k in range(1, 8) if info[0] >> k & 1],
            "prebuilt": [bool(info[0] >> (8 + flavour) & 1) for flavour in range(3)],
            "program_words": info[1],
            "compiled_slots": info[2], "event_slots": info[3], "wave_slots": info[4],
            "param_groups": info[5] & 0xffff, "size_classes": info[5] >> 16, "terms": info[6],
            "peak_points": info[7]}


def llmem_compiled_tables(tables: "Tables"):
    """(words, first): the compiled form of the tables and the first word of each architecture."""
    words = (ctypes.c_uint32 * PROGRAM_WORDS)()
    first = (ctypes.c_int32 * MAX_ARCH)()
    n = load_library().llmem_compiled_tables(ctypes.byref(tables.struct), words, PROGRAM_WORDS, first)
    if n < 0:
        _check(n)
    return list(words[:n]), list(first)


def llmem_config_bytes(n: int) -> int:
    return int(load_library().llmem_config_bytes(n))


def llmem_events_bytes(n: int) -> int:
    return int(load_library().llmem_events_bytes(n))


def llmem_strerror(code: int) -> str:
    return load_library().llmem_strerror(code).decode()


def llmem_abi_version() -> int:
    return int(load_library().llmem_abi_version())


def llmem_kernels_release() -> int:
    """Unloads the kernels built at run time (synchronizes their devices first).  Returns how many."""
    got = int(load_library().llmem_kernels_release())
    if got < 0:
        _check(got)
    return got
