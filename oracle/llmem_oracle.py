"""CPU oracle A: the peak-GPU-memory estimator, written out in exact integers.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the HIP path
is checked against.  Nothing in the product imports it; it imports nothing from
the product.  Python integers are unbounded, and every value that an int64
implementation would hold is asserted to fit (`_fit`).

What is computed, with the passage each function follows:

  Sec. 4.2   m_peak^s = m_base + m_p + m_os + m_out + m_lm          -> `compose`
  Sec. 4.2   m_p   (chunk rounding, then page rounding)             -> `param_memory`
  Sec. 4.2   m_os  (per-tensor page rounding, Embedding + Linear)   -> `optimizer_memory`
  Sec. 4.2   m_out (kept embedding and block outputs)               -> `output_memory`
  Sec. 4.2   m_lm  (logits, two shifted copies, lm_head params)     -> `lm_memory`
  Sec. 5     m_peak^dp (ZeRO-3), m_peak^tp, m_back^tp               -> `compose`, `tp_backward_memory`
  Sec. 4.1   chunk size chosen to minimise waste                    -> `chunk_search`
  Sec. 2.1 / Sec. 3.1  traversal of the operator timeline with live tensors and
             512-byte blocks                                        -> `timeline_peak`, `event_list_peaks`

Readings adopted where the paper is silent (each is listed in the design notes):
sizes named "param size" are element counts; ceil(x * a / b) is one exact rational
ceiling; division by gpu_n is a ceiling, then rounded to the 512-byte block; the
chunk size 2^k MiB is the byte size of one fp16 chunk; only the token embedding is
embed_p; lm_head bytes are added unrounded and carry no optimizer state.

Parity pins: tests/test_oracle_pins.py (closed forms, hand-worked example,
special cases, invariants, brute-force allocator simulation).  The printed
estimates of the paper's Table 1 cannot be reproduced (m_base, chunk size, batch
and tensor lists are not printed): parity unpinned by printed values.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

B16 = 2          # bytes per fp16 value (Notation table)
B32 = 4          # bytes per fp32 value (Notation table)
INT64_MAX = (1 << 63) - 1

# detail columns
(D_PEAK, D_PARAM, D_GRAD, D_OS, D_OUT, D_LM, D_BACK, D_K, D_LIVE, D_NPARAMS, D_TMAX, D_FLAGS) = range(12)
NDETAIL = 12

# flag bits of the detail column D_FLAGS
ERR_ARCH, ERR_METHOD, ERR_D, ERR_HEADS, ERR_CHUNK, CHUNK_INFEASIBLE = 1, 2, 4, 8, 16, 32
ERR_MASK = ERR_ARCH | ERR_METHOD | ERR_D | ERR_HEADS | ERR_CHUNK

# config flag bits
CFG_LOGITS_FP32, CFG_TIED, CFG_GRAD_ALIAS = 1, 2, 4

K_MIN, K_MAX = 2, 10          # chunk-size search range: 2^k MiB, k = 2..10
K_FIXED_MAX = 16              # largest k accepted when the chunk size is given

# explicit event lists (second entry point): fixed allocator constants
EVENT_ALIGN = 512
EVENT_SPLIT = 2 * 1024 * 1024     # rounded size below this -> small pool
EVENT_SEGMENT = 2 * 1024 * 1024   # reserved memory grows in segments of this size


def _fit(x: int) -> int:
    assert -INT64_MAX - 1 <= x <= INT64_MAX, "value does not fit int64"
    return x


def cdiv(a: int, b: int) -> int:
    """ceil(a / b) for a >= 0, b > 0."""
    assert a >= 0 and b > 0
    return (a + b - 1) // b


def up(a: int, unit: int) -> int:
    """a rounded up to a multiple of unit."""
    return _fit(cdiv(a, unit) * unit)


# ---------------------------------------------------------------------------
# model description -> sizes
# ---------------------------------------------------------------------------
def dim_vector(c: Dict[str, int]) -> Dict[str, int]:
    """The per-configuration dimensions a table monomial may refer to."""
    head_dim = c["h"] // c["n_heads"]
    return {
        "one": 1, "bs": c["bs"], "sl": c["sl"], "sl_m1": max(c["sl"] - 1, 0), "h": c["h"],
        "ffn": c["ffn"], "n_heads": c["n_heads"], "n_kv": c["n_kv"], "head_dim": head_dim,
        "kv_dim": c["n_kv"] * head_dim, "V": c["V"], "P": c["P"], "L": c["L"],
        "B_logits": B32 if c["flags"] & CFG_LOGITS_FP32 else B16, "d": c["d"],
    }


def monomial(coef: int, dims: Sequence[str], D: Dict[str, int]) -> int:
    x = coef
    for name in dims:
        x = _fit(x * D[name])
    return x


def param_census(table, D: Dict[str, int], tied: bool):
    """Notation table: embed_p, lm_p, other_p (element counts); plus the largest
    single tensor among `other` (needed by the chunk search), the parameter count
    and e_n, the number of Embedding operators of the transformer part."""
    L = D["L"]
    embed_p = lm_p = other_p = t_max = e_n = 0
    for p in table.params:
        t_p = monomial(p.coef, p.dims, D)
        count = L if p.per_layer else 1
        if p.role == "EMBED_TOK":
            embed_p += t_p * count
        elif p.role == "LM_HEAD":
            lm_p += t_p * count
        else:
            other_p += t_p * count
            t_max = max(t_max, t_p)
        if p.cls == "E" and p.role != "LM_HEAD":
            e_n += 1
    n_params = embed_p + other_p + (0 if tied else lm_p)
    return _fit(embed_p), _fit(lm_p), _fit(other_p), t_max, _fit(n_params), e_n


def chunk_elems(k: int) -> int:
    """cs in elements: a chunk of 2^k MiB holds fp16 values."""
    return (1 << k) * 1024 * 1024 // B16


def param_memory(embed_p: int, other_p: int, cs: int, cu_p: int) -> Tuple[int, int, int]:
    """Sec. 4.2, equation for m_p; m_{p,16} and m_{p,32} (Sec. 5) are the same
    chunked element count with one of the two byte widths, each page-rounded."""
    chunked = _fit(embed_p + cdiv(other_p, cs) * cs)
    m_p = up(_fit(chunked * (B16 + B32)), cu_p)
    m_p16 = up(_fit(chunked * B16), cu_p)
    m_p32 = up(_fit(chunked * B32), cu_p)
    return m_p, m_p16, m_p32


def optimizer_memory(table, D: Dict[str, int], cu_p: int) -> int:
    """Sec. 4.2, equation for m_os: momentum + variance (fp32 each), page-rounded
    per tensor, over Embedding and Linear operators of the transformer part."""
    total = 0
    for p in table.params:
        if p.cls in ("E", "L") and p.role != "LM_HEAD":
            t_p = monomial(p.coef, p.dims, D)
            one = up(_fit(t_p * (B32 + B32)), cu_p)
            for _ in range(D["L"] if p.per_layer else 1):
                total += one
    return _fit(total)


def output_memory(e_n: int, D: Dict[str, int], cu_p: int) -> int:
    """Sec. 4.2, equation for m_out: (e_n + l_n) hidden-state tensors kept under
    gradient checkpointing; o_n is the hidden width."""
    return up(_fit((e_n + D["L"]) * (D["bs"] * D["sl"] * D["h"]) * B16), cu_p)


def lm_memory(lm_p: int, D: Dict[str, int], cu_p: int) -> int:
    """Sec. 4.2, equation for m_lm: logits, two copies shifted by one position,
    and the lm_head parameters at their actual size."""
    B = D["B_logits"]
    logits = up(_fit(D["bs"] * D["sl"] * D["V"] * B), cu_p)
    shifted = up(_fit(D["bs"] * D["sl_m1"] * D["V"] * B), cu_p)
    return _fit(logits + 2 * shifted + lm_p * B16)


def tp_backward_memory(D: Dict[str, int], d: int, cu_p: int) -> int:
    """Sec. 5, equation for m_back^tp."""
    num = _fit(D["L"] * (D["bs"] * D["sl"] * D["h"]) * (d - 1) * B16)
    return _fit(cdiv(num, d * cu_p) * cu_p)


def compose(method: int, d: int, m_base: int, m_p: int, m_p16: int, m_p32: int, m_os: int,
            m_out: int, m_lm: int, m_back: int, align: int) -> int:
    """Sec. 4.2 (single GPU = conventional DP), Sec. 5 (ZeRO-3 and 1-D TP)."""
    if method == 0:
        return _fit(m_base + m_p + m_os + m_out + m_lm)
    if method == 1:
        return _fit(m_base + m_p16 + up(cdiv(m_p32 + m_os, d), align) + m_out + m_lm)
    return _fit(m_base + up(cdiv(m_p + m_os, d), align) + m_out + m_lm + m_back)


def gradient_terms(method: int, d: int, trainable: int, grad_alias: bool, cu_p: int, align: int):
    """Sec. 4.1: gradient fp16 shares the space of param fp16, so it adds nothing.
    The logical size is still reported; with aliasing switched off it is added."""
    logical = trainable * B16 if method == 0 else cdiv(trainable * B16, d)
    if grad_alias:
        extra = 0
    elif method == 0:
        extra = up(trainable * B16, cu_p)
    else:
        extra = up(cdiv(up(trainable * B16, cu_p), d), align)
    return _fit(logical), _fit(extra)


def resident_bytes(method: int, d: int, m_p: int, m_p16: int, m_p32: int, m_os: int, align: int):
    """Per-GPU parameter and optimizer-state bytes, each shard a separate block."""
    if method == 0:
        return m_p, m_os
    if method == 1:
        return _fit(m_p16 + up(cdiv(m_p32, d), align)), up(cdiv(m_os, d), align)
    return up(cdiv(m_p, d), align), up(cdiv(m_os, d), align)


# ---------------------------------------------------------------------------
# timeline traversal
# ---------------------------------------------------------------------------
def event_value(e, D: Dict[str, int], method: int, align: int) -> int:
    """Signed, block-rounded size of one table event under `method` (0 if the
    event does not exist under it)."""
    if method not in e.methods:
        return 0
    raw = _fit(monomial(e.coef, e.dims, D) * e.elem_bytes)
    if e.scale == "tp_gather":
        raw = cdiv(_fit(raw * (D["d"] - 1)), D["d"])
    r = up(raw, align)
    if e.times_L:
        r = _fit(r * D["L"])
    return e.sign * r


def timeline_peak(table, D: Dict[str, int], method: int, prelude: int, align: int) -> int:
    """Walk one fine-tuning iteration event by event and return the largest number
    of live bytes seen: resident state first, then A, F once per block, H, B once
    per block (last block first), Z."""
    by_seg = {s: [e for e in table.events if e.seg == s] for s in "AFHBZ"}
    live = peak = prelude
    order = ["A"] + ["F"] * D["L"] + ["H"] + ["B"] * D["L"] + ["Z"]
    for s in order:
        for e in by_seg[s]:
            live = _fit(live + event_value(e, D, method, align))
            if live > peak:
                peak = live
    return peak


# ---------------------------------------------------------------------------
# one configuration
# ---------------------------------------------------------------------------
def chunk_search(embed_p: int, other_p: int, t_max: int, cu_p: int) -> Tuple[int, bool]:
    """Sec. 4.1: the chunk size is chosen to minimise wasted memory.  Candidates
    2^k MiB, k = 2..10; a candidate is feasible when the largest tensor fits in one
    chunk; waste is the padding of the last chunk; ties go to the smaller chunk.
    Returns (k, feasible)."""
    best_k, best_waste = None, None
    for k in range(K_MIN, K_MAX + 1):
        cs = chunk_elems(k)
        if t_max > cs:
            continue
        waste = cdiv(other_p, cs) * cs - other_p
        if best_waste is None or waste < best_waste:
            best_k, best_waste = k, waste
    if best_k is None:
        return K_MAX, False
    return best_k, True


def estimate_one(c: Dict[str, int], tables: Sequence, const, timeline: bool = True) -> List[int]:
    """All detail columns of one configuration."""
    err = 0
    if c["arch_id"] >= len(tables):
        err |= ERR_ARCH
    if c["method"] > 2:
        err |= ERR_METHOD
    if c["d"] == 0:
        err |= ERR_D
    if c["n_heads"] == 0:
        err |= ERR_HEADS
    if not (c["chunk_k"] == -1 or 0 <= c["chunk_k"] <= K_FIXED_MAX):
        err |= ERR_CHUNK
    if err:
        out = [0] * NDETAIL
        out[D_PEAK], out[D_FLAGS] = -1, err
        return out

    table = tables[c["arch_id"]]
    method, d = c["method"], c["d"]
    cu_p, align, m_base = const.cu_p, const.align, const.m_base
    D = dim_vector(c)
    embed_p, lm_p, other_p, t_max, n_params, e_n = param_census(
        table, D, bool(c["flags"] & CFG_TIED))
    m_os = optimizer_memory(table, D, cu_p)
    m_out = output_memory(e_n, D, cu_p)
    m_lm = lm_memory(lm_p, D, cu_p)
    m_back = tp_backward_memory(D, d, cu_p) if method == 2 else 0
    grad_logical, grad_extra = gradient_terms(
        method, d, embed_p + other_p, bool(c["flags"] & CFG_GRAD_ALIAS), cu_p, align)

    def peak_at(k: int):
        m_p, m_p16, m_p32 = param_memory(embed_p, other_p, chunk_elems(k), cu_p)
        peak = compose(method, d, m_base, m_p, m_p16, m_p32, m_os, m_out, m_lm, m_back, align)
        return _fit(peak + grad_extra), (m_p, m_p16, m_p32)

    if c["chunk_k"] == -1:
        # every candidate is estimated; the least-waste feasible one is reported
        inner = {k: peak_at(k) for k in range(K_MIN, K_MAX + 1)}
        k, _ = chunk_search(embed_p, other_p, t_max, cu_p)
        m_peak, (m_p, m_p16, m_p32) = inner[k]
    else:
        k = c["chunk_k"]
        m_peak, (m_p, m_p16, m_p32) = peak_at(k)
    flags = CHUNK_INFEASIBLE if t_max > chunk_elems(k) else 0

    param_gpu, os_gpu = resident_bytes(method, d, m_p, m_p16, m_p32, m_os, align)
    live = 0
    if timeline:
        prelude = _fit(m_base + param_gpu + os_gpu + lm_p * B16 + grad_extra)
        live = timeline_peak(table, D, method, prelude, align)
    return [m_peak, param_gpu, grad_logical, os_gpu, m_out, m_lm, m_back, k, live,
            n_params, t_max, flags]


def estimate(cfg: Dict[str, Sequence[int]], tables: Sequence, const, timeline: bool = True):
    """Every configuration of a structure-of-arrays grid; returns a list of rows."""
    names = list(cfg.keys())
    n = len(cfg[names[0]])
    rows = []
    for i in range(n):
        c = {k: int(cfg[k][i]) for k in names}
        rows.append(estimate_one(c, tables, const, timeline))
    return rows


# ---------------------------------------------------------------------------
# explicit event lists (allocator timeline of one iteration given as data)
# ---------------------------------------------------------------------------
def event_list_peaks(events: Sequence[int]) -> Tuple[int, int]:
    """Sec. 3.1 (512-byte blocks) applied to a list of signed raw sizes.  Two
    pools split by rounded size; a release goes to the pool of its own size.
    allocated = largest total of live rounded bytes; reserved = each pool's own
    largest live total, rounded up to whole segments, summed.  The empty prefix
    (nothing live) counts, so both are >= 0."""
    live_small = live_large = 0
    peak_small = peak_large = peak_total = 0
    for raw in events:
        raw = int(raw)
        r = up(abs(raw), EVENT_ALIGN)
        delta = r if raw >= 0 else -r
        if r < EVENT_SPLIT:
            live_small = _fit(live_small + delta)
        else:
            live_large = _fit(live_large + delta)
        peak_small = max(peak_small, live_small)
        peak_large = max(peak_large, live_large)
        peak_total = max(peak_total, live_small + live_large)
    reserved = up(peak_small, EVENT_SEGMENT) + up(peak_large, EVENT_SEGMENT)
    return _fit(peak_total), _fit(reserved)


def event_lists_peaks(events, offsets):
    alloc, resv = [], []
    for i in range(len(offsets) - 1):
        a, r = event_list_peaks(events[int(offsets[i]):int(offsets[i + 1])])
        alloc.append(a)
        resv.append(r)
    return alloc, resv
