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
  Sec. 5     m_peak^{dp+tp} (combination of DP and TP)              -> `hybrid_peak`, `method_peaks`
  Sec. 6     Algorithm 1: largest batch size per method under the
             GPU's capacity, scores, choice of the method           -> `decide_one`
  Sec. 6     the same questions asked of a whole grid of configurations at
             once (how many fit, the extremes, the best-scoring one that
             fits, per method and gpu_n)                            -> `sweep`

Readings adopted where the paper is silent (each is listed in the design notes):
sizes named "param size" are element counts; ceil(x * a / b) is one exact rational
ceiling; division by gpu_n is a ceiling, then rounded to the 512-byte block; the
chunk size 2^k MiB is the byte size of one fp16 chunk; only the token embedding is
embed_p; lm_head bytes are added unrounded and carry no optimizer state.  In the
DP+TP equation the subtracted share of param fp16 is taken as printed
(m_p16 * tp_n / gpu_n, the same ceiling-then-block division); a flag marks the
configurations where the other natural reading, m_p16 * (tp_n - 1) / tp_n, differs.
Algorithm 1: a method whose estimate exceeds the capacity already at bs = 1 gets
batch size 0; the fallback test is the printed one (on the TP score alone), and a
flag marks the queries where the prose's test (all scores zero) decides otherwise.

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
ERR_TP = 64                      # tp_n > 0 that does not divide gpu_n
HYBRID_READINGS_DIFFER = 128     # the two readings of the DP+TP subtrahend differ
FALLBACK_READINGS_DIFFER = 256   # Algorithm 1: listing and prose disagree on the fallback
ERR_MASK = ERR_ARCH | ERR_METHOD | ERR_D | ERR_HEADS | ERR_CHUNK | ERR_TP

# columns of a decision row (Algorithm 1)
(C_METHOD, C_BS, C_BS_CDP, C_BS_ADP, C_BS_TP, C_BS_HYBRID, C_SCORE2_CDP, C_SCORE2_ADP, C_SCORE2_TP,
 C_SCORE2_HYBRID, C_PEAK, C_FLAGS) = range(12)
NDECIDE = 12
METHOD_OFFLOAD = 4               # "4, 0": heterogeneous training with CPU memory

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
# DP+TP and the method decision
# ---------------------------------------------------------------------------
def hybrid_subtrahends(m_p16: int, tp_n: int, gpu_n: int, align: int) -> Tuple[int, int]:
    """Sec. 5, equation for m_peak^{dp+tp}: the share of param fp16 that tensor
    parallelism removes from a GPU.  Returns (as printed, other reading)."""
    printed = up(cdiv(_fit(m_p16 * tp_n), gpu_n), align)
    other = up(cdiv(_fit(m_p16 * (tp_n - 1)), tp_n), align)
    return printed, other


def hybrid_peak(c: Dict[str, int], tp_n: int, tables: Sequence, const) -> Tuple[int, int]:
    """Sec. 5: m_peak^{dp+tp} = m_peak^dp - m_p16 * tp_n / gpu_n + m_back^tp, with
    m_peak^dp the ZeRO-3 estimate over all gpu_n GPUs and the all-gather buffer
    of a tensor-parallel group of tp_n GPUs.  `c` is a valid configuration with
    d = gpu_n; tp_n divides gpu_n.  Returns (peak, flags)."""
    gpu_n = c["d"]
    assert tp_n >= 1 and gpu_n % tp_n == 0
    dp = estimate_one(dict(c, method=1), tables, const, timeline=False)
    table = tables[c["arch_id"]]
    D = dim_vector(c)
    embed_p, _lm_p, other_p, _t_max, _n, _e_n = param_census(table, D, bool(c["flags"] & CFG_TIED))
    _m_p, m_p16, _m_p32 = param_memory(embed_p, other_p, chunk_elems(dp[D_K]), const.cu_p)
    printed, other = hybrid_subtrahends(m_p16, tp_n, gpu_n, const.align)
    m_back = tp_backward_memory(D, tp_n, const.cu_p)
    flags = dp[D_FLAGS] | (HYBRID_READINGS_DIFFER if printed != other else 0)
    return _fit(dp[D_PEAK] - printed + m_back), flags


def _query_errors(c: Dict[str, int], tp_n: int, n_tables: int) -> int:
    err = 0
    if c["arch_id"] >= n_tables:
        err |= ERR_ARCH
    if c["d"] == 0:
        err |= ERR_D
    if c["n_heads"] == 0:
        err |= ERR_HEADS
    if not (c["chunk_k"] == -1 or 0 <= c["chunk_k"] <= K_FIXED_MAX):
        err |= ERR_CHUNK
    if tp_n > 0 and c["d"] > 0 and c["d"] % tp_n != 0:
        err |= ERR_TP
    return err


def method_peaks(c: Dict[str, int], tp_n: int, tables: Sequence, const) -> List[int]:
    """[m_peak^s, m_peak^dp, m_peak^tp, m_peak^{dp+tp}, flags] of one configuration
    (its `method` field is not read; d is gpu_n).  tp_n = 0: no DP+TP set-up, that
    entry is -1.  An invalid configuration gives -1 everywhere and its error bits."""
    err = _query_errors(c, tp_n, len(tables))
    if err:
        return [-1, -1, -1, -1, err]
    peaks, flags = [], 0
    for method in (0, 1, 2):
        row = estimate_one(dict(c, method=method), tables, const, timeline=False)
        peaks.append(row[D_PEAK])
        flags |= row[D_FLAGS]
    if tp_n > 0:
        peak, f = hybrid_peak(c, tp_n, tables, const)
        peaks.append(peak)
        flags |= f
    else:
        peaks.append(-1)
    return peaks + [flags]


def largest_batch(peak_of_bs, bs_cap: int, m_total: int) -> Tuple[int, int]:
    """Algorithm 1, inner loop of one method: start at bs = 1 and add one until the
    estimate exceeds m_total (or bs_cap is passed); the batch size before that is
    the largest one that avoids running out of memory (0 if even bs = 1 does not
    fit).  Returns (bs, estimate at that bs or 0)."""
    bs, last_peak = 1, 0
    while bs <= bs_cap:
        m_peak = peak_of_bs(bs)
        if m_peak > m_total:
            break
        last_peak = m_peak
        bs += 1
    return bs - 1, last_peak


def scores_doubled(bs_list: Sequence[int], gpu_n: int, dp_n: int) -> List[int]:
    """Algorithm 1: eval = [bs * gpu_n * 1.5, bs * gpu_n, bs, bs * dp_n] for CDP,
    ADP, TP, DP+TP; returned times two so that every score is an integer."""
    return [_fit(3 * bs_list[0] * gpu_n), _fit(2 * bs_list[1] * gpu_n), 2 * bs_list[2],
            _fit(2 * bs_list[3] * dp_n)]


def choose(score2: Sequence[int], bs_list: Sequence[int]) -> Tuple[int, int, bool]:
    """Algorithm 1, last two steps: the first index of the highest score (ties go
    to CDP, ADP, TP, DP+TP in that order) with its batch size, unless the TP score
    is 0, which selects the CPU-memory alternative "4, 0".  The third value tells
    whether the prose's test (all scores 0) would have decided differently."""
    idx = 0
    for i in range(1, len(score2)):
        if score2[i] > score2[idx]:
            idx = i
    if score2[2] != 0:
        return idx, bs_list[idx], False
    return METHOD_OFFLOAD, 0, any(x != 0 for x in score2)


def decide_one(q: Dict[str, int], tp_n: int, tables: Sequence, const, m_total: int) -> List[int]:
    """Sec. 6, Algorithm 1, for one query: model shape, gpu_n (`d`), `sl`; `bs` is
    the largest batch size considered, tp_n the tensor-parallel degree of the DP+TP
    set-up (0: none, its batch size and score stay 0).  Returns a row of NDECIDE
    columns."""
    row = [0] * NDECIDE
    err = _query_errors(q, tp_n, len(tables))
    if err:
        row[C_METHOD], row[C_FLAGS] = -1, err
        return row
    assert all("bs" not in p.dims for p in tables[q["arch_id"]].params), "parameter sizes must not depend on bs"
    gpu_n, bs_cap = q["d"], q["bs"]
    # which chunk is used and how the DP+TP term reads do not depend on bs
    flags = method_peaks(dict(q, bs=1), tp_n, tables, const)[4]
    bs_list, peak_at = [0, 0, 0, 0], [0, 0, 0, 0]
    for i in range(4 if tp_n > 0 else 3):
        bs_list[i], peak_at[i] = largest_batch(
            lambda bs: method_peaks(dict(q, bs=bs), tp_n, tables, const)[i], bs_cap, m_total)
    score2 = scores_doubled(bs_list, gpu_n, gpu_n // tp_n if tp_n > 0 else 0)
    method, bs, differ = choose(score2, bs_list)
    row[C_METHOD], row[C_BS] = method, bs
    row[C_BS_CDP:C_BS_CDP + 4] = bs_list
    row[C_SCORE2_CDP:C_SCORE2_CDP + 4] = score2
    row[C_PEAK] = peak_at[method] if method < 4 else 0
    row[C_FLAGS] = flags | (FALLBACK_READINGS_DIFFER if differ else 0)
    return row


# ---------------------------------------------------------------------------
# sweep: statistics of a grid of configurations per (method, gpu_n)
# ---------------------------------------------------------------------------
SWEEP_D_MAX = 16
SWEEP_GROUPS = 3 * SWEEP_D_MAX       # group = method * 16 + (gpu_n - 1)
(S_COUNT, S_FIT, S_MAX_PEAK, S_MIN_PEAK, S_MAX_LIVE, S_BEST, S_K_SUM, S_MAX_NPARAMS_FIT) = range(8)
NSWEEP = 8
SWEEP_INDEX_BITS = 40                # indices below 2^40
SWEEP_NONE = INT64_MAX               # S_MIN_PEAK of a group without configurations


def config_score2(method: int, bs: int, gpu_n: int) -> int:
    """Algorithm 1's score of one configuration, doubled: the batch processed per
    step over all GPUs, times 1.5 for conventional DP; a TP group processes one
    batch whatever its size."""
    return [3 * bs * gpu_n, 2 * bs * gpu_n, 2 * bs][method]


def pack_best(score2: int, index: int) -> int:
    """One int64 that orders (higher score, then lower index) as plain numbers."""
    assert 0 <= index < (1 << SWEEP_INDEX_BITS) and 0 <= score2 < (1 << 23)
    return (score2 << SWEEP_INDEX_BITS) | ((1 << SWEEP_INDEX_BITS) - 1 - index)


def unpack_best(best: int) -> Tuple[int, int]:
    return best >> SWEEP_INDEX_BITS, (1 << SWEEP_INDEX_BITS) - 1 - (best & ((1 << SWEEP_INDEX_BITS) - 1))


def sweep_rows(indices: Sequence[int], cfg: Dict[str, Sequence[int]], rows: Sequence[Sequence[int]],
               m_total: int) -> List[List[int]]:
    """Folds estimated configurations (`rows[j]` = detail row of configuration j,
    whose index in the grid is `indices[j]`) into NSWEEP statistics per group:
    how many there are, how many have m_peak <= m_total (Algorithm 1's test), the
    largest and smallest m_peak, the largest peak of the timeline, the
    best-scoring configuration that fits (ties: the lowest index; 0 if none), the
    sum of the chunk exponents used, the largest parameter count that fits.  A
    configuration with an input error, or with gpu_n above 16, counts nowhere.
    Returns stats[column][group]."""
    stats = [[0] * SWEEP_GROUPS for _ in range(NSWEEP)]
    stats[S_MIN_PEAK] = [SWEEP_NONE] * SWEEP_GROUPS
    best = [None] * SWEEP_GROUPS                 # (score2, index) of the best one that fits
    for j, row in enumerate(rows):
        method, d, bs = int(cfg["method"][j]), int(cfg["d"][j]), int(cfg["bs"][j])
        if row[D_PEAK] < 0 or row[D_FLAGS] & ERR_MASK or d > SWEEP_D_MAX:
            continue
        g = method * SWEEP_D_MAX + (d - 1)
        stats[S_COUNT][g] += 1
        stats[S_MAX_PEAK][g] = max(stats[S_MAX_PEAK][g], row[D_PEAK])
        stats[S_MIN_PEAK][g] = min(stats[S_MIN_PEAK][g], row[D_PEAK])
        stats[S_MAX_LIVE][g] = max(stats[S_MAX_LIVE][g], row[D_LIVE])
        stats[S_K_SUM][g] += row[D_K]
        if row[D_PEAK] <= m_total:
            stats[S_FIT][g] += 1
            stats[S_MAX_NPARAMS_FIT][g] = max(stats[S_MAX_NPARAMS_FIT][g], row[D_NPARAMS])
            score2, index = config_score2(method, bs, d), int(indices[j])
            if best[g] is None or score2 > best[g][0] or (score2 == best[g][0] and index < best[g][1]):
                best[g] = (score2, index)
    for g in range(SWEEP_GROUPS):
        if best[g] is not None:
            stats[S_BEST][g] = pack_best(*best[g])
    return stats


def sweep(cfg: Dict[str, Sequence[int]], first: int, tables: Sequence, const, m_total: int) -> List[List[int]]:
    """The statistics of `sweep_rows` for the configurations `cfg`, which are the
    ones with indices first, first + 1, ... of their grid."""
    rows = estimate(cfg, tables, const)
    return sweep_rows(range(first, first + len(rows)), cfg, rows, m_total)


def sweep_merge(a: Sequence[Sequence[int]], b: Sequence[Sequence[int]]) -> List[List[int]]:
    """Statistics of the union of two disjoint sets of configurations."""
    out = [list(col) for col in a]
    for g in range(SWEEP_GROUPS):
        for col in (S_COUNT, S_FIT, S_K_SUM):
            out[col][g] = a[col][g] + b[col][g]
        for col in (S_MAX_PEAK, S_MAX_LIVE, S_BEST, S_MAX_NPARAMS_FIT):
            out[col][g] = max(a[col][g], b[col][g])
        out[S_MIN_PEAK][g] = min(a[S_MIN_PEAK][g], b[S_MIN_PEAK][g])
    return out


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
