"""Seeded configuration grids (structure-of-arrays, one numpy array per field).

Synthetic grids stand in for the paper's real models and dataset (Sec. 7.1
fine-tunes OPT, BLOOM, CodeGen, GPT-Neo, LLaMA ... on alpaca at sl = 512); the
estimator consumes only shapes, so each grid draws decoder shapes of those
families.  Every random draw is   lo + mix64(seed, index, field) mod span   with
the 64-bit mixer below, so any slice [first, first+n) of a grid can be produced
independently.  No estimator arithmetic lives here.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

# field order = column order of a configuration (names follow the Notation table
# where the paper has one: bs, sl; h is o_n, V is dict_n, L is l_n, d is gpu_n)
FIELDS = (
    ("arch_id", np.uint8), ("h", np.uint32), ("L", np.uint16), ("n_heads", np.uint16),
    ("n_kv", np.uint16), ("ffn", np.uint32), ("V", np.uint32), ("P", np.uint32),
    ("bs", np.uint16), ("sl", np.uint16), ("method", np.uint8), ("d", np.uint8),
    ("chunk_k", np.int8), ("flags", np.uint8),
)
FIELD_DTYPE = dict(FIELDS)

FLAG_LOGITS_FP32 = 1     # B = 4 bytes per logit instead of 2 (Sec. 4.2, "B is either B16 or B32")
FLAG_TIED_LM_HEAD = 2    # lm_head shares the input embedding (affects n_params only)
FLAG_GRAD_ALIAS = 4      # gradient fp16 lives in the param fp16 chunks (Sec. 4.1)

CHUNK_SEARCH = -1        # chunk_k value asking for the chunk-size search over k = 2..10

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_FMUL = np.uint64(0xD1B54A32D192ED03)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def mix64(seed: int, index: np.ndarray, field: int) -> np.ndarray:
    """Counter-based 64-bit hash: splitmix64's finaliser over
    seed + GOLD*(index+1) + FMUL*(field+1)  (all mod 2^64)."""
    with np.errstate(over="ignore"):
        x = (np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
             + _GOLD * (index.astype(np.uint64) + np.uint64(1))
             + _FMUL * np.uint64(field + 1))
        x ^= x >> np.uint64(30)
        x *= _C1
        x ^= x >> np.uint64(27)
        x *= _C2
        x ^= x >> np.uint64(31)
    return x


def _uniform(seed, idx, field, lo, hi):
    return (np.uint64(lo) + mix64(seed, idx, field) % np.uint64(hi - lo + 1)).astype(np.int64)


def _choice(seed, idx, field, values):
    v = np.asarray(values, dtype=np.int64)
    return v[(mix64(seed, idx, field) % np.uint64(len(values))).astype(np.int64)]


def _pack(cols: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {name: np.ascontiguousarray(cols[name].astype(dt)) for name, dt in FIELDS}


# hash field ids (fixed; part of the grid definitions)
F_H, F_L, F_V, F_BS, F_SL, F_METHOD, F_D, F_K, F_NKV, F_TP = range(10)


def grid1() -> Dict[str, np.ndarray]:
    """Tiny full Cartesian product: GPT-style L=4, h=256, 4 heads, ffn=4h, V=8192,
    P=512, untied, 2-byte logits; bs x sl x method x d x chunk (16/32/64 MiB)."""
    rows = [(bs, sl, m, d, k)
            for bs in (1, 2, 4, 8) for sl in (128, 256, 512)
            for m in (0, 1, 2) for d in (1, 2, 3, 4) for k in (4, 5, 6)]
    a = np.asarray(rows, dtype=np.int64)
    n = len(rows)
    one = np.ones(n, dtype=np.int64)
    return _pack(dict(arch_id=0 * one, h=256 * one, L=4 * one, n_heads=4 * one, n_kv=4 * one,
                      ffn=1024 * one, V=8192 * one, P=512 * one, bs=a[:, 0], sl=a[:, 1],
                      method=a[:, 2], d=a[:, 3], chunk_k=a[:, 4],
                      flags=FLAG_GRAD_ALIAS * one))


def grid2(n: int = 100_000, seed: int = 0, first: int = 0) -> Dict[str, np.ndarray]:
    """OPT/GPT-style decoders, heads = h/64, ffn = 4h, learned positions P = 2048,
    tied lm_head, 2-byte logits, chunk 2^k MiB with k in [4, 8]."""
    i = np.arange(first, first + n, dtype=np.uint64)
    h = _choice(seed, i, F_H, (768, 1024, 2048, 2560, 4096))
    one = np.ones(n, dtype=np.int64)
    return _pack(dict(
        arch_id=0 * one, h=h, L=_uniform(seed, i, F_L, 12, 32), n_heads=h // 64, n_kv=h // 64,
        ffn=4 * h, V=_choice(seed, i, F_V, (32000, 50272)), P=2048 * one,
        bs=_uniform(seed, i, F_BS, 1, 32), sl=_choice(seed, i, F_SL, (256, 512, 1024, 2048)),
        method=_uniform(seed, i, F_METHOD, 0, 2), d=_uniform(seed, i, F_D, 1, 16),
        chunk_k=_uniform(seed, i, F_K, 4, 8),
        flags=(FLAG_TIED_LM_HEAD | FLAG_GRAD_ALIAS) * one))


def _llama(n, seed, first, search):
    i = np.arange(first, first + n, dtype=np.uint64)
    h = _choice(seed, i, F_H, (2048, 4096, 5120, 8192))
    ffn = ((8 * h + 2) // 3 + 255) // 256 * 256          # SwiGLU width ~ 8h/3 rounded up to 256
    one = np.ones(n, dtype=np.int64)
    k = CHUNK_SEARCH * one if search else _uniform(seed, i, F_K, 4, 8)
    return _pack(dict(
        arch_id=0 * one, h=h, L=_uniform(seed, i, F_L, 16, 80), n_heads=h // 128,
        n_kv=_choice(seed, i, F_NKV, (1, 4, 8)), ffn=ffn,
        V=_choice(seed, i, F_V, (32000, 128256)), P=0 * one,
        bs=_uniform(seed, i, F_BS, 1, 64),
        sl=_choice(seed, i, F_SL, (512, 1024, 2048, 4096, 8192)),
        method=_uniform(seed, i, F_METHOD, 0, 2), d=_uniform(seed, i, F_D, 1, 16),
        chunk_k=k, flags=(FLAG_LOGITS_FP32 | FLAG_GRAD_ALIAS) * one))


def grid3(n: int = 1_000_000, seed: int = 0, first: int = 0):
    """Llama-style decoders (SwiGLU, RMSNorm, GQA with n_kv in {1,4,8}, heads = h/128),
    untied lm_head, 4-byte logits, fixed chunk 2^k MiB, k in [4, 8]."""
    return _llama(n, seed, first, search=False)


def grid4(n: int = 10_000_000, seed: int = 0, first: int = 0):
    """Grid 3's distribution, every configuration asking for the chunk-size search."""
    return _llama(n, seed, first, search=True)


QUERY_BS_CAP = 4096      # largest batch size a query of grid 6 considers


def grid6(n: int = 1_000_000, seed: int = 0, first: int = 0):
    """Queries of the method decision (Sec. 6, Algorithm 1 inputs: model, gpu_n, sl):
    grid 4's Llama-style shapes and sequence lengths, gpu_n in {1, 2, 4, 8, 16} in the
    column `d`, the largest batch size considered in the column `bs`, chunk-size search.
    Returns (configuration columns, tp_n): tp_n = 2^j, j uniform in [0, log2 gpu_n], is the
    tensor-parallel degree of the DP+TP set-up."""
    cols = _llama(n, seed, first, search=True)
    i = np.arange(first, first + n, dtype=np.uint64)
    log_g = (mix64(seed, i, F_D) % np.uint64(5)).astype(np.int64)
    log_t = (mix64(seed, i, F_TP) % (log_g + 1).astype(np.uint64)).astype(np.int64)
    cols["d"] = (1 << log_g).astype(np.uint8)
    cols["bs"] = np.full(n, QUERY_BS_CAP, dtype=np.uint16)
    cols["method"] = np.zeros(n, dtype=np.uint8)
    return cols, np.ascontiguousarray((1 << log_t).astype(np.uint8))


def random_queries(rng, n: int, n_arch: int = 1, wild: bool = False, bs_cap: int = 48):
    """Unstructured queries for edge-case parity tests: `random_configs` with small
    batch-size caps, plus a tp_n column (mostly a divisor of gpu_n, sometimes 0 = no
    DP+TP set-up; `wild`: sometimes not a divisor)."""
    cols = random_configs(rng, n, n_arch=n_arch, wild=wild)
    cols["bs"] = rng.integers(0, bs_cap + 1, size=n).astype(np.uint16)
    d = cols["d"].astype(np.int64)
    tp = np.ones(n, dtype=np.int64)
    for j in range(n):
        g = int(d[j])
        divs = [t for t in range(1, g + 1) if g % t == 0] or [1]
        tp[j] = divs[int(rng.integers(0, len(divs)))]
    tp = np.where(rng.random(n) < 0.1, 0, tp)
    if wild:
        tp = np.where(rng.random(n) < 0.1, rng.integers(0, 256, size=n), tp)
    return cols, np.ascontiguousarray(tp.astype(np.uint8))


GRIDS = {
    "g1": dict(make=lambda n=None, seed=0, first=0: grid1(), family="gpt", n=432),
    "g2": dict(make=grid2, family="opt", n=100_000),
    "g3": dict(make=grid3, family="llama", n=1_000_000),
    "g4": dict(make=grid4, family="llama", n=10_000_000),
}


def random_configs(rng, n: int, n_arch: int = 1, wild: bool = False) -> Dict[str, np.ndarray]:
    """Unstructured configurations for edge-case parity tests (`rng`: numpy
    Generator).  `wild` also draws invalid fields (d = 0, method 3, n_heads = 0,
    arch_id out of range, chunk_k out of range) and degenerate ones (L = 0, sl = 1)."""
    h_heads = rng.integers(1, 33, size=n)
    hd = rng.choice((16, 32, 64, 128), size=n)
    h = h_heads * hd
    cols = dict(
        arch_id=rng.integers(0, n_arch, size=n), h=h, L=rng.integers(1, 41, size=n),
        n_heads=h_heads, n_kv=rng.integers(1, 9, size=n), ffn=rng.integers(1, 20000, size=n),
        V=rng.integers(1, 200000, size=n), P=rng.integers(0, 4097, size=n),
        bs=rng.integers(1, 65, size=n), sl=rng.integers(1, 8193, size=n),
        method=rng.integers(0, 3, size=n), d=rng.integers(1, 65, size=n),
        chunk_k=rng.integers(-1, 11, size=n), flags=rng.integers(0, 8, size=n))
    if wild:
        def some(p):
            return rng.random(n) < p
        cols["d"] = np.where(some(0.05), 0, cols["d"])
        cols["d"] = np.where(some(0.05), 255, cols["d"])
        cols["method"] = np.where(some(0.05), rng.integers(3, 256, size=n), cols["method"])
        cols["n_heads"] = np.where(some(0.05), 0, cols["n_heads"])
        cols["arch_id"] = np.where(some(0.05), rng.integers(n_arch, 256, size=n), cols["arch_id"])
        cols["chunk_k"] = np.where(some(0.05), rng.integers(-128, 128, size=n), cols["chunk_k"])
        cols["L"] = np.where(some(0.05), 0, cols["L"])
        cols["sl"] = np.where(some(0.05), 1, cols["sl"])
        cols["bs"] = np.where(some(0.03), 0, cols["bs"])
    return _pack(cols)


def slice_configs(cfg: Dict[str, np.ndarray], idx) -> Dict[str, np.ndarray]:
    return {k: np.ascontiguousarray(v[idx]) for k, v in cfg.items()}
