"""Pins of CPU oracle A for the sweep statistics (the questions of Sec. 6 asked of a
whole grid): a hand-worked example (tests/golden), a brute-force restatement that
filters and sorts instead of folding, merging of disjoint index ranges, the order
of the packed best entry, and planted mistakes the pins must notice."""
import functools
import random

import numpy as np
import pytest

from oracle import llmem_oracle as O
from workloads import tables as T
from workloads import grids as G

CONST0 = T.Constants(m_base=0)


def _group(method, gpu_n):
    return method * 16 + gpu_n - 1


def test_worked_sweep(golden):
    g = golden("worked_sweep_gpt_tiny.txt")
    cfg = G.grid1()
    stats = O.sweep(cfg, 0, [T.gpt_table()], CONST0, g["m_total"])
    for method in range(3):
        for d in range(1, 5):
            q = _group(method, d)
            assert stats[O.S_COUNT][q] == g["count"]
            assert stats[O.S_K_SUM][q] == g["k_sum"]
            assert stats[O.S_MAX_NPARAMS_FIT][q] == g["n_params"]
        for d in range(5, 17):
            q = _group(method, d)
            assert [stats[c][q] for c in range(O.NSWEEP)] == [0, 0, 0, O.SWEEP_NONE, 0, 0, 0, 0]
    for d in range(1, 5):
        q = _group(0, d)
        assert (stats[O.S_FIT][q], stats[O.S_MAX_PEAK][q], stats[O.S_MIN_PEAK][q]) == (
            g["cdp_fit"], g["cdp_max_peak"], g["cdp_min_peak"])
    for d in (1, 2):
        assert O.unpack_best(stats[O.S_BEST][_group(0, d)]) == (g[f"cdp{d}_best_score2"], g[f"cdp{d}_best_index"])
    for name, q in (("adp3", _group(1, 3)), ("tp4", _group(2, 4))):
        assert (stats[O.S_FIT][q], stats[O.S_MAX_PEAK][q], stats[O.S_MIN_PEAK][q]) == (
            g[f"{name}_fit"], g[f"{name}_max_peak"], g[f"{name}_min_peak"])
        assert O.unpack_best(stats[O.S_BEST][q]) == (g[f"{name}_best_score2"], g[f"{name}_best_index"])
    tight = O.sweep(cfg, 0, [T.gpt_table()], CONST0, g["tight_m_total"])
    q = _group(2, 4)
    assert (tight[O.S_FIT][q], tight[O.S_BEST][q], tight[O.S_MAX_NPARAMS_FIT][q]) == (
        g["tight_tp4_fit"], g["tight_tp4_best"], g["tight_tp4_max_nparams_fit"])
    assert tight[O.S_MIN_PEAK][q] == g["tp4_min_peak"] and tight[O.S_COUNT][q] == g["count"]


def _brute(indices, cfg, rows, m_total):
    """The same statistics by selecting each group's configurations and sorting them."""
    stats = np.zeros((O.NSWEEP, O.SWEEP_GROUPS), dtype=object)
    for method in range(3):
        for d in range(1, 17):
            q = _group(method, d)
            members = [j for j in range(len(rows)) if cfg["method"][j] == method and cfg["d"][j] == d
                       and not (rows[j][O.D_FLAGS] & O.ERR_MASK)]
            peaks = sorted(rows[j][O.D_PEAK] for j in members)
            fitting = [j for j in members if not rows[j][O.D_PEAK] > m_total]
            stats[O.S_COUNT][q] = len(members)
            stats[O.S_FIT][q] = len(fitting)
            stats[O.S_MAX_PEAK][q] = peaks[-1] if peaks else 0
            stats[O.S_MIN_PEAK][q] = peaks[0] if peaks else O.SWEEP_NONE
            stats[O.S_MAX_LIVE][q] = max([rows[j][O.D_LIVE] for j in members], default=0)
            stats[O.S_K_SUM][q] = sum(rows[j][O.D_K] for j in members)
            stats[O.S_MAX_NPARAMS_FIT][q] = max([rows[j][O.D_NPARAMS] for j in fitting], default=0)
            # throughput per step as a fraction-free product: bs * gpus * 3/2, bs * gpus, bs
            ranked = sorted(fitting, key=lambda j: (-int(cfg["bs"][j]) * (1 if method == 2 else d) * (3 if method == 0 else 2),
                                                    indices[j]))
            if ranked:
                j = ranked[0]
                score2 = int(cfg["bs"][j]) * (1 if method == 2 else d) * (3 if method == 0 else 2)
                stats[O.S_BEST][q] = score2 * 2 ** 40 + (2 ** 40 - 1 - indices[j])
    return stats.tolist()


@functools.lru_cache(maxsize=None)
def _estimated(seed, n=300):
    rng = random.Random(seed)
    cfg = G.random_configs(np.random.default_rng(seed), n, n_arch=2, wild=(seed == 3))
    cfg["d"] = np.minimum(cfg["d"], 20).astype(cfg["d"].dtype)        # a few above 16: skipped
    rows = O.estimate(cfg, [T.gpt_table(), T.llama_table()], CONST0)
    indices = [rng.randrange(0, 2 ** 40) for _ in range(n)]
    indices[:50] = sorted(indices[:50])
    return cfg, rows, indices


@pytest.mark.parametrize("seed", (1, 2, 3))
def test_sweep_against_selection_and_sorting(seed):
    cfg, rows, indices = _estimated(seed)
    peaks = sorted(r[O.D_PEAK] for r in rows if r[O.D_PEAK] > 0)
    for m_total in (peaks[len(peaks) // 3], peaks[-1], peaks[0] - 1, 0):
        got = O.sweep_rows(indices, cfg, rows, m_total)
        assert got == _brute(indices, cfg, rows, m_total)
    assert sum(got[O.S_COUNT]) == sum(1 for j, r in enumerate(rows) if r[O.D_PEAK] >= 0 and cfg["d"][j] <= 16)


def test_ties_go_to_the_lowest_index():
    cfg = G.slice_configs(G.grid1(), [324] * 5)
    rows = O.estimate(cfg, [T.gpt_table()], CONST0)
    stats = O.sweep_rows([900, 17, 512, 17, 40], cfg, rows, rows[0][O.D_PEAK])
    assert O.unpack_best(stats[O.S_BEST][_group(0, 1)]) == (24, 17)
    assert stats[O.S_FIT][_group(0, 1)] == 5


def test_merge_of_disjoint_ranges():
    cfg = G.grid2(300, seed=3)
    tables = [T.opt_table()]
    m_total = 24 << 30
    whole = O.sweep(cfg, 1000, tables, CONST0, m_total)
    parts = None
    for lo, hi in ((0, 1), (1, 250), (250, 251), (251, 300)):
        part = O.sweep(G.slice_configs(cfg, np.arange(lo, hi)), 1000 + lo, tables, CONST0, m_total)
        parts = part if parts is None else O.sweep_merge(parts, part)
    assert parts == whole
    assert 0 < sum(whole[O.S_FIT]) < sum(whole[O.S_COUNT]) == 300


def test_packed_best_orders_like_score_then_index():
    rng = random.Random(9)
    pairs = [(rng.randrange(0, 1 << 22), rng.randrange(0, 1 << 40)) for _ in range(300)]
    pairs += [(5, 0), (5, (1 << 40) - 1), (0, 0), ((1 << 23) - 1, 7)]
    for s1, i1 in pairs[:60]:
        for s2, i2 in pairs:
            better = s1 > s2 or (s1 == s2 and i1 < i2)
            assert (O.pack_best(s1, i1) > O.pack_best(s2, i2)) == better
    for s, i in pairs:
        assert O.unpack_best(O.pack_best(s, i)) == (s, i) and 0 <= O.pack_best(s, i) < 2 ** 63


# ---- planted mistakes: each must fail at least one pin above ------------------------------------
def _strict_fit(indices, cfg, rows, m_total):
    return _ORIGINAL(indices, cfg, rows, m_total - 1)


def _tp_scored_like_dp(method, bs, gpu_n):
    return [3 * bs * gpu_n, 2 * bs * gpu_n, 2 * bs * gpu_n][method]


def _cdp_without_bonus(method, bs, gpu_n):
    return [2 * bs * gpu_n, 2 * bs * gpu_n, 2 * bs][method]


def _pack_prefers_high_index(score2, index):
    return (score2 << 40) | index


_ORIGINAL = O.sweep_rows
MUTANTS = {
    "fit_is_strict": ("sweep_rows", _strict_fit),
    "tp_scored_like_dp": ("config_score2", _tp_scored_like_dp),
    "cdp_without_bonus": ("config_score2", _cdp_without_bonus),
    "ties_to_the_highest_index": ("pack_best", _pack_prefers_high_index),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistakes(name, golden, monkeypatch):
    attr, fn = MUTANTS[name]
    monkeypatch.setattr(O, attr, fn)
    failures = 0
    for pin in (lambda: test_worked_sweep(golden), lambda: test_sweep_against_selection_and_sorting(1),
                test_packed_best_orders_like_score_then_index):
        try:
            pin()
        except AssertionError:
            failures += 1
    assert failures > 0
