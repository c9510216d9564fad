"""Oracle B (C, int64 with overflow checks) restates oracle A (Python, unbounded
integers): the two must agree on every detail column, on whole grid 1, on seeded
samples of grids 2-4, on random tables with wild configurations and on explicit
event lists, and on the DP+TP estimate and the method decision for seeded and
random queries.  Oracle A carries the pins; this extends them to B."""
import numpy as np
import pytest

from oracle import llmem_oracle as A
from oracle import oracle_c as B
from workloads import events as E
from workloads import grids as G
from workloads import tables as T

CONST = T.Constants(m_base=256 << 20)


def _same(cfg, tables, const=CONST):
    rows = np.asarray(A.estimate(cfg, tables, const), dtype=np.int64)
    peaks, detail = B.estimate(cfg, tables, const, threads=4)
    assert (rows == detail).all()
    assert (peaks == detail[:, 0]).all()
    p2, _ = B.estimate(cfg, tables, const, timeline=False, want_detail=False)
    assert (p2 == peaks).all()


def test_grid1_all_configs():
    g = G.grid1()
    assert len(g["h"]) == 432
    _same(g, [T.gpt_table()])


@pytest.mark.parametrize("name,n", [("g2", 120), ("g3", 60), ("g4", 60)])
def test_grid_samples(name, n):
    spec = G.GRIDS[name]
    first = 12345 if name != "g1" else 0
    _same(spec["make"](n=n, seed=0, first=first), [T.FAMILIES[spec["family"]]()])


def test_random_tables_wild_configs():
    rng = np.random.default_rng(7)
    tabs = [T.random_table(rng, 9, 150, "r0"), T.llama_table(), T.random_table(rng, 0, 0, "empty"),
            T.random_table(rng, 64, 700, "r3")]
    cfg = G.random_configs(rng, 300, n_arch=len(tabs), wild=True)
    _same(cfg, tabs, T.Constants(m_base=1, cu_p=4096, align=512))
    _same(cfg, tabs, T.Constants(m_base=0, cu_p=2 << 20, align=512))


def test_event_lists():
    ev, off = E.generate(40, seed=3, first=7)
    a1, r1 = A.event_lists_peaks(ev, off)
    a2, r2 = B.event_lists_peaks(ev, off, threads=3)
    assert (np.asarray(a1) == a2).all() and (np.asarray(r1) == r2).all()
    ev, off = E.from_lists([[], [5], [-5, 5], [2097152, 1, -2097152], []])
    a1, r1 = A.event_lists_peaks(ev, off)
    a2, r2 = B.event_lists_peaks(ev, off)
    assert list(a2) == a1 and list(r2) == r1


def _rows_a(cfg, tp, fn):
    names = list(cfg.keys())
    return np.asarray([fn({k: int(cfg[k][i]) for k in names}, int(tp[i])) for i in range(len(tp))], dtype=np.int64)


def test_method_peaks_and_decision_on_query_grid():
    tabs = [T.llama_table()]
    cfg, tp = G.grid6(n=40, seed=0, first=777)
    cfg["bs"] = (cfg["bs"] % 7).astype(np.uint16)                       # as configurations: small batch sizes
    peaks, flags = B.method_peaks(cfg, tp, tabs, CONST, threads=2)
    want = _rows_a(cfg, tp, lambda c, t: A.method_peaks(c, t, tabs, CONST))
    assert (peaks == want[:, :4]).all() and (flags == want[:, 4]).all()
    cfg["bs"][:] = 40                                                   # as queries: batch sizes up to 40
    for m_total in (24 << 30, 80 << 30):
        rows = B.decide(cfg, tp, tabs, CONST, m_total, threads=2)
        want = _rows_a(cfg, tp, lambda c, t: A.decide_one(c, t, tabs, CONST, m_total))
        assert (rows == want).all()
        assert len(set(rows[:, A.C_METHOD])) >= 3


def test_method_peaks_and_decision_random_tables_wild_queries():
    rng = np.random.default_rng(11)
    tabs = [T.random_table(rng, 9, 0, "r0"), T.gpt_table(), T.random_table(rng, 0, 0, "empty"),
            T.random_table(rng, 40, 0, "r3")]
    cfg, tp = G.random_queries(rng, 250, n_arch=len(tabs), wild=True, bs_cap=10)
    for const in (T.Constants(m_base=1, cu_p=4096, align=512), T.Constants(m_base=0, cu_p=2 << 20, align=512)):
        peaks, flags = B.method_peaks(cfg, tp, tabs, const)
        want = _rows_a(cfg, tp, lambda c, t: A.method_peaks(c, t, tabs, const))
        assert (peaks == want[:, :4]).all() and (flags == want[:, 4]).all()
        valid = peaks[:, 0] >= 0
        for m_total in (0, int(np.median(peaks[valid, 1])), int(np.median(peaks[valid, 0])), 1 << 62):
            rows = B.decide(cfg, tp, tabs, const, m_total, threads=3)
            want = _rows_a(cfg, tp, lambda c, t: A.decide_one(c, t, tabs, const, m_total))
            assert (rows == want).all()
    assert (flags & A.ERR_TP).any() and (peaks[:, 3] == -1).any()


def test_sweep_statistics():
    """Oracle B's sweep against oracle A's, on grids and on unstructured configurations with
    invalid ones among them, for capacities that let all, some and none fit."""
    cases = [(G.grid1(), 0, [T.gpt_table()]), (G.grid4(n=150, seed=2, first=77), 77, [T.llama_table()])]
    rng = np.random.default_rng(11)
    wild = G.random_configs(rng, 200, n_arch=2, wild=True)
    wild["d"] = np.minimum(wild["d"], 18).astype(wild["d"].dtype)
    cases.append((wild, (1 << 40) - 200, [T.gpt_table(), T.llama_table()]))
    for cfg, first, tabs in cases:
        rows = A.estimate(cfg, tabs, CONST)
        n = len(rows)
        peaks = sorted(r[A.D_PEAK] for r in rows if r[A.D_PEAK] >= 0)
        for m_total in (peaks[len(peaks) // 2], peaks[-1], peaks[0] - 1, peaks[0]):
            a = A.sweep_rows(range(first, first + n), cfg, rows, m_total)
            b = B.sweep(cfg, first, tabs, CONST, m_total, threads=2)
            assert b.shape == (A.NSWEEP, A.SWEEP_GROUPS) and b.tolist() == a
    with pytest.raises(ValueError):
        B.sweep(G.grid1(), (1 << 40) - 431, [T.gpt_table()], CONST, 1 << 40)


def test_decision_rejects_batch_dependent_parameters():
    t = T.ArchTable("odd", (T.ParamEntry("w", 1, ("h", "bs"), "L", "OTHER", False),), ())
    cfg, tp = G.random_queries(np.random.default_rng(0), 4)
    with pytest.raises(ValueError):
        B.decide(cfg, tp, [t], CONST, 1 << 40)


def test_oracle_b_reports_overflow():
    t = T.ArchTable("big", (), (T.EventEntry("x", "A", +1, 2**31, ("V", "V", "V", "V"), 8),))
    cfg = G.random_configs(np.random.default_rng(0), 4)
    cfg["V"][:] = 200000
    with pytest.raises(OverflowError):
        B.estimate(cfg, [t], CONST)
