"""Parity of the HIP path with the CPU oracle for the estimates of all four
methods (incl. DP+TP, Sec. 5) and the method decision (Sec. 6, Algorithm 1):
element by element and bit exact, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import llmem_oracle as A
from oracle import oracle_c as B
from workloads import grids as G
from workloads import tables as T

pytestmark = pytest.mark.gpu

CONST = T.Constants(m_base=256 << 20)
GIB = 1 << 30


@pytest.fixture(scope="module")
def U():
    import gpu_util
    return gpu_util


def _check_methods(U, cfg, tp, tables, const=CONST, threads=8):
    want_p, want_f = B.method_peaks(cfg, np.zeros(len(cfg["h"]), np.uint8) if tp is None else tp, tables, const,
                                    threads=threads)
    got_p, got_f = U.hip_methods(cfg, tp, tables, const)
    U.assert_same("method peaks", got_p, want_p)
    U.assert_same("method flags", got_f, want_f)
    got_p2, none = U.hip_methods(cfg, tp, tables, const, flags=False)
    assert none is None
    U.assert_same("method peaks, no flags", got_p2, want_p)


def _check_decide(U, cfg, tp, tables, m_total, const=CONST, threads=8):
    want = B.decide(cfg, np.zeros(len(cfg["h"]), np.uint8) if tp is None else tp, tables, const, m_total,
                    threads=threads)
    method, bs, rows = U.hip_decide(cfg, tp, tables, const, m_total)
    U.assert_same(f"decision rows (m_total {m_total})", rows, want)
    U.assert_same("method", method, want[:, A.C_METHOD])
    U.assert_same("bs", bs, want[:, A.C_BS])
    method2, bs2, none = U.hip_decide(cfg, tp, tables, const, m_total, detail=False)
    assert none is None
    U.assert_same("method, no detail", method2, want[:, A.C_METHOD])
    U.assert_same("bs, no detail", bs2, want[:, A.C_BS])
    _, _, rows3 = U.hip_decide(cfg, tp, tables, const, m_total, short=False)
    U.assert_same("detail alone", rows3, want)
    return want


def _one(**kw):
    base = dict(arch_id=0, h=256, L=4, n_heads=4, n_kv=4, ffn=1024, V=8192, P=512, bs=64, sl=256, method=0, d=4,
                chunk_k=4, flags=G.FLAG_GRAD_ALIAS)
    base.update(kw)
    return {k: np.asarray([v]).astype(G.FIELD_DTYPE[k]) for k, v in base.items()}


def test_worked_example_through_the_hip_path(U, golden):
    """The hand-worked values of tests/golden directly, not via the oracle."""
    g = golden("worked_decision_gpt_tiny.txt")
    gpt, c0 = [T.gpt_table()], T.Constants(m_base=0)
    ex = golden("worked_example_gpt_tiny.txt")
    for tp in (2, 4):
        p, f = U.hip_methods(_one(bs=4), np.asarray([tp], np.uint8), gpt, c0)
        assert p[0].tolist() == [ex["peak_cdp"], ex["peak_zero3_d4"], ex["peak_tp_d4"], g[f"hybrid_tp{tp}_bs4"]]
        assert bool(f[0] & A.HYBRID_READINGS_DIFFER) == bool(g[f"hybrid_tp{tp}_readings_differ"])
    _, _, r = U.hip_decide(_one(), np.asarray([2], np.uint8), gpt, c0, g["case1_m_total"])
    assert r[0].tolist() == [g["case1_method"], g["case1_bs"], g["case1_bs_cdp"], g["case1_bs_adp"], g["case1_bs_tp"],
                             g["case1_bs_hybrid"], g["case1_score2_cdp"], g["case1_score2_adp"], g["case1_score2_tp"],
                             g["case1_score2_hybrid"], g["case1_peak"], 0]
    _, _, r = U.hip_decide(_one(), np.asarray([2], np.uint8), gpt, c0, g["case2_m_total"])
    assert r[0].tolist() == [g["case2_method"], g["case2_bs"], 0, 0, g["case2_bs_tp"], g["case2_bs_hybrid"], 0, 0, 4, 4,
                             g["case2_peak"], 0]
    _, _, r = U.hip_decide(_one(), np.asarray([2], np.uint8), gpt, c0, g["case3_m_total"])
    assert r[0].tolist() == [4, 0] + [0] * 10
    m, b, r = U.hip_decide(_one(), np.asarray([4], np.uint8), gpt, c0, g["case4_m_total"])
    assert (m[0], b[0]) == (4, 0) and r[0][A.C_BS_HYBRID] == 1 and r[0][A.C_SCORE2_HYBRID] == 2
    assert r[0][A.C_FLAGS] == A.HYBRID_READINGS_DIFFER | A.FALLBACK_READINGS_DIFFER


def test_grid1_configurations_all_methods(U):
    cfg = G.grid1()
    n = len(cfg["h"])
    d = cfg["d"].astype(int)
    divisors = {g: [t for t in range(1, g + 1) if g % t == 0] for g in set(d.tolist())}
    tp = np.asarray([divisors[g][i % len(divisors[g])] for i, g in enumerate(d.tolist())], dtype=np.uint8)
    _check_methods(U, cfg, tp, [T.gpt_table()])
    # and directly against the Python oracle that carries the pins
    names = list(cfg.keys())
    want = np.asarray([A.method_peaks({k: int(cfg[k][i]) for k in names}, int(tp[i]), [T.gpt_table()], CONST)
                       for i in range(n)], dtype=np.int64)
    got_p, got_f = U.hip_methods(cfg, tp, [T.gpt_table()], CONST)
    U.assert_same("peaks vs oracle A", got_p, want[:, :4])
    U.assert_same("flags vs oracle A", got_f, want[:, 4])
    cfg["bs"][:] = 24
    for m_total in (300 << 20, 420 << 20, 700 << 20):
        rows = _check_decide(U, cfg, tp, [T.gpt_table()], m_total)
        want_a = np.asarray([A.decide_one({k: int(cfg[k][i]) for k in names}, int(tp[i]), [T.gpt_table()], CONST, m_total)
                             for i in range(0, n, 7)], dtype=np.int64)
        U.assert_same("decision vs oracle A", rows[::7], want_a)


@pytest.mark.parametrize("n,first", [(64 * 150 + 37, 0), (64 * 40 + 1, 900_000)])
def test_query_grid_slices(U, n, first):
    """Seeded slices of the decision grid: several tiles and a ragged tail."""
    tables = [T.llama_table()]
    cfg, tp = G.grid6(n=n, seed=0, first=first)
    as_cfg = dict(cfg)
    as_cfg["bs"] = (np.arange(n) % 67).astype(np.uint16)
    _check_methods(U, as_cfg, tp, tables, threads=16)
    seen = set()
    for m_total in (16 * GIB, 80 * GIB, 288 * GIB):
        rows = _check_decide(U, cfg, tp, tables, m_total, threads=16)
        seen |= set(rows[:, A.C_METHOD].tolist())
    assert seen == {0, 1, 2, 3, 4}
    _check_decide(U, cfg, None, tables, 80 * GIB, threads=16)            # no DP+TP set-up anywhere


def test_random_tables_wild_queries(U):
    """Several architectures mixed inside a wavefront, invalid and degenerate fields, tp_n that is 0
    or does not divide gpu_n."""
    rng = np.random.default_rng(21)
    tabs = [T.random_table(rng, 9, 0, "r0"), T.gpt_table(), T.random_table(rng, 0, 0, "empty"),
            T.random_table(rng, 64, 0, "r3"), T.llama_table(), T.random_table(rng, 1, 0, "one"), T.opt_table(),
            T.random_table(rng, 30, 0, "r7")]
    cfg, tp = G.random_queries(rng, 64 * 30 + 11, n_arch=len(tabs), wild=True, bs_cap=40)
    for const in (T.Constants(m_base=1, cu_p=4096, align=512), T.Constants(m_base=12345, cu_p=1 << 16, align=1),
                  T.Constants(m_base=0, cu_p=2 << 20, align=512)):
        _check_methods(U, cfg, tp, tabs, const)
        peaks, _ = B.method_peaks(cfg, tp, tabs, const, threads=8)
        ok = peaks[:, 0] >= 0
        for m_total in (0, int(np.percentile(peaks[ok, 2], 30)), int(np.median(peaks[ok, 0])), 1 << 62, -5):
            _check_decide(U, cfg, tp, tabs, m_total, const)


def test_ragged_and_empty_inputs(U):
    tables = [T.llama_table()]
    for n in (0, 1, 63, 64, 65, 257):
        cfg, tp = G.grid6(n=n, seed=5, first=1000)
        cfg["bs"] = (cfg["bs"] % 100).astype(np.uint16)
        _check_methods(U, cfg, tp, tables)
        _check_decide(U, cfg, tp, tables, 40 * GIB)


def test_large_batch_size_caps(U):
    """Caps up to 65535 (16 bits of the search) on small models whose answers are large."""
    tables = [T.gpt_table()]
    rng = np.random.default_rng(3)
    n = 80
    cfg = {k: np.repeat(v, n) for k, v in _one(h=64, L=2, n_heads=1, n_kv=1, ffn=256, V=1000, P=16, sl=16).items()}
    cfg["bs"] = rng.choice([65535, 65534, 32768, 32767, 4097, 255, 1, 0], size=n).astype(np.uint16)
    cfg["d"] = rng.choice([1, 2, 4, 8], size=n).astype(np.uint8)
    tp = np.where(rng.random(n) < 0.5, 1, cfg["d"]).astype(np.uint8)
    c0 = T.Constants(m_base=0)
    for m_total in (40 << 20, 900 << 20, 1 << 50):
        rows = _check_decide(U, cfg, tp, tables, m_total, c0, threads=16)
    assert rows[:, A.C_BS].max() == 65535                                  # the cap itself is reached
    rows = _check_decide(U, cfg, tp, tables, 2 * GIB, c0, threads=16)
    assert ((rows[:, A.C_BS_CDP] > 4097) & (rows[:, A.C_BS_CDP] < 32767)).any()


def _size_expressions(table):
    return {(p.coef, tuple(sorted(d for d in p.dims if d != "one"))) for p in table.params}


def test_entry_form_census_and_byte_form_probes(U):
    """The forms the kernel falls back to: tables with more distinct parameter sizes than travel
    in the kernel arguments (census entry by entry), and queries whose page counts pass 2^31 at
    their cap or whose page is above 2^31 bytes (probes in bytes)."""
    rng = np.random.default_rng(33)
    tabs = [T.random_table(rng, 64, 0, f"r{j}") for j in range(8)]
    assert sum(len(_size_expressions(t)) for t in tabs) > 200
    cfg, tp = G.random_queries(rng, 64 * 12 + 5, n_arch=len(tabs), wild=True, bs_cap=300)
    const = T.Constants(m_base=77, cu_p=1 << 14, align=64)
    _check_methods(U, cfg, tp, tabs, const)
    peaks, _ = B.method_peaks(cfg, tp, tabs, const, threads=8)
    ok = peaks[:, 0] >= 0
    for m_total in (int(np.percentile(peaks[ok, 2], 40)), int(np.median(peaks[ok, 1])), 1 << 55):
        _check_decide(U, cfg, tp, tabs, m_total, const)

    tables = [T.llama_table()]
    n = 64 * 9 + 3
    cfg, tp = G.grid6(n=n, seed=12, first=500)
    cfg["bs"] = rng.choice([65535, 40000, 4096, 300, 7, 1, 0], size=n).astype(np.uint16)
    small_page = T.Constants(m_base=3, cu_p=512, align=512)
    beyond = (((cfg["L"].astype(np.int64) + 1) * cfg["sl"] * cfg["h"] * 2) >> 9) * cfg["bs"] >= 1 << 31
    assert beyond.any() and not beyond.all()
    for m_total in (80 * GIB, 1 << 41, 1 << 45):
        rows = _check_decide(U, cfg, tp, tables, m_total, small_page, threads=16)
    assert rows[:, A.C_BS].max() == 65535
    huge_page = T.Constants(m_base=0, cu_p=1 << 33, align=512)
    for m_total in (400 * GIB, 1 << 41, 1 << 44):
        _check_decide(U, cfg, tp, tables, m_total, huge_page, threads=16)
    cfg["bs"] = np.minimum(cfg["bs"], 900).astype(np.uint16)               # the page form again, small pages
    for m_total in (80 * GIB, 1 << 40):
        _check_decide(U, cfg, tp, tables, m_total, T.Constants(m_base=3, cu_p=4096, align=512), threads=16)


def test_capacities_at_the_edge_of_a_batch_size(U):
    """m_total equal to an estimate at some batch size, and one byte either side of it, for batch
    sizes up to the 16-bit cap: where a bracket that is off by one would show.  The oracle's
    estimates at the answers decide: the answer fits, the next batch size does not."""
    tables = [T.gpt_table()]
    rng = np.random.default_rng(44)
    n = 128
    cfg = {k: np.repeat(v, n) for k, v in _one(h=64, L=2, n_heads=1, n_kv=1, ffn=256, V=1000, P=16, sl=16).items()}
    cfg["h"] = (64 * rng.integers(1, 5, size=n)).astype(np.uint32)
    cfg["L"] = rng.integers(1, 6, size=n).astype(np.uint16)
    cfg["sl"] = rng.choice([1, 2, 16, 100, 128], size=n).astype(np.uint16)
    cfg["V"] = rng.choice([1000, 1024, 32768], size=n).astype(np.uint32)
    cfg["d"] = rng.choice([1, 2, 3, 4, 8, 16], size=n).astype(np.uint8)
    cfg["bs"] = np.full(n, 65535, np.uint16)
    tp = np.where(rng.random(n) < 0.5, 1, cfg["d"]).astype(np.uint8)
    const = T.Constants(m_base=12345)

    def peaks_at(bs):
        at = dict(cfg)
        at["bs"] = bs.astype(np.uint16)
        return B.method_peaks(at, tp, tables, const, threads=8)[0]

    capacities = set()
    for b in (1, 2, 999, 4097, 30000, 65534, 65535):
        p = peaks_at(np.full(n, b))
        for j, m in zip(rng.integers(0, n, size=3), rng.integers(0, 4, size=3)):
            capacities |= {int(p[j, m]) - 1, int(p[j, m]), int(p[j, m]) + 1}
    assert len(capacities) > 50
    for m_total in sorted(capacities):
        _, _, rows = U.hip_decide(cfg, tp, tables, const, m_total)
        for m in range(4):
            best = rows[:, A.C_BS_CDP + m]
            assert ((best >= 0) & (best <= 65535)).all()
            here, above = peaks_at(best)[:, m], peaks_at(np.minimum(best + 1, 65535))[:, m]
            assert ((here <= m_total) | (best == 0)).all(), (m_total, m)
            assert ((above > m_total) | (best == 65535)).all(), (m_total, m)
            first = peaks_at(np.ones(n))[:, m]
            assert ((best > 0) | (first > m_total)).all(), (m_total, m)


def test_determinism_and_stream(U):
    tables = [T.llama_table()]
    cfg, tp = G.grid6(n=5000, seed=9, first=0)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        a = U.hip_decide(cfg, tp, tables, CONST, 80 * GIB, stream=s)
    b = U.hip_decide(cfg, tp, tables, CONST, 80 * GIB)
    U.assert_same("decision twice", a[2], b[2])


def test_queries_generator(U):
    import paper_2404_10933_amd as M
    for n, first, seed in ((100_001, 0, 0), (4097, 123_456_789, 77)):
        want, want_tp = G.grid6(n=n, seed=seed, first=first)
        dev = M.DeviceConfigs.empty(n)
        tp = torch.empty(n, dtype=torch.uint8, device="cuda")
        M.llmem_queries_generate(seed, first, n, dev, tp)
        torch.cuda.synchronize()
        got = dev.to_numpy()
        for k in want:
            assert got[k].dtype == want[k].dtype and (got[k] == want[k]).all(), k
        assert (tp.cpu().numpy() == want_tp).all()


def test_outputs_beyond_four_gib(U):
    """45 000 019 queries generated on the device: the decision columns take 4.3 GB, the last of
    them beyond 2^32 bytes from the start of the output.  Slices at the start, in the middle and
    at the ragged end against the oracle; everywhere else the fill value must be gone."""
    import paper_2404_10933_amd as M
    n, m_total = 45_000_019, 80 * GIB
    tables = [T.llama_table()]
    dev = M.DeviceConfigs.empty(n)
    tp = torch.empty(n, dtype=torch.uint8, device="cuda")
    M.llmem_queries_generate(3, 0, n, dev, tp)
    tab = M.Tables(tables, m_base=CONST.m_base, cu_p=CONST.cu_p, align=CONST.align)
    method = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    bs = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    det = torch.full((M.NDECIDE, n), -7, dtype=torch.int64, device="cuda")
    assert det.numel() * 8 > (1 << 32)
    M.llmem_decide(dev, tp, tab, m_total, method, bs, det)
    torch.cuda.synchronize()
    for first, m in ((0, 700), (n // 2 - 300, 700), (n - 723, 723)):
        cfg, tp_np = G.grid6(n=m, seed=3, first=first)
        want = B.decide(cfg, tp_np, tables, CONST, m_total, threads=16)
        U.assert_same(f"decision rows from {first}", det[:, first:first + m].cpu().numpy().T, want)
        U.assert_same(f"method from {first}", method[first:first + m].cpu().numpy(), want[:, A.C_METHOD])
        U.assert_same(f"bs from {first}", bs[first:first + m].cpu().numpy(), want[:, A.C_BS])
    assert int((method == -7).sum().item()) == 0 and int((bs == -7).sum().item()) == 0
    for c in range(M.NDECIDE):
        assert int((det[c] == -7).sum().item()) == 0, c
    # the four estimates at once: 4 columns of 360 MB
    del det
    peaks = torch.full((4, n), -7, dtype=torch.int64, device="cuda")
    M.llmem_estimate_methods(dev, tp, tab, peaks)
    torch.cuda.synchronize()
    first, m = n - 723, 723
    cfg, tp_np = G.grid6(n=m, seed=3, first=first)
    U.assert_same("estimates of the four methods at the end", peaks[:, first:].cpu().numpy().T,
                  B.method_peaks(cfg, tp_np, tables, CONST, threads=8)[0])
    assert int((peaks == -7).sum().item()) == 0


def test_full_size_decision_grid(U):
    """4 * 10^6 queries generated on the device, in the launch configuration the benchmark times:
    sampled queries against the oracle; for all of them the properties that define the result."""
    import paper_2404_10933_amd as M
    n, m_total = 4_000_000, 80 * GIB
    tables = [T.llama_table()]
    dev = M.DeviceConfigs.empty(n)
    tp = torch.empty(n, dtype=torch.uint8, device="cuda")
    M.llmem_queries_generate(0, 0, n, dev, tp)
    tab = M.Tables(tables, m_base=CONST.m_base, cu_p=CONST.cu_p, align=CONST.align)
    method = torch.empty(n, dtype=torch.int32, device="cuda")
    bs = torch.empty(n, dtype=torch.int32, device="cuda")
    det = torch.empty((M.NDECIDE, n), dtype=torch.int64, device="cuda")
    M.llmem_decide(dev, tp, tab, m_total, method, bs, det)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    idx = np.unique(np.concatenate([np.arange(256), np.arange(n - 256, n), rng.integers(0, n, size=6000)]))
    cfg, tp_np = G.grid6(n=n, seed=0)
    want = B.decide(G.slice_configs(cfg, idx), tp_np[idx], tables, CONST, m_total, threads=16)
    got = det[:, torch.from_numpy(idx).cuda()].cpu().numpy().T
    U.assert_same("decision rows, sampled", got, want)
    # properties over all queries, checked with the estimator kernel itself: each method's batch size
    # fits, the next one does not (or the cap is reached)
    rows = det.cpu().numpy()
    assert (rows[A.C_METHOD] == method.cpu().numpy()).all() and (rows[A.C_BS] == bs.cpu().numpy()).all()
    assert ((rows[A.C_METHOD] >= 0) & (rows[A.C_METHOD] <= 4)).all()
    peaks = torch.empty((4, n), dtype=torch.int64, device="cuda")
    for m in range(4):
        for step, fits in ((0, True), (1, False)):
            col = rows[A.C_BS_CDP + m] + step
            probe = (col > 0) & (col <= G.QUERY_BS_CAP)
            dev.columns["bs"].copy_(torch.from_numpy(np.where(probe, col, 1).astype(np.uint16)).cuda())
            M.llmem_estimate_methods(dev, tp, tab, peaks)
            torch.cuda.synchronize()
            p = peaks[m].cpu().numpy()
            assert ((p <= m_total) == fits)[probe].all(), (m, step)
            if step == 0:
                chosen = probe & (rows[A.C_METHOD] == m)
                assert (p[chosen] == rows[A.C_PEAK][chosen]).all()
