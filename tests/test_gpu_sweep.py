"""Parity of the streaming sweep (configurations drawn, estimated and folded into
statistics per (method, gpu_n) inside one kernel) with the CPU oracle: every
statistic of every group, bit exact, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import llmem_oracle as A
from oracle import oracle_c as B
from workloads import grids as G
from workloads import tables as T

pytestmark = pytest.mark.gpu

CONST = T.Constants(m_base=256 << 20)
CONST0 = T.Constants(m_base=0)
GIB = 1 << 30
KERNEL_LANE_EVENTS, KERNEL_LANE_COMPILED, KERNEL_LANE_SPECIALIZED, KERNEL_LANE_RUNTIME, KERNEL_LANE_DIRECT = 3, 4, 5, 6, 7   # LLMEM_KERNEL_*
GRIDS = {1: (G.grid1, "gpt"), 2: (G.grid2, "opt"), 3: (G.grid3, "llama"), 4: (G.grid4, "llama")}


@pytest.fixture(scope="module")
def U():
    import gpu_util
    return gpu_util


def _grid(grid_id, n, seed, first):
    if grid_id == 1:
        return G.slice_configs(G.grid1(), np.arange(first, first + n))
    return GRIDS[grid_id][0](n=n, seed=seed, first=first)


def _check(U, grid_id, seed, first, n, m_total, const=CONST, tables=None, kernel=0, threads=8):
    tables = tables or [T.FAMILIES[GRIDS[grid_id][1]]()]
    want = B.sweep(_grid(grid_id, n, seed, first), first, tables, const, m_total, threads=threads)
    got = U.hip_sweep(grid_id, seed, first, n, tables, const, m_total, kernel=kernel)
    for c, name in enumerate(("count", "fit", "max_peak", "min_peak", "max_live", "best", "k_sum", "max_nparams_fit")):
        U.assert_same(f"grid {grid_id} n {n} first {first} m_total {m_total}: {name}", got[c], want[c])
    return want


def test_worked_example_through_the_hip_path(U, golden):
    """The hand-worked values of tests/golden directly, not via the oracle."""
    g = golden("worked_sweep_gpt_tiny.txt")
    s = U.hip_sweep(1, 0, 0, 432, [T.gpt_table()], CONST0, g["m_total"])
    for method, d, name in ((0, 1, "cdp"), (0, 4, "cdp"), (1, 3, "adp3"), (2, 4, "tp4")):
        q = method * 16 + d - 1
        assert (s[A.S_COUNT][q], s[A.S_K_SUM][q], s[A.S_MAX_NPARAMS_FIT][q]) == (g["count"], g["k_sum"], g["n_params"])
        assert (s[A.S_FIT][q], s[A.S_MAX_PEAK][q], s[A.S_MIN_PEAK][q]) == (
            g[f"{name}_fit"], g[f"{name}_max_peak"], g[f"{name}_min_peak"])
    for q, name in ((0, "cdp1"), (1, "cdp2"), (16 + 2, "adp3"), (32 + 3, "tp4")):
        assert A.unpack_best(int(s[A.S_BEST][q])) == (g[f"{name}_best_score2"], g[f"{name}_best_index"])
    s = U.hip_sweep(1, 0, 0, 432, [T.gpt_table()], CONST0, g["tight_m_total"])
    q = 32 + 3
    assert (s[A.S_FIT][q], s[A.S_BEST][q], s[A.S_MAX_NPARAMS_FIT][q], s[A.S_MIN_PEAK][q]) == (
        0, 0, 0, g["tp4_min_peak"])


def test_grid1_whole_and_in_parts(U):
    for m_total in (190_840_832 + (256 << 20), 1 << 40, 0, -1):
        _check(U, 1, 0, 0, 432, m_total)
    _check(U, 1, 0, 0, 432, 190_840_832, const=CONST0)
    _check(U, 1, 0, 400, 32, 300 << 20)
    _check(U, 1, 0, 63, 130, 300 << 20)           # ragged at both ends of a wave's 64


@pytest.mark.parametrize("grid_id,n", ((2, 20_000), (3, 30_000), (4, 30_000)))
def test_random_grids(U, grid_id, n):
    """Several workgroups' worth of batches and a ragged tail, capacities from 'nothing fits' to
    'everything fits', a second seed, a range that does not start at 0."""
    for seed, first, m_total in ((0, 0, 40 * GIB), (0, 0, 2 * GIB), (0, 0, 1 << 50), (7, 123_456_789, 80 * GIB)):
        want = _check(U, grid_id, seed, first, n + 37, m_total)
    assert want[A.S_COUNT].sum() == n + 37 and 0 < want[A.S_FIT].sum() < n + 37


def test_events_form_of_the_kernel(U):
    _check(U, 4, 0, 0, 5_000, 40 * GIB, kernel=KERNEL_LANE_EVENTS)
    _check(U, 1, 0, 0, 432, 300 << 20, kernel=KERNEL_LANE_EVENTS)
    # and with every event evaluated where it stands (what tables with very many distinct sizes get)
    _check(U, 4, 0, 0, 5_000, 40 * GIB, kernel=KERNEL_LANE_DIRECT)
    _check(U, 1, 0, 0, 432, 300 << 20, kernel=KERNEL_LANE_DIRECT)
    rng = np.random.default_rng(23)
    _check(U, 2, 5, 1000, 3_000, 10 * GIB, tables=[T.random_table(rng, 20, 300, "many sizes")], kernel=0)


@pytest.mark.parametrize("grid_id,n", ((1, 432), (2, 20_000), (4, 30_037)))
def test_specialized_form_of_the_kernel(U, grid_id, n):
    """The sweep with the tables as constants: the kernel built into the library for the shipped
    tables, the same built at run time, and the form that reads the compiled tables from its
    arguments; a table set the library does not ship gets a run-time build of its own."""
    for seed, first, m_total in ((0, 0, 40 * GIB), (7, 123_456_789 if grid_id > 1 else 0, 2 * GIB)):
        for kernel in (KERNEL_LANE_SPECIALIZED, KERNEL_LANE_RUNTIME, KERNEL_LANE_COMPILED):
            _check(U, grid_id, seed, first, n, m_total, kernel=kernel)
    if grid_id == 4:
        for kernel in (KERNEL_LANE_SPECIALIZED, KERNEL_LANE_RUNTIME):
            _check(U, 4, 3, 0, 8_000, 60 * GIB, tables=[T.llama_table(checkpoint=False)], kernel=kernel)
        # several architectures in one specialization (the grids draw architecture 0 only): the shipped
        # set of three, and a pair that is built at run time
        _check(U, 2, 3, 0, 8_000, 60 * GIB, tables=[T.gpt_table(), T.opt_table(), T.llama_table()], kernel=0)
        _check(U, 4, 3, 0, 8_000, 60 * GIB, tables=[T.llama_table(), T.gpt_table()], kernel=KERNEL_LANE_SPECIALIZED)


def test_full_traversal_tables_and_second_architecture_unused(U):
    _check(U, 4, 3, 0, 8_000, 60 * GIB, tables=[T.llama_table(checkpoint=False), T.gpt_table()])


def test_accumulates_over_ranges_and_streams(U):
    """llmem_sweep adds to what the array holds: four consecutive ranges (one of them empty) on
    a side stream give the statistics of the whole; index limits."""
    import paper_2404_10933_amd as M
    tables = [T.llama_table()]
    n, m_total = 50_000, 40 * GIB
    want = B.sweep(G.grid4(n=n, seed=5, first=1000), 1000, tables, CONST, m_total, threads=8)
    stream = torch.cuda.Stream()
    stats = torch.full((M.NSWEEP, M.SWEEP_GROUPS), -7, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        M.llmem_sweep_reset(stats, stream=stream)
        for lo, hi in ((0, 1), (1, 20_001), (20_001, 20_001), (20_001, n)):
            U.hip_sweep(4, 5, 1000 + lo, hi - lo, tables, CONST, m_total, into=stats, stream=stream)
    torch.cuda.synchronize()
    U.assert_same("accumulated", stats.cpu().numpy(), want)
    # the last representable indices
    first = (1 << 40) - 1000
    _check(U, 4, 1, first, 1000, 40 * GIB)
    tab = M.Tables(tables, m_base=CONST.m_base)
    with pytest.raises(M.LlmemError):
        M.llmem_sweep(4, 1, first, 1001, tab, m_total, stats)
    with pytest.raises(M.LlmemError):
        M.llmem_sweep(6, 1, 0, 10, tab, m_total, stats)


def test_a_grid_that_would_not_fit_in_memory(U):
    """2 * 10^9 configurations (62 GB of columns and 208 GB of detail output if they were stored):
    every configuration is counted, the halves add up to the whole (counts add, extremes
    combine), and the oracle confirms a slice in the middle exactly."""
    tables = [T.llama_table()]
    n, m_total = 2_000_000_000, 64 * GIB
    whole = U.hip_sweep(4, 0, 0, n, tables, CONST, m_total, kernel=KERNEL_LANE_SPECIALIZED)
    assert whole[A.S_COUNT].sum() == n and 0 < whole[A.S_FIT].sum() < n
    low = U.hip_sweep(4, 0, 0, n // 2, tables, CONST, m_total, kernel=KERNEL_LANE_SPECIALIZED)
    high = U.hip_sweep(4, 0, n // 2, n // 2, tables, CONST, m_total, kernel=KERNEL_LANE_SPECIALIZED)
    U.assert_same("halves merged", np.array(A.sweep_merge(low.tolist(), high.tolist())), whole)
    _check(U, 4, 0, 1_234_567_890, 50_000, m_total, kernel=KERNEL_LANE_SPECIALIZED)


def test_full_size_grid4(U):
    """10^7 configurations in the benchmark's launch configurations (the kernel built at run time
    and the built-in one): every statistic of every group against the oracle's sweep of the whole
    grid, and the best entries of a few groups confirmed one by one by oracle A."""
    tables = [T.llama_table()]
    n, m_total = 10_000_000, 64 * GIB
    want = B.sweep(G.grid4(n=n, seed=0), 0, tables, CONST, m_total, threads=16)
    assert want[A.S_COUNT].sum() == n
    for kernel in (KERNEL_LANE_SPECIALIZED, 0):
        got = U.hip_sweep(4, 0, 0, n, tables, CONST, m_total, kernel=kernel)
        U.assert_same(f"all statistics, 10^7 (kernel {kernel})", got, want)
    for q in (0, 5, 16 + 7, 32 + 15):
        score2, index = A.unpack_best(int(want[A.S_BEST][q]))
        cfg = G.grid4(n=1, seed=0, first=index)
        row = A.estimate(cfg, tables, CONST)[0]
        method, d, bs = int(cfg["method"][0]), int(cfg["d"][0]), int(cfg["bs"][0])
        assert method * 16 + d - 1 == q and row[A.D_PEAK] <= m_total
        assert A.config_score2(method, bs, d) == score2


@pytest.mark.parametrize("kernel", (0, 4, 6))
def test_calls_recorded_in_a_graph_and_replayed(U, kernel):
    """The entry points allocate nothing and do not synchronize (the run-time build aside, done by
    a call before the capture): estimate, decision, sweep reset and sweep recorded into one HIP
    graph, replayed with new inputs in the same buffers and eager work in between; every replay
    equals the oracle.  The library's own choice (the specialization built into it) and the form
    that reads its tables from the arguments are recorded without any call before the capture."""
    import paper_2404_10933_amd as M
    n, m_total = 64 * 25 + 7, 70 << 30
    tables = [T.llama_table()]
    tab = M.Tables(tables, m_base=CONST.m_base, cu_p=CONST.cu_p, align=CONST.align, kernel=kernel)
    qtab = M.Tables(tables, m_base=CONST.m_base, cu_p=CONST.cu_p, align=CONST.align)
    dev, qdev = M.DeviceConfigs.empty(n), M.DeviceConfigs.empty(n)
    tp = torch.empty(n, dtype=torch.uint8, device="cuda")
    peaks = torch.empty(n, dtype=torch.int64, device="cuda")
    det = torch.empty((M.NDETAIL, n), dtype=torch.int64, device="cuda")
    rows = torch.empty((M.NDECIDE, n), dtype=torch.int64, device="cuda")
    stats = torch.empty((M.NSWEEP, M.SWEEP_GROUPS), dtype=torch.int64, device="cuda")

    def calls():
        M.llmem_estimate_ex(dev, tab, peaks, det)
        M.llmem_decide(qdev, tp, qtab, m_total, None, None, rows)
        M.llmem_sweep_reset(stats)
        M.llmem_sweep(4, 11, 1000, n, tab, m_total, stats)

    def load(first):
        cfg = G.grid4(n=n, seed=3, first=first)
        q, q_tp = G.grid6(n=n, seed=3, first=first)
        for k, v in cfg.items():
            dev.columns[k].copy_(torch.from_numpy(v).cuda())
        for k, v in q.items():
            qdev.columns[k].copy_(torch.from_numpy(v).cuda())
        tp.copy_(torch.from_numpy(q_tp).cuda())
        return cfg, q, q_tp

    load(0)
    if kernel == 6:
        calls()                                           # builds the specialized kernels
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls()
    want_stats = B.sweep(G.grid4(n=n, seed=11, first=1000), 1000, tables, CONST, m_total, threads=8)
    for rep, first in enumerate((0, 12345, 999_000)):
        cfg, q, q_tp = load(first)
        for t in (peaks, det, rows, stats):
            t.fill_(-3)                                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_p, want_d = B.estimate(cfg, tables, CONST, threads=8)
        U.assert_same(f"peaks, replay {rep}", peaks.cpu().numpy(), want_p)
        U.assert_same(f"detail, replay {rep}", det.cpu().numpy().T, want_d)
        U.assert_same(f"decision, replay {rep}", rows.cpu().numpy().T, B.decide(q, q_tp, tables, CONST, m_total, threads=8))
        U.assert_same(f"sweep, replay {rep}", stats.cpu().numpy(), want_stats)
