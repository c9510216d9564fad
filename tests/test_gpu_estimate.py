"""Parity of the HIP estimator with the CPU oracle, element by element and bit
exact (all integer byte arithmetic), through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import llmem_oracle as A
from oracle import oracle_c as B
from workloads import grids as G
from workloads import tables as T

pytestmark = pytest.mark.gpu

CONST = T.Constants(m_base=256 << 20)


@pytest.fixture(scope="module")
def U():
    import gpu_util
    return gpu_util


WAVE, LANE, LANE_EVENTS, LANE_COMPILED, LANE_SPECIALIZED, LANE_RUNTIME, LANE_DIRECT = 1, 2, 3, 4, 5, 6, 7     # LLMEM_KERNEL_*
BOTH = (WAVE, LANE_EVENTS, LANE_COMPILED, LANE_SPECIALIZED, LANE_RUNTIME, LANE_DIRECT)
BUILT = (LANE, LANE_SPECIALIZED, LANE_RUNTIME)                  # follow from the others


def _check(U, cfg, tables, const=CONST, threads=8, expect=None, prebuilt=None):
    """Every kernel form the tables allow (one wavefront per configuration; one lane per
    configuration walking all events through size classes, or evaluating each where it stands; the
    same with the host-compiled tables; the same with those tables as constants, built into the
    library where it ships the tables, else built at run time; and always built at run time), each
    forced, plus the library's own choice, against the oracle.
    `expect`: forms that must be allowed; `prebuilt`: whether the library must hold built-in
    specializations for these tables."""
    import paper_2404_10933_amd as M
    forms = M.llmem_kernel_forms(M.Tables(tables, m_base=const.m_base, cu_p=const.cu_p, align=const.align, device=None))
    allowed = forms["allowed"]
    if expect is not None:
        assert sorted(k for k in allowed if k not in BUILT) == sorted(k for k in expect if k not in BUILT), allowed
    assert (LANE_SPECIALIZED in allowed) == (LANE_COMPILED in allowed) == (LANE_RUNTIME in allowed)
    if prebuilt is not None:
        assert forms["prebuilt"] == [prebuilt] * 3, forms
    want_p, want_d = B.estimate(cfg, tables, const, threads=threads)
    for kernel in [0] + allowed:
        got_p, got_d = U.hip_estimate(cfg, tables, const, kernel=kernel)
        U.assert_same(f"detail (kernel {kernel})", got_d, want_d)
        U.assert_same(f"peaks (kernel {kernel})", got_p, want_p)
        got_p2, _ = U.hip_estimate(cfg, tables, const, detail=False, kernel=kernel)
        U.assert_same(f"peaks, no detail (kernel {kernel})", got_p2, want_p)
    assert LANE in allowed and LANE_DIRECT in allowed
    for kernel in (WAVE, LANE_EVENTS, LANE_COMPILED, LANE_SPECIALIZED, LANE_RUNTIME):
        if kernel not in allowed:
            with pytest.raises(M.LlmemError) as e:
                U.hip_estimate(cfg, tables, const, kernel=kernel)
            assert e.value.code == -3


def _one(**kw):
    base = dict(arch_id=0, h=256, L=4, n_heads=4, n_kv=4, ffn=1024, V=8192, P=512, bs=4, sl=256, method=0, d=1,
                chunk_k=4, flags=G.FLAG_GRAD_ALIAS)
    base.update(kw)
    return {k: np.asarray([v]).astype(G.FIELD_DTYPE[k]) for k, v in base.items()}


def _rows(*configs):
    return {k: np.concatenate([c[k] for c in configs]) for k in configs[0]}


def test_worked_examples_through_the_hip_path(U, golden):
    """The hand-worked values of tests/golden directly, not via the oracle, with every kernel
    form the tables allow: the closed-form example with its gradient and per-GPU columns, both
    hand-walked timelines, a table without events, and a head declared as an Embedding."""
    import paper_2404_10933_amd as M
    g = golden("worked_example_gpt_tiny.txt")
    c0 = T.Constants(m_base=0)
    no_alias = 0
    cfg = _rows(_one(), *[_one(method=1, d=d) for d in (2, 3, 4, 7)], *[_one(method=2, d=d) for d in (2, 3, 4, 7)],
                _one(chunk_k=2), _one(chunk_k=-1), _one(flags=no_alias),
                *[_one(method=m, d=d, flags=no_alias) for m in (1, 2) for d in (3, 7)], _one(method=1, d=5, flags=no_alias),
                _one(method=1, d=5), _one(method=2, d=5))
    want_peak = [g["peak_cdp"]] + [g[f"peak_zero3_d{d}"] for d in (2, 3, 4, 7)] + [g[f"peak_tp_d{d}"] for d in (2, 3, 4, 7)] \
        + [g["peak_cdp"] - g["m_p"] + g["m_p_k2"], g["peak_cdp_search"], g["peak_cdp_noalias"],
           g["peak_zero3_d3_noalias"], g["peak_zero3_d7_noalias"], g["peak_tp_d3_noalias"], g["peak_tp_d7_noalias"],
           g["peak_zero3_d5_noalias"]]
    tables = [T.gpt_table()]
    allowed = M.llmem_kernel_forms(M.Tables(tables, m_base=0, device=None))["allowed"]
    for kernel in [0] + allowed:
        p, d = U.hip_estimate(cfg, tables, c0, kernel=kernel)
        assert p[:len(want_peak)].tolist() == want_peak, kernel
        assert (d[0, A.D_NPARAMS], d[0, A.D_TMAX], d[0, A.D_PARAM], d[0, A.D_OS], d[0, A.D_OUT], d[0, A.D_LM]) == (
            g["n_params"], g["t_max"], g["m_p"], g["m_os"], g["m_out"], g["m_lm"]), kernel
        assert d[5, A.D_BACK] == g["m_back_d2"] and d[10, A.D_K] == g["search_k"]
        assert d[11, A.D_GRAD] == d[0, A.D_GRAD] == g["grad_logical_cdp"]
        assert (d[4, A.D_PARAM], d[4, A.D_OS], d[4, A.D_GRAD]) == (g["param_gpu_zero3_d7"], g["os_gpu_d7"], g["grad_logical_d7"])
        assert (d[8, A.D_PARAM], d[8, A.D_OS], d[8, A.D_GRAD]) == (g["param_gpu_tp_d7"], g["os_gpu_d7"], g["grad_logical_d7"])
        assert d[12, A.D_GRAD] == d[14, A.D_GRAD] == g["grad_logical_d3"]
        assert d[17, A.D_OS] == d[18, A.D_OS] == g["os_gpu_d5"]
    # the hand-walked timelines
    from test_oracle_pins import _tiny_timeline_table, _second_timeline_table
    w = golden("worked_timeline_tiny.txt")
    c5 = T.Constants(m_base=5000)
    cases = [(_tiny_timeline_table(), _rows(_one(L=3), _one(L=3, method=2, d=4), _one(L=3, method=1, d=4)),
              [w["peak_live_cdp"], w["peak_live_tp_d4"], w["peak_live_cdp"]]),
             (_second_timeline_table(), _rows(_one(L=3), _one(L=3, method=2, d=3), _one(L=3, method=2, d=1), _one(L=3, method=1, d=3)),
              [w["peak_live2_cdp"], w["peak_live2_tp_d3"], w["peak_live2_tp_d1"], w["peak_live2_cdp"]]),
             (T.ArchTable("none", (), ()), _one(L=3), [w["peak_live_no_events"]])]
    for table, rows, want in cases:
        allowed = M.llmem_kernel_forms(M.Tables([table], m_base=5000, device=None))["allowed"]
        for kernel in [0] + allowed:
            _, d = U.hip_estimate(rows, [table], c5, kernel=kernel)
            assert d[:, A.D_LIVE].tolist() == want, (table.name, kernel)
    # e_n leaves out a head that is declared as an Embedding: m_out is one hidden-state tensor, exactly a page
    P = T.ParamEntry
    tied = T.ArchTable("tied", (P("tok", 1, ("V", "h"), "E", "EMBED_TOK", False), P("head", 1, ("V", "h"), "E", "LM_HEAD", False)), ())
    for kernel in [0] + M.llmem_kernel_forms(M.Tables([tied], m_base=0, device=None))["allowed"]:
        _, d = U.hip_estimate(_one(L=0, bs=4, sl=512, h=512, V=1000), [tied], c0, kernel=kernel)
        assert d[0, A.D_OUT] == 2 * 1024 * 1024, kernel


def test_grid1_all(U):
    cfg = G.grid1()
    _check(U, cfg, [T.gpt_table()], expect=BOTH, prebuilt=True)
    # and directly against the Python oracle that carries the pins
    rows = np.asarray(A.estimate(cfg, [T.gpt_table()], CONST), dtype=np.int64)
    _, got = U.hip_estimate(cfg, [T.gpt_table()], CONST)
    U.assert_same("detail vs oracle A", got, rows)


@pytest.mark.parametrize("name,n,first", [("g2", 100_000, 0), ("g3", 64 * 300 + 37, 500_000),
                                          ("g4", 64 * 300 + 1, 9_000_000), ("g3", 1_000_000, 0)])
def test_grid_slices(U, name, n, first):
    """Grids 2 and 3 whole (10^5 and 10^6 configurations, every column of every configuration
    against the oracle), and slices from the far ends of grids 3 and 4."""
    spec = G.GRIDS[name]
    _check(U, spec["make"](n=n, seed=0, first=first), [T.FAMILIES[spec["family"]]()], expect=BOTH, threads=16, prebuilt=True)


@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 65, 127, 128, 129, 1000])
def test_ragged_sizes(U, n):
    cfg = G.grid4(n=n, seed=3)
    _check(U, cfg, [T.llama_table()])


def test_random_tables_wild_configs(U):
    rng = np.random.default_rng(11)
    tabs = [T.random_table(rng, 9, 150, "r0"), T.llama_table(), T.random_table(rng, 0, 0, "empty"),
            T.random_table(rng, 64, 700, "r3"), T.gpt_table(), T.random_table(rng, 1, 1, "one"),
            T.random_table(rng, 30, 1024, "max")]
    cfg = G.random_configs(rng, 64 * 40 + 5, n_arch=len(tabs), wild=True)
    # hundreds of distinct sizes in one architecture: no form with class slots applies; the library takes
    # the lane form that evaluates every event where it stands
    _check(U, cfg, tabs, T.Constants(m_base=1, cu_p=4096, align=512), expect=(WAVE, LANE_DIRECT))
    _check(U, cfg, tabs, T.Constants(m_base=0, cu_p=2 << 20, align=512), expect=(WAVE, LANE_DIRECT))
    _check(U, cfg, tabs, T.Constants(m_base=12345, cu_p=1 << 16, align=1), expect=(WAVE, LANE_DIRECT))


def test_tables_with_many_size_classes(U):
    """Between 49 and 120 distinct sizes per architecture: the events form keeps a slot per class and
    launches fewer wavefronts per workgroup so that the slots fit the LDS (two, then one)."""
    import paper_2404_10933_amd as M
    rng = np.random.default_rng(17)
    for n_event, n_sizes, with_slots in ((150, 70, True), (200, 100, True), (400, 120, False)):
        tabs = [T.random_table(rng, 7, n_event, "wide", n_sizes=n_sizes), T.gpt_table()]
        forms = M.llmem_kernel_forms(M.Tables(tabs, device=None))
        assert 48 < forms["event_slots"] - 1 <= 120, forms
        # the largest of these needs more LDS than one wavefront's workgroup may ask for: direct form
        assert (LANE_EVENTS in forms["allowed"]) == with_slots, forms
        cfg = G.random_configs(rng, 64 * 30 + 11, n_arch=2, wild=True)
        _check(U, cfg, tabs, T.Constants(m_base=77, cu_p=1 << 16, align=512))


def test_random_tables_few_sizes(U):
    """Random tables whose events share at most 32 size expressions, several
    architectures mixed inside each wavefront's 64 configurations."""
    rng = np.random.default_rng(13)
    tabs = [T.random_table(rng, 9, 150, "r0", n_sizes=22), T.llama_table(), T.random_table(rng, 0, 0, "empty"),
            T.random_table(rng, 64, 1024, "r3", n_sizes=20), T.gpt_table(), T.random_table(rng, 1, 1, "one", n_sizes=1),
            T.random_table(rng, 30, 600, "r6", n_sizes=7), T.opt_table()]
    cfg = G.random_configs(rng, 64 * 40 + 5, n_arch=len(tabs), wild=True)
    # all eight together do not fit the kernel arguments in compiled form
    _check(U, cfg, tabs, T.Constants(m_base=1, cu_p=4096, align=512), expect=(WAVE, LANE_EVENTS, LANE_DIRECT))
    _check(U, cfg, tabs, T.Constants(m_base=12345, cu_p=1 << 16, align=1), expect=(WAVE, LANE_EVENTS, LANE_DIRECT))
    # subsets that do fit: every form
    small = T.random_table(rng, 12, 140, "r8", n_sizes=9)
    for subset in ([tabs[7], tabs[5], tabs[4]], [tabs[1], tabs[4]], [small, tabs[2], tabs[5]]):
        sub = G.random_configs(rng, 64 * 20 + 3, n_arch=len(subset), wild=True)
        _check(U, sub, subset, T.Constants(m_base=0, cu_p=2 << 20, align=512), expect=BOTH)
        _check(U, sub, subset, T.Constants(m_base=7, cu_p=4096, align=512), expect=BOTH)


def test_degenerate_and_flag_cases(U):
    rng = np.random.default_rng(12)
    tabs = [T.degenerate_table(T.llama_table()), T.opt_table()]
    cfg = G.random_configs(rng, 3000, n_arch=2)
    cfg["flags"][:] = rng.integers(0, 8, size=3000)       # tied / untied, aliasing on and off, both logit widths
    cfg["L"][:100] = 0
    cfg["sl"][100:200] = 1
    cfg["chunk_k"][200:300] = -1
    cfg["h"][200:260] = 40000                              # no feasible chunk candidate
    cfg["n_heads"][200:260] = 8
    cfg["ffn"][200:260] = 60000
    _check(U, cfg, tabs)


@pytest.mark.parametrize("name,n,first", [("g2", 64 * 100 + 3, 0), ("g3", 64 * 120 + 37, 400_000), ("g4", 64 * 60 + 1, 5_000_000)])
def test_full_traversal_tables(U, name, n, first):
    """The tables without gradient checkpointing (every saved forward output stays alive until
    its backward: much longer live ranges, Sec. 3.1), alone and mixed with the checkpointed
    table of the same family inside every wavefront."""
    spec = G.GRIDS[name]
    make = T.FAMILIES[spec["family"]]
    cfg = spec["make"](n=n, seed=0, first=first)
    _check(U, cfg, [make(checkpoint=False)], expect=BOTH, prebuilt=True)
    cfg["arch_id"] = (np.arange(n) % 2).astype(np.uint8)
    _check(U, cfg, [make(checkpoint=False), make()], CONST, prebuilt=False)


def test_sizes_on_both_sides_of_2_to_31_blocks(U):
    """The compiled form walks 32-bit block counts while every size of a wavefront's 64
    configurations is at most 2^31 allocator blocks, and 64-bit bytes otherwise: wavefronts
    entirely below, entirely above, and with single large configurations in either half."""
    E = T.EventEntry
    events = (E("a0", "A", +1, 3, ("V", "V"), 8), E("a1", "A", +1, 1, ("bs", "sl", "h"), 2),
              E("f0", "F", +1, 1, ("V", "ffn"), 4), E("f1", "F", -1, 1, ("V", "ffn"), 4, times_L=False),
              E("f2", "F", +1, 2, ("bs", "sl", "h"), 2), E("h0", "H", +1, 1, ("V", "V", "h"), 8, frozenset({0, 2})),
              E("h1", "H", -1, 3, ("V", "V"), 8), E("b0", "B", +1, 5, ("V", "ffn"), 4, scale="tp_gather"),
              E("b1", "B", -1, 2, ("bs", "sl", "h"), 2), E("z0", "Z", +1, 7, ("V", "V"), 1, times_L=True),
              E("z1", "Z", -1, 1, ("V", "V", "h"), 8, frozenset({0, 2})))
    table = T.ArchTable("wide", T.gpt_table().params, events)
    rng = np.random.default_rng(4)
    n = 64 * 8 + 9
    cfg = G.random_configs(rng, n, n_arch=1)
    cfg["V"][:] = rng.integers(1, 3000, size=n)             # 3 * V * V * 8 below 2^31 * 512
    cfg["ffn"][:] = rng.integers(1, 20000, size=n)
    big = np.zeros(n, dtype=bool)
    big[64:128] = True                                       # a whole wavefront of large sizes
    big[64 * 3 + 5] = True                                   # one configuration in the lower half
    big[64 * 5 + 40] = True                                  # one in the upper half
    big[64 * 6 + 31] = big[64 * 6 + 32] = True               # one in each half
    big[n - 1] = True                                        # in the ragged tail
    cfg["V"][big] = rng.integers(150_000, 200_000, size=int(big.sum()))
    for const in (CONST, T.Constants(m_base=3, cu_p=4096, align=1), T.Constants(m_base=0, cu_p=1 << 30, align=1 << 20)):
        _check(U, cfg, [table], const, expect=BOTH)
    # sizes straddling the limit exactly: 2^31 blocks of 512 bytes = 2^40 bytes = coef * V * V * 8 with V = 2^18, coef = 2
    edge = T.ArchTable("edge", T.gpt_table().params, (E("a", "A", +1, 2, ("V", "V"), 8), E("b", "A", -1, 2, ("V", "V"), 8),
                                                     E("c", "F", +1, 1, ("V", "P"), 8)))
    cfg = G.random_configs(rng, 64 * 3, n_arch=1)
    cfg["V"][:] = 1 << 18                                    # exactly 2^31 blocks: the last size the 32-bit walk takes
    cfg["V"][::7] = (1 << 18) - 1
    cfg["V"][64 * 2 + 3::7] = (1 << 18) + 1                  # just above, in the last wavefront only
    cfg["P"][:] = rng.integers(0, 3, size=64 * 3)
    _check(U, cfg, [edge], CONST, expect=BOTH)


def test_peak_points_with_sums_far_from_zero(U):
    """Peak points whose sums, counted from the start of their segment, are hundreds of times 2^31
    allocator blocks above and below zero (the compiled form compares such sums by their bit
    patterns, moved into the range of positive doubles): wavefronts that take the 32-bit walk, with
    every large size exactly 2^31 blocks, and wavefronts that take the 64-bit walk."""
    E = T.EventEntry
    big = (2, ("V", "V"), 8)                                  # 2^40 bytes = 2^31 blocks at V = 2^18
    small = (3, ("P",), 4)
    many = lambda tag, seg, sign, count: tuple(E(f"{tag}{j}", seg, sign, *big) for j in range(count))
    events = (many("a", "A", +1, 150)
              + many("f", "F", -1, 100) + (E("fs", "F", +1, *small), E("ft", "F", -1, *small)) + many("g", "F", +1, 100)
              + many("h", "H", +1, 150) + many("i", "H", -1, 150)
              + many("b", "B", -1, 90) + (E("bs", "B", +1, *small), E("bt", "B", -1, *small)) + many("c", "B", +1, 91)
              + (E("bu", "B", -1, *big),) + many("z", "Z", -1, 150))
    table = T.ArchTable("far", T.gpt_table().params, events)
    rng = np.random.default_rng(21)
    n = 64 * 4 + 7
    cfg = G.random_configs(rng, n, n_arch=1)
    cfg["L"][:] = rng.integers(0, 9, size=n)
    cfg["P"][:] = rng.integers(0, 5000, size=n)
    cfg["V"][:] = 1 << 18
    cfg["V"][5:128:9] = rng.integers(1, 1 << 18, size=len(cfg["V"][5:128:9]))
    cfg["V"][64 * 2 + 11] = (1 << 18) + 1                     # this wavefront and the next walk in 64 bits
    cfg["V"][64 * 3:] = rng.integers(1 << 18, 1 << 19, size=n - 64 * 3)
    _check(U, cfg, [table], CONST, expect=BOTH)
    want_p, want_d = B.estimate(cfg, [table], CONST)
    import paper_2404_10933_amd as M
    assert int(want_d[:, M.DETAIL_COLUMNS.index("peak_live")].max()) >= 300 << 40      # the sums are of that size


def test_determinism_and_stream(U):
    cfg = G.grid3(n=20_000, seed=5)
    for kernel in BOTH:
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            a = U.hip_estimate(cfg, [T.llama_table()], CONST, stream=s, kernel=kernel)
        b = U.hip_estimate(cfg, [T.llama_table()], CONST, kernel=kernel)
        U.assert_same("detail twice", a[1], b[1])


_FULL = {}


def _full_size_reference():
    """Oracle results for the 10^7 grid (every column of every configuration), computed once
    for both kernel forms."""
    if not _FULL:
        n = 10_000_000
        cfg = G.grid4(n=n, seed=0)
        tables = [T.llama_table()]
        want_p, want_d = B.estimate(cfg, tables, CONST, threads=16)
        _FULL.update(n=n, cfg=cfg, tables=tables, want_p=want_p, want_d=want_d)
    return _FULL


def test_host_threads_with_their_own_tables_and_streams(U):
    """Four host threads, each with its own tables (so each makes the library build its own
    specialized kernel at run time), stream and outputs, calling at the same time: the builds run
    side by side (none holds the library's lock while it compiles), every result equals the
    oracle's; then the same tables again from four threads at once, which wait for one build each."""
    import threading
    rng = np.random.default_rng(61)
    jobs = []
    for j, tables in enumerate(([T.gpt_table()], [T.opt_table()], [T.llama_table()],
                                [T.random_table(rng, 12, 40, "t", n_sizes=6), T.gpt_table()])):
        cfg = G.random_configs(np.random.default_rng(70 + j), 64 * 20 + 9, n_arch=len(tables))
        const = T.Constants(m_base=1000 + j)
        jobs.append((cfg, tables, const, B.estimate(cfg, tables, const, threads=8)))
    results, errors = [None] * len(jobs), []

    def work(j):
        try:
            cfg, tables, const, _ = jobs[j]
            stream = torch.cuda.Stream()
            out = []
            for _ in range(3):
                with torch.cuda.stream(stream):
                    out.append(U.hip_estimate(cfg, tables, const, stream=stream, kernel=LANE_RUNTIME))
            results[j] = out
        except Exception as e:                                  # reported by the main thread
            errors.append((j, repr(e)))

    threads = [threading.Thread(target=work, args=(j,)) for j in range(len(jobs))]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=200)
    assert not errors, errors
    for j, (_, _, _, (want_p, want_d)) in enumerate(jobs):
        for got_p, got_d in results[j]:
            U.assert_same(f"peaks, thread {j}", got_p, want_p)
            U.assert_same(f"detail, thread {j}", got_d, want_d)
    # one new table set asked for by four threads at the same time: one of them builds, the others wait
    shared = [T.random_table(rng, 10, 30, "shared", n_sizes=5)]
    cfg = G.random_configs(np.random.default_rng(80), 64 * 10 + 3, n_arch=1)
    want_p, want_d = B.estimate(cfg, shared, CONST, threads=8)
    jobs[:] = [(cfg, shared, CONST, None)] * 4
    results[:] = [None] * 4
    threads = [threading.Thread(target=work, args=(j,)) for j in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=200)
    assert not errors, errors
    for j in range(4):
        for got_p, got_d in results[j]:
            U.assert_same(f"peaks, shared tables, thread {j}", got_p, want_p)
            U.assert_same(f"detail, shared tables, thread {j}", got_d, want_d)


def test_profiled_process_runs_everything_but_the_run_time_build(U):
    """A process with a profiler's tool library named in its environment: asking for a kernel that
    would have to be built at run time is an error with a message, while the built-in
    specialization and the interpreting forms run."""
    from profiled_child import run_profiled_child
    run_profiled_child(True)


@pytest.mark.parametrize("kernel", (0, LANE_COMPILED, LANE_RUNTIME))
def test_full_size_grid4(U, kernel):
    """10^7 configurations, in the launch configurations the benchmark times (the library's own
    choice, which is the specialized kernel built into it for the Llama-style table; the form that
    reads the compiled tables from its arguments; the specialized kernel built at run time):
    m_peak and all detail columns (including the timeline walk) of every configuration against
    the oracle."""
    import paper_2404_10933_amd as M
    ref = _full_size_reference()
    n = ref["n"]
    dev = M.DeviceConfigs.from_numpy(ref["cfg"])
    tab = M.Tables(ref["tables"], m_base=CONST.m_base, cu_p=CONST.cu_p, align=CONST.align, kernel=kernel)
    assert M.llmem_kernel_forms(tab)["prebuilt"] == [True, True, True]
    peaks = torch.empty(n, dtype=torch.int64, device="cuda")
    det = torch.empty((M.NDETAIL, n), dtype=torch.int64, device="cuda")
    M.llmem_estimate_ex(dev, tab, peaks, det)
    torch.cuda.synchronize()
    U.assert_same("m_peak, all 10^7", peaks.cpu().numpy(), ref["want_p"])
    want_d = ref["want_d"]
    for c in range(M.NDETAIL):
        U.assert_same(f"detail column {c}, all 10^7", det[c].cpu().numpy(), want_d[:, c])


def test_outputs_beyond_four_gib(U):
    """45 000 037 configurations generated on the device: the detail columns take 4.3 GB, so the
    last of them lie beyond 2^32 bytes from the start of the output (and of a column: 360 MB).
    The oracle computes slices at the start, in the middle and at the ragged end; everything the
    kernels wrote elsewhere must at least differ from the fill value."""
    import paper_2404_10933_amd as M
    n = 45_000_037
    dev = M.DeviceConfigs.empty(n)
    M.llmem_grid_generate(4, 7, 0, n, dev)
    tables = [T.llama_table()]
    slices = [(0, 4096), (n // 2 - 1000, 3000), (n - 4101, 4101)]
    want = [B.estimate(G.grid4(n=m, seed=7, first=first), tables, CONST, threads=8) for first, m in slices]
    peaks = torch.empty(n, dtype=torch.int64, device="cuda")
    det = torch.empty((M.NDETAIL, n), dtype=torch.int64, device="cuda")
    assert det.numel() * 8 > (1 << 32)
    for kernel in (0, LANE_COMPILED, LANE_EVENTS, LANE_DIRECT):
        peaks.fill_(-7)
        det.fill_(-7)
        tab = M.Tables(tables, m_base=CONST.m_base, cu_p=CONST.cu_p, align=CONST.align, kernel=kernel)
        M.llmem_estimate_ex(dev, tab, peaks, det)
        torch.cuda.synchronize()
        for (first, m), (want_p, want_d) in zip(slices, want):
            U.assert_same(f"m_peak from {first} (kernel {kernel})", peaks[first:first + m].cpu().numpy(), want_p)
            U.assert_same(f"detail from {first} (kernel {kernel})", det[:, first:first + m].cpu().numpy().T, want_d)
        assert int((peaks == -7).sum().item()) == 0 and int((det[M.NDETAIL - 1] == -7).sum().item()) == 0
        assert int((det[A.D_LIVE] <= 0).sum().item()) == 0                       # every timeline peak was written
    del det, peaks


def test_release_of_kernels_built_at_run_time(U):
    """llmem_kernels_release unloads what was built at run time and nothing else: the count it
    returns, a second call that finds nothing, the same tables built again with the same results,
    and the built-in kernels and table-driven forms untouched in between."""
    import paper_2404_10933_amd as M
    torch.cuda.synchronize()
    M.llmem_kernels_release()                                   # whatever earlier tests left
    base = T.opt_table()
    table = T.ArchTable("release", base.params, base.events[:-1] + (T.EventEntry("z8", "Z", +1, 131, ("h", "sl"), 2),))
    cfg = G.grid2(n=5000, seed=4)
    want_p, want_d = B.estimate(cfg, [table], CONST, threads=8)
    for round_ in range(2):
        got_p, got_d = U.hip_estimate(cfg, [table], CONST, kernel=LANE_RUNTIME)          # detail flavour
        U.assert_same(f"detail, round {round_}", got_d, want_d)
        got_p, _ = U.hip_estimate(cfg, [table], CONST, kernel=LANE_RUNTIME, detail=False)   # m_peak flavour
        U.assert_same(f"m_peak, round {round_}", got_p, want_p)
        torch.cuda.synchronize()
        assert M.llmem_kernels_release() == 2
        assert M.llmem_kernels_release() == 0
        # nothing else went with them
        other = G.grid4(n=1000, seed=5)
        U.assert_same("built-in kernel after the release", U.hip_estimate(other, [T.llama_table()], CONST)[1],
                      B.estimate(other, [T.llama_table()], CONST, threads=8)[1])
        got_p, got_d = U.hip_estimate(cfg, [table], CONST, kernel=LANE_COMPILED)
        U.assert_same("compiled form after the release", got_d, want_d)


def test_kept_run_time_builds_are_bounded(U):
    """A process keeps a bounded number of kernels built at run time per device (LLMEM_KERNELS_KEPT,
    read once: a child process with a limit of 4).  Seven table sets in turn, the first one again
    (its kernel has been unloaded meanwhile and is built again), every result equal to the oracle's,
    and what is left loaded at the end is within the limit."""
    import os
    import subprocess
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    child = (
        "import sys, numpy as np\n"
        f"sys.path[:0] = [{repr(os.path.dirname(here))}, {repr(here)}]\n"
        "import torch, gpu_util as U\n"
        "import paper_2404_10933_amd as M\n"
        "from oracle import oracle_c as B\n"
        "from workloads import grids as G, tables as T\n"
        "const = T.Constants(m_base=256 << 20)\n"
        "base = T.gpt_table()\n"
        "tables = [T.ArchTable('t%d' % j, base.params, base.events[:-1] + (T.EventEntry('z', 'Z', +1, 100 + j, ('h', 'ffn'), 2),)) for j in range(7)]\n"
        "cfg = G.grid2(n=2000, seed=5)\n"
        "for t in tables + tables[:1]:\n"
        "    want_p, want_d = B.estimate(cfg, [t], const, threads=8)\n"
        "    got_p, got_d = U.hip_estimate(cfg, [t], const, kernel=6)\n"
        "    assert (got_d == want_d).all() and (got_p == want_p).all(), t.name\n"
        "torch.cuda.synchronize()\n"
        "left = M.llmem_kernels_release()\n"
        "assert 1 <= left <= 4, left\n"
        "print('child ok', left)\n")
    env = dict(os.environ, LLMEM_KERNELS_KEPT="4")
    out = subprocess.run([sys.executable, "-c", child], env=env, capture_output=True, text=True, timeout=200)
    assert out.returncode == 0 and "child ok" in out.stdout, (out.stdout[-500:], out.stderr[-2000:])


def test_built_kernels_are_kept_between_processes(U, tmp_path):
    """LLMEM_KERNEL_CACHE: a build writes one file; a second process loads it instead of building
    (the file is not rewritten) and computes the same; a file with a foreign identity is ignored."""
    import os
    import subprocess
    import sys
    import paper_2404_10933_amd as M
    cache = tmp_path / "kernels"
    cache.mkdir()
    # a table no other test uses, so that this process has to build it
    base = T.gpt_table()
    table = T.ArchTable("cache", base.params, base.events[:-1] + (T.EventEntry("z9", "Z", +1, 77, ("h", "ffn"), 2),))
    cfg = G.grid2(n=3000, seed=9)
    want_p, want_d = B.estimate(cfg, [table], CONST, threads=8)
    os.environ["LLMEM_KERNEL_CACHE"] = str(cache)
    try:
        got_p, got_d = U.hip_estimate(cfg, [table], CONST, kernel=LANE_SPECIALIZED)
    finally:
        del os.environ["LLMEM_KERNEL_CACHE"]
    U.assert_same("detail", got_d, want_d)
    files = sorted(cache.iterdir())
    assert len(files) == 1 and files[0].suffix == ".co" and files[0].stat().st_size > 10_000
    stamp = files[0].stat().st_mtime_ns
    np.save(tmp_path / "want.npy", want_d)
    child = (
        "import sys, numpy as np\n"
        f"sys.path[:0] = [{repr(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))}, {repr(os.path.dirname(os.path.abspath(__file__)))}]\n"
        "import gpu_util as U\n"
        "from workloads import grids as G, tables as T\n"
        "base = T.gpt_table()\n"
        "table = T.ArchTable('cache', base.params, base.events[:-1] + (T.EventEntry('z9', 'Z', +1, 77, ('h', 'ffn'), 2),))\n"
        "p, d = U.hip_estimate(G.grid2(n=3000, seed=9), [table], T.Constants(m_base=256 << 20), kernel=5)\n"
        f"assert (d == np.load({repr(str(tmp_path / 'want.npy'))})).all()\n"
        "print('child ok')\n")
    env = dict(os.environ, LLMEM_KERNEL_CACHE=str(cache))
    out = subprocess.run([sys.executable, "-c", child], env=env, capture_output=True, text=True, timeout=170)
    assert out.returncode == 0 and "child ok" in out.stdout, out.stderr[-2000:]
    assert sorted(cache.iterdir()) == files and files[0].stat().st_mtime_ns == stamp     # loaded, not rebuilt
    # a file under the expected name whose recorded identity is another one: rebuilt and replaced
    files[0].write_bytes(b"\x05\x00\x00\x00\x00\x00\x00\x00wrong" + b"x" * 100)
    out = subprocess.run([sys.executable, "-c", child], env=env, capture_output=True, text=True, timeout=170)
    assert out.returncode == 0 and "child ok" in out.stdout, out.stderr[-2000:]
    assert files[0].stat().st_size > 10_000
    # the right identity in front of a code object cut short: the size and checksum kept with it do not
    # match, so it never reaches the loader; it is built again and replaced
    whole = files[0].read_bytes()
    files[0].write_bytes(whole[:len(whole) - 3000])
    out = subprocess.run([sys.executable, "-c", child], env=env, capture_output=True, text=True, timeout=170)
    assert out.returncode == 0 and "child ok" in out.stdout, out.stderr[-2000:]
    assert files[0].stat().st_size == len(whole)
