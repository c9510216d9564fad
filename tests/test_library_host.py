"""Host-side behaviour of the C-ABI library that needs no GPU: it loads, exports
every declared symbol, validates arguments before touching the device, and its
multiply-high division constants are exact."""
import ctypes
import os
import random
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2404_10933_amd as M
    if not os.path.exists(M.library_path()):
        from paper_2404_10933_amd import build
        build.build()
    return M.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "llmem.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(llmem_[a-z_]+)\s*\(", header))
    assert {"llmem_estimate", "llmem_estimate_ex", "llmem_timeline_peaks", "llmem_grid_generate",
            "llmem_events_count", "llmem_events_generate", "llmem_config_bytes", "llmem_events_bytes",
            "llmem_strerror", "llmem_abi_version", "llmem_selftest_divide", "llmem_kernel_forms", "llmem_kernels_release",
            "llmem_estimate_methods", "llmem_decide", "llmem_queries_generate", "llmem_sweep",
            "llmem_sweep_reset", "llmem_compiled_tables"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c_and_links(lib, tmp_path):
    """include/llmem.h compiles as C99 with warnings as errors, and a C program linked against the
    library calls its host-only entry points (no GPU call is made)."""
    import subprocess
    import paper_2404_10933_amd as M
    src = tmp_path / "use.c"
    src.write_text(
        '#include <stdio.h>\n#include <string.h>\n#include "llmem.h"\n'
        "int main(void) {\n"
        "    llmem_tables t; llmem_configs c; int32_t info[8];\n"
        "    memset(&t, 0, sizeof t); memset(&c, 0, sizeof c);\n"
        "    if (llmem_abi_version() != LLMEM_ABI_VERSION) return 1;\n"
        "    if (llmem_kernel_forms(&t, info) != LLMEM_EINVAL_TABLE) return 2;      /* no architecture */\n"
        "    if (llmem_estimate(&c, -1, &t, (int64_t *)0) != LLMEM_EINVAL_NULL) return 3;\n"
        "    if (llmem_config_bytes(3) != 93 || llmem_kernels_release() != 0) return 4;\n"
        '    printf("%s\\n", llmem_strerror(LLMEM_EINVAL_N));\n'
        "    return 0;\n}\n")
    exe = tmp_path / "use"
    lib_dir = os.path.dirname(M.library_path())
    build = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                            str(src), "-o", str(exe), "-L", lib_dir, "-l:libllmem.so", f"-Wl,-rpath,{lib_dir}"],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0 and run.stdout.strip(), (run.returncode, run.stdout, run.stderr)


def test_abi_and_sizes(lib):
    import paper_2404_10933_amd as M
    assert M.llmem_abi_version() == 5
    assert M.llmem_config_bytes(10) == 10 * 31 and M.llmem_config_bytes(-1) == 0
    assert M.llmem_events_bytes(2) == 2 * 6 * 3450 * 8
    assert "NULL" in M.llmem_strerror(-1) and "unknown" in M.llmem_strerror(-99)


def test_release_with_nothing_built(lib):
    """No kernel has been built at run time in a process without a GPU: nothing to release, and
    no device call is made to find that out."""
    import paper_2404_10933_amd as M
    assert M.llmem_kernels_release() == 0 and M.llmem_kernels_release() == 0


def test_division_constants_are_exact(lib):
    rng = random.Random(0)
    for d in range(1, 256):
        xs = [0, 1, d - 1, d, d + 1, 2 ** 63 - 1, 2 ** 63 - d, 2 ** 62, 2 ** 32 - 1, 2 ** 32, 2 ** 32 + 1]
        xs += [rng.randrange(2 ** 63) for _ in range(300)]
        xs += [min(d * rng.randrange(2 ** 55) + e, 2 ** 63 - 1) for e in (-1, 0, 1) for _ in range(30)]
        for x in xs:
            x = max(x, 0)
            assert lib.llmem_selftest_divide(x, d) == x // d, (x, d)
    assert lib.llmem_selftest_divide(5, 0) == 0 and lib.llmem_selftest_divide(5, 256) == 0


def _structs():
    from paper_2404_10933_amd import binding as Bd
    return Bd


def _host_tables(Bd, params, events, n_arch=1, cu_p=2 << 20, align=512, m_base=0, arch=None):
    t = Bd._Tables()
    t.m_base, t.cu_p, t.align, t.n_arch = m_base, cu_p, align, n_arch
    t.n_param_total, t.n_event_total = len(params), len(events)
    a = arch or [(0, len(params), 0, len(events))]
    for i, d in enumerate(a):
        t.arch[i] = Bd._ArchDesc(*d)
    fake_dev = 0x1000                                       # never dereferenced: validation fails first / n == 0
    t.params_host = params.ctypes.data if len(params) else None
    t.events_host = events.ctypes.data if len(events) else None
    t.params_dev = fake_dev if len(params) else None
    t.events_dev = fake_dev if len(events) else None
    return t


def test_argument_validation_without_gpu(lib):
    Bd = _structs()
    params = np.zeros(2, dtype=Bd.PARAM_DTYPE)
    events = np.zeros(3, dtype=Bd.EVENT_DTYPE)
    events["seg"] = [0, 1, 4]
    cfg = Bd._Configs()
    out = ctypes.c_void_p(0x2000)
    ok = _host_tables(Bd, params, events)
    est = lib.llmem_estimate_ex
    assert est(ctypes.byref(cfg), 0, ctypes.byref(ok), out, None, None) == 0          # n == 0: no-op
    assert est(ctypes.byref(cfg), -1, ctypes.byref(ok), out, None, None) == -2
    assert est(None, 0, ctypes.byref(ok), out, None, None) == -1
    assert est(ctypes.byref(cfg), 0, None, out, None, None) == -1
    assert est(ctypes.byref(cfg), 0, ctypes.byref(ok), None, None, None) == -1
    assert est(ctypes.byref(cfg), 5, ctypes.byref(ok), out, None, None) == -1          # NULL columns
    assert lib.llmem_estimate(ctypes.byref(cfg), 0, ctypes.byref(ok), None) == -1

    def bad(**kw):
        p, e = params.copy(), events.copy()
        mut = kw.pop("mut", None)
        if mut:
            mut(p, e)
        t = _host_tables(Bd, p, e, **kw)
        return est(ctypes.byref(cfg), 0, ctypes.byref(t), out, None, None)

    assert bad(n_arch=0) == -3 and bad(n_arch=9) == -3
    assert bad(cu_p=3 << 20) == -3 and bad(align=500) == -3 and bad(align=4 << 20) == -3 and bad(m_base=-1) == -3
    assert bad(arch=[(0, 3, 0, 3)]) == -3 and bad(arch=[(0, 2, 1, 3)]) == -3 and bad(arch=[(-1, 2, 0, 3)]) == -3
    assert bad(mut=lambda p, e: p["dim"].__setitem__((0, 1), 15)) == -3               # selector out of range
    assert bad(mut=lambda p, e: p["cls"].__setitem__(0, 4)) == -3
    assert bad(mut=lambda p, e: p["role"].__setitem__(1, 3)) == -3
    assert bad(mut=lambda p, e: e["seg"].__setitem__(1, 5)) == -3
    assert bad(mut=lambda p, e: e["seg"].__setitem__(2, 0)) == -3                      # segments out of order
    assert bad(mut=lambda p, e: e["flags"].__setitem__(0, 8)) == -3
    assert bad(mut=lambda p, e: e["method_mask"].__setitem__(0, 8)) == -3
    too_many = np.zeros(1025, dtype=Bd.EVENT_DTYPE)
    t = _host_tables(Bd, params, too_many)
    assert est(ctypes.byref(cfg), 0, ctypes.byref(t), out, None, None) == -3

    tl = lib.llmem_timeline_peaks
    assert tl(None, None, -1, None, None, None) == -2 and tl(None, None, 0, None, None, None) == 0
    assert tl(None, None, 3, None, None, None) == -1
    assert lib.llmem_grid_generate(5, 0, 0, 0, ctypes.byref(cfg), None) == -5
    assert lib.llmem_grid_generate(1, 0, 400, 33, ctypes.byref(cfg), None) == -5
    assert lib.llmem_grid_generate(2, 0, 0, -1, ctypes.byref(cfg), None) == -2
    assert lib.llmem_grid_generate(2, 0, 0, 4, ctypes.byref(cfg), None) == -1
    assert lib.llmem_events_count(0, 0, 4, None, None) == -1
    assert lib.llmem_events_generate(0, 0, 4, None, None, None) == -1

    # estimates of all methods and the method decision: same table checks, own argument checks
    em, dec = lib.llmem_estimate_methods, lib.llmem_decide
    c, t_ok = ctypes.byref(cfg), ctypes.byref(ok)
    assert em(c, None, 0, t_ok, out, None, None) == 0 and dec(c, None, 0, t_ok, 1 << 30, out, out, None, None) == 0
    assert em(c, None, 0, t_ok, None, None, None) == -1                               # no output
    assert dec(c, None, 0, t_ok, 1 << 30, out, None, None, None) == -1                # method without bs, no detail
    assert dec(c, None, 0, t_ok, 1 << 30, None, None, out, None) == 0                 # detail alone is enough
    assert em(c, None, -1, t_ok, out, None, None) == -2 and dec(c, None, -1, t_ok, 0, out, out, None, None) == -2
    assert em(None, None, 0, t_ok, out, None, None) == -1 and dec(c, None, 0, None, 0, out, out, None, None) == -1
    assert em(c, None, 3, t_ok, out, None, None) == -1 and dec(c, None, 3, t_ok, 0, out, out, None, None) == -1
    t_bad = _host_tables(Bd, params, events, cu_p=3 << 20)
    assert em(c, None, 0, ctypes.byref(t_bad), out, None, None) == -3
    assert dec(c, None, 0, ctypes.byref(t_bad), 0, out, out, None, None) == -3
    p_bs = params.copy()
    p_bs["dim"][1, 2] = 1                                                              # LLMEM_DIM_BS in a parameter size
    t_bs = _host_tables(Bd, p_bs, events)
    assert em(c, None, 0, ctypes.byref(t_bs), out, None, None) == 0
    assert dec(c, None, 0, ctypes.byref(t_bs), 0, out, out, None, None) == -3
    qg = lib.llmem_queries_generate
    assert qg(0, 0, 0, c, None, None) == 0 and qg(0, 0, -1, c, None, None) == -2 and qg(0, -1, 1, c, None, None) == -2
    assert qg(0, 0, 4, c, None, None) == -1 and qg(0, 0, 4, None, out, None) == -1

    # sweep: argument checks come before any launch
    sw = lib.llmem_sweep
    assert sw(4, 0, 0, 0, t_ok, 1 << 30, out, None) == 0                               # n == 0: no-op
    assert sw(4, 0, 0, 8, None, 1 << 30, out, None) == -1 and sw(4, 0, 0, 8, t_ok, 1 << 30, None, None) == -1
    assert sw(4, 0, 0, -1, t_ok, 0, out, None) == -2 and sw(4, 0, -1, 1, t_ok, 0, out, None) == -2
    assert sw(0, 0, 0, 8, t_ok, 0, out, None) == -5 and sw(5, 0, 0, 8, t_ok, 0, out, None) == -5
    assert sw(6, 0, 0, 8, t_ok, 0, out, None) == -5                                    # the query grid is not swept
    assert sw(1, 0, 400, 33, t_ok, 0, out, None) == -5
    assert sw(4, 0, (1 << 40) - 7, 8, t_ok, 0, out, None) == -5 and sw(4, 0, (1 << 40) - 8, 0, t_ok, 0, out, None) == 0
    assert sw(4, 0, 0, 0, ctypes.byref(t_bad), 0, out, None) == -3
    assert lib.llmem_sweep_reset(None, None) == -1


def test_embedded_sources_cover_the_kernel_and_its_headers():
    """The run-time build compiles the files that build.py embeds: every file the kernel source
    or one of its headers includes by name must be among them (or be the constants header that
    is written at run time)."""
    from paper_2404_10933_amd import build
    text = open(build.write_embedded_sources()).read()
    embedded = [name for name, _ in build.EMBEDDED]
    assert embedded[0] == "estimate_batch.hip" and text.count('R"LLMEM_SRC(') >= len(embedded)
    for name, path in build.EMBEDDED:
        assert f'"{name}"' in text
        for inc in re.findall(r'#include "([^"]+)"', open(path).read()):
            assert os.path.basename(inc) in embedded + ["specialized_prog.h"], (name, inc)
    # the constants header is included through a macro whose default is the run-time build's file
    assert '#define LLMEM_SPEC_HEADER "specialized_prog.h"' in open(build.EMBEDDED[0][1]).read()


def _compiled_counts(table):
    """What the host compiler of the tables should arrive at, counted from the table's own
    definition by the oracle side's census: parameter groups (equal size expressions), size
    classes of the events, and per segment the peak points (an allocation followed by a release
    or the segment's end) that no other point of the segment dominates, plus the terms of the
    kept points and net changes."""
    from oracle import census
    return census.lean_counts(table)


def test_table_compiler_statistics(lib):
    """llmem_kernel_forms reports what the host made of the tables (no device involved)."""
    import paper_2404_10933_amd as M
    from workloads import tables as T
    rng = np.random.default_rng(8)
    cases = [T.gpt_table(), T.opt_table(), T.llama_table(), T.llama_table(checkpoint=False),
             T.random_table(rng, 20, 60, "r", n_sizes=7), T.random_table(rng, 40, 90, "s", n_sizes=12)]
    for t in cases:
        forms = M.llmem_kernel_forms(M.Tables([t], device=None))
        want = _compiled_counts(t)
        assert {k: forms[k] for k in want} == want, t.name
        assert {4, 5, 6} <= set(forms["allowed"])
    llama = M.llmem_kernel_forms(M.Tables([T.llama_table()], device=None))
    assert (llama["param_groups"], llama["size_classes"], llama["peak_points"], llama["terms"]) == (5, 20, 33, 125)
    both = M.llmem_kernel_forms(M.Tables([T.gpt_table(), T.llama_table()], device=None))
    assert both["param_groups"] == _compiled_counts(T.gpt_table())["param_groups"] + 5
    # more size classes than the forms with class slots take: the lane form that evaluates every event
    # where it stands is left (and is what the library chooses), and the wavefront-per-configuration kernel
    many = T.random_table(rng, 5, 400, "many")
    assert _compiled_counts(many)["size_classes"] > 120
    assert M.llmem_kernel_forms(M.Tables([many], device=None))["allowed"] == [1, 2, 7]
    # up to 120 classes the events form takes them, with fewer wavefronts per workgroup
    some = T.random_table(rng, 5, 100, "some")
    assert 48 < _compiled_counts(some)["size_classes"] <= 120
    assert 3 in M.llmem_kernel_forms(M.Tables([some], device=None))["allowed"]


def test_built_in_specializations_match_the_shipped_tables(lib):
    """Every table set the build step lists has a built-in specialized kernel for each flavour,
    found by comparing the compiled words; other tables, and the same tables in another order
    or with one coefficient changed, have none."""
    import dataclasses
    import paper_2404_10933_amd as M
    from paper_2404_10933_amd import build
    from workloads import tables as T
    sets = build.shipped_table_sets()
    assert {name for name, _ in sets} >= {"gpt", "opt", "llama", "llama_full", "zoo"}
    for name, tables in sets:
        for consts in (dict(), dict(m_base=1 << 28, cu_p=1 << 20, align=256)):       # constants are not part of the words
            forms = M.llmem_kernel_forms(M.Tables(tables, device=None, **consts))
            assert forms["prebuilt"] == [True, True, True], name
        words, first = M.llmem_compiled_tables(M.Tables(tables, device=None))
        assert len(words) == forms["program_words"] and first[0] == 0 and len(first) == 8
        assert all(first[q] == 0 for q in range(len(tables), 8))
    rng = np.random.default_rng(9)
    others = [[T.random_table(rng, 20, 60, "r", n_sizes=7)], [T.llama_table(), T.gpt_table()],
              [T.opt_table(), T.gpt_table(), T.llama_table()]]
    llama = T.llama_table()
    changed = dataclasses.replace(llama, events=(dataclasses.replace(llama.events[0], coef=llama.events[0].coef + 1),)
                                  + llama.events[1:])
    others.append([changed])
    for tables in others:
        forms = M.llmem_kernel_forms(M.Tables(tables, device=None))
        assert forms["prebuilt"] == [False, False, False] and 5 in forms["allowed"]
    # tables that do not admit the compiled form have no words
    many = T.random_table(rng, 5, 400, "many")
    with pytest.raises(M.LlmemError) as e:
        M.llmem_compiled_tables(M.Tables([many], device=None))
    assert e.value.code == -3


def test_build_step_takes_further_table_sets(monkeypatch):
    """LLMEM_BUILD_TABLES names a function whose table sets the build step compiles kernels for
    beside the shipped ones (checked here up to the list of sets: no compile)."""
    from paper_2404_10933_amd import build
    shipped = [name for name, _ in build.shipped_table_sets()]
    monkeypatch.setenv("LLMEM_BUILD_TABLES", "extra_tables_for_the_build:more")
    both = build.shipped_table_sets()
    assert [name for name, _ in both] == shipped + ["mine", "mine_and_gpt"]
    assert len(both[-1][1]) == 2 and both[-2][1][0].name == "mine"
    monkeypatch.setenv("LLMEM_BUILD_TABLES", "extra_tables_for_the_build:repeated")
    with pytest.raises(ValueError):
        build.shipped_table_sets()


def test_kept_plans_follow_the_tables_contents(lib):
    """The library keeps, per host thread, what it made of the last few table sets and reuses it
    when every byte is the same.  A change anywhere in the host tables must therefore show at the
    next call: edited in place (same addresses), in the constants, in the ranges, and back again;
    and more table sets than are kept, taken in turn, must each keep their own answer."""
    import paper_2404_10933_amd as M
    from workloads import tables as T
    tab = M.Tables([T.llama_table()], device=None)
    first = M.llmem_kernel_forms(tab)
    assert M.llmem_kernel_forms(tab) == first and first["prebuilt"] == [True, True, True]
    words, _ = M.llmem_compiled_tables(tab)
    # one coefficient edited in place: another size class, other words, no built-in kernel any more
    field = "coef" if "coef" in tab.events_host.dtype.names else tab.events_host.dtype.names[0]
    old = tab.events_host[field][5]
    tab.events_host[field][5] = old + 12345
    changed = M.llmem_kernel_forms(tab)
    assert changed["prebuilt"] == [False, False, False] and changed["size_classes"] == first["size_classes"] + 1
    assert M.llmem_compiled_tables(tab)[0] != words
    tab.events_host[field][5] = old
    assert M.llmem_kernel_forms(tab) == first and M.llmem_compiled_tables(tab)[0] == words
    # an invalid entry is reported although the same tables were accepted a call ago
    dim = tab.events_host["dim"][7].copy()
    tab.events_host["dim"][7] = 200
    with pytest.raises(M.LlmemError) as e:
        M.llmem_kernel_forms(tab)
    assert e.value.code == -3
    tab.events_host["dim"][7] = dim
    assert M.llmem_kernel_forms(tab) == first
    # constants are part of what is compared
    tab.struct.cu_p = 3 << 20
    with pytest.raises(M.LlmemError):
        M.llmem_kernel_forms(tab)
    tab.struct.cu_p = 1 << 21
    # a shorter range of the same array
    tab.struct.arch[0].n_event -= 1
    assert M.llmem_kernel_forms(tab) != first
    tab.struct.arch[0].n_event += 1
    assert M.llmem_kernel_forms(tab) == first
    # six table sets in turn, twice
    rng = np.random.default_rng(21)
    sets = [M.Tables([T.random_table(rng, 10 + j, 40 + 7 * j, f"t{j}", n_sizes=5 + j)], device=None) for j in range(6)]
    want = [M.llmem_kernel_forms(t) for t in sets]
    assert len({w["program_words"] for w in want}) > 3
    for _ in range(2):
        for t, w in zip(sets, want):
            assert M.llmem_kernel_forms(t) == w


def test_run_time_build_refused_under_a_profiler(lib):
    """With a profiler's tool library named in the environment (and no directory of kept code
    objects) the library does not start the run-time compiler: a call that would have to build
    returns LLMEM_EHIP with a message naming LLMEM_KERNEL_CACHE, before any device or compiler call
    - so this runs without a GPU, on host tensors that are never touched.  In a child process, so
    that the variable is set before the library loads."""
    from profiled_child import run_profiled_child
    run_profiled_child(False)


def test_every_entry_point_raises_without_the_library():
    """No fallback of any kind: with the shared library absent every binding call raises, and the
    package does not import the oracle."""
    import subprocess
    import sys
    code = """
import sys
sys.path.insert(0, %r)
import torch
import paper_2404_10933_amd as M
from paper_2404_10933_amd import binding
from workloads import tables as T
binding._LIB_PATH = "/nonexistent/libllmem.so"
binding._lib = None
assert not any(name == "oracle" or name.startswith("oracle.") for name in sys.modules)
n = 8
cfg = M.DeviceConfigs.empty(n, device="cpu")              # host tensors: nothing here reaches a kernel
tab = M.Tables([T.gpt_table()], device=None)
i64 = lambda *shape: torch.zeros(shape, dtype=torch.int64)
i32 = lambda *shape: torch.zeros(shape, dtype=torch.int32)
tp = torch.ones(n, dtype=torch.uint8)
calls = [lambda: M.llmem_abi_version(), lambda: M.llmem_config_bytes(3), lambda: M.llmem_events_bytes(3),
         lambda: M.llmem_strerror(0), lambda: M.llmem_kernel_forms(tab), lambda: M.llmem_compiled_tables(tab),
         lambda: M.llmem_kernels_release(),
         lambda: M.llmem_estimate(cfg, tab, i64(n)), lambda: M.llmem_estimate_ex(cfg, tab, i64(n), i64(M.NDETAIL, n)),
         lambda: M.llmem_estimate_methods(cfg, tp, tab, i64(4, n)),
         lambda: M.llmem_decide(cfg, tp, tab, 1 << 30, i32(n), i32(n), i64(M.NDECIDE, n)),
         lambda: M.llmem_sweep(4, 0, 0, n, tab, 1 << 30, i64(M.NSWEEP, M.SWEEP_GROUPS)),
         lambda: M.llmem_sweep_reset(i64(M.NSWEEP, M.SWEEP_GROUPS)),
         lambda: M.llmem_timeline_peaks(i64(4), i64(2), i64(1), i64(1)),
         lambda: M.llmem_grid_generate(4, 0, 0, n, cfg), lambda: M.llmem_queries_generate(0, 0, n, cfg, tp),
         lambda: M.llmem_events_count(0, 0, 1, i64(1)), lambda: M.llmem_events_generate(0, 0, 1, i64(2), i64(4))]
for j, call in enumerate(calls):
    try:
        call()
    except FileNotFoundError as e:
        assert "no CPU fallback" in str(e), j
    else:
        raise SystemExit("call %%d returned without the library" %% j)
print("ok")
""" % ROOT
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr


def test_table_packing_layout():
    """The binding's 16-byte records match the C structs field by field."""
    Bd = _structs()
    assert [Bd.PARAM_DTYPE.fields[k][1] for k in ("coef", "dim", "cls", "role", "per_layer")] == [0, 4, 8, 9, 10]
    assert [Bd.EVENT_DTYPE.fields[k][1] for k in ("coef", "dim", "elem_bytes", "seg", "flags", "method_mask")] \
        == [0, 4, 8, 9, 10, 11]
    assert ctypes.sizeof(Bd._ArchDesc) == 16
    assert Bd._Tables.arch.offset == 40 and Bd._Tables.params_host.offset == 40 + 8 * 16
