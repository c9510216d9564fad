"""Pins of CPU oracle A against what the paper and arithmetic fix: hand-worked
values (tests/golden), closed forms, special cases, invariants and a brute-force
allocator simulation.  None of these re-type an oracle formula: expected values
come from the golden text files, from textbook parameter-count formulas, from
relations between outputs, or from a block-by-block simulator."""
import random

import numpy as np
import pytest

from oracle import llmem_oracle as O
from workloads import tables as T
from workloads import grids as G

CU_P = 2 * 1024 * 1024
CONST0 = T.Constants(m_base=0)


def cfg(**kw):
    base = dict(arch_id=0, h=256, L=4, n_heads=4, n_kv=4, ffn=1024, V=8192, P=512, bs=4, sl=256,
                method=0, d=1, chunk_k=4, flags=G.FLAG_GRAD_ALIAS)
    base.update(kw)
    return base


def est(c, table, const=CONST0, timeline=False):
    return O.estimate_one(c, [table], const, timeline)


# ---------------------------------------------------------------------------
# hand-worked example
# ---------------------------------------------------------------------------
def test_worked_example(golden):
    g = golden("worked_example_gpt_tiny.txt")
    gpt = T.gpt_table()
    r = est(cfg(), gpt)
    assert r[O.D_NPARAMS] == g["n_params"]
    assert r[O.D_TMAX] == g["t_max"]
    assert r[O.D_PARAM] == g["m_p"]
    assert r[O.D_OS] == g["m_os"]
    assert r[O.D_OUT] == g["m_out"]
    assert r[O.D_LM] == g["m_lm"]
    assert r[O.D_PEAK] == g["peak_cdp"]
    for d in (2, 3, 4):
        assert est(cfg(method=1, d=d), gpt)[O.D_PEAK] == g[f"peak_zero3_d{d}"]
        assert est(cfg(method=2, d=d), gpt)[O.D_PEAK] == g[f"peak_tp_d{d}"]
    assert est(cfg(method=2, d=2), gpt)[O.D_BACK] == g["m_back_d2"]
    # ZeRO-3 keeps all of param fp16 and shards param fp32
    z = est(cfg(method=1, d=2), gpt)
    assert z[O.D_PARAM] == g["m_p16"] + g["m_p32"] // 2
    assert est(cfg(chunk_k=2), gpt)[O.D_PARAM] == g["m_p_k2"]
    s = est(cfg(chunk_k=-1), gpt)
    assert (s[O.D_K], s[O.D_PEAK]) == (g["search_k"], g["peak_cdp_search"])
    D = O.dim_vector(cfg())
    embed_p, lm_p, other_p, t_max, n_params, e_n = O.param_census(gpt, D, False)
    assert (other_p, e_n) == (g["other_p"], 2)
    assert O.param_memory(embed_p, other_p, O.chunk_elems(4), CU_P) == (g["m_p"], g["m_p16"], g["m_p32"])
    # gradients with a space of their own, and the per-GPU shares of the model states (d = 7: no
    # page count of the example is a multiple of 7, so every ceiling and block round-up shows)
    no_alias = G.FLAG_GRAD_ALIAS ^ cfg()["flags"]
    assert no_alias & G.FLAG_GRAD_ALIAS == 0
    c0 = est(cfg(flags=no_alias), gpt)
    assert (c0[O.D_PEAK], c0[O.D_GRAD]) == (g["peak_cdp_noalias"], g["grad_logical_cdp"])
    assert c0[O.D_PEAK] - r[O.D_PEAK] == g["grad_pages_bytes"]
    assert r[O.D_GRAD] == g["grad_logical_cdp"]                       # reported also when it shares param fp16's space
    for method, name in ((1, "zero3"), (2, "tp")):
        shared = est(cfg(method=method, d=7), gpt)
        own = est(cfg(method=method, d=7, flags=no_alias), gpt)
        assert shared[O.D_PEAK] == g[f"peak_{name}_d7"]
        assert own[O.D_PEAK] == g[f"peak_{name}_d7_noalias"]
        assert own[O.D_PEAK] - shared[O.D_PEAK] == g["grad_extra_d7"]
        assert own[O.D_GRAD] == shared[O.D_GRAD] == g["grad_logical_d7"]
        assert own[O.D_PARAM] == shared[O.D_PARAM] == g[f"param_gpu_{name}_d7"]
        assert own[O.D_OS] == shared[O.D_OS] == g["os_gpu_d7"]
        assert est(cfg(method=method, d=3, flags=no_alias), gpt)[O.D_PEAK] == g[f"peak_{name}_d3_noalias"]
        assert est(cfg(method=method, d=3, flags=no_alias), gpt)[O.D_GRAD] == g["grad_logical_d3"]
        assert est(cfg(method=method, d=5), gpt)[O.D_OS] == g["os_gpu_d5"]
        five = est(cfg(method=method, d=5, flags=no_alias), gpt)
        assert five[O.D_PEAK] - est(cfg(method=method, d=5), gpt)[O.D_PEAK] == g["grad_extra_d5"]
    assert est(cfg(method=1, d=5, flags=no_alias), gpt)[O.D_PEAK] == g["peak_zero3_d5_noalias"]
    assert est(cfg(method=1, d=7), gpt)[O.D_PEAK] - g["m_p16"] - g["m_out"] - g["m_lm"] == g["zero3_share_d7"]


def _tiny_timeline_table():
    E = T.EventEntry
    one = ("one",)
    tp = frozenset((2,))
    ev = (
        E("a", "A", +1, 1000, one, 1),
        E("f1", "F", +1, 600, one, 1), E("f2", "F", +1, 100, one, 1), E("f2-", "F", -1, 100, one, 1),
        E("h", "H", +1, 3000, one, 1), E("h-", "H", -1, 3000, one, 1),
        E("b1", "B", +1, 700, one, 1), E("buf", "B", +1, 900, one, 1, tp, "tp_gather"),
        E("b-", "B", -1, 600, one, 1),
        E("z", "Z", -1, 1000, one, 1), E("buf-", "Z", -1, 900, one, 1, tp, "tp_gather", True),
    )
    return T.ArchTable("tiny", (), ev)


def _second_timeline_table():
    E = T.EventEntry
    one = ("one",)
    tp = frozenset((2,))
    ev = (
        E("a", "A", +1, 300, one, 1, T.ALL_METHODS, "none", True),
        E("f", "F", +1, 600, one, 1), E("f-", "F", -1, 600, one, 1),
        E("buf", "B", +1, 1537, one, 1, tp, "tp_gather"), E("b", "B", +1, 200, one, 1), E("b-", "B", -1, 200, one, 1),
        E("a-", "Z", -1, 300, one, 1, T.ALL_METHODS, "none", True), E("buf-", "Z", -1, 1537, one, 1, tp, "tp_gather", True),
    )
    return T.ArchTable("second", (), ev)


def test_worked_timeline(golden):
    g = golden("worked_timeline_tiny.txt")
    t = _tiny_timeline_table()
    const = T.Constants(m_base=5000)
    assert est(cfg(L=3), t, const, True)[O.D_LIVE] == g["peak_live_cdp"]
    assert est(cfg(L=3, method=2, d=4), t, const, True)[O.D_LIVE] == g["peak_live_tp_d4"]
    # ZeRO-3 does not see the TP-only events
    assert est(cfg(L=3, method=1, d=4), t, const, True)[O.D_LIVE] == g["peak_live_cdp"]
    # per-block allocation in one event; an all-gather buffer that is no whole number of bytes
    t2 = _second_timeline_table()
    assert est(cfg(L=3), t2, const, True)[O.D_LIVE] == g["peak_live2_cdp"]
    assert est(cfg(L=3, method=2, d=3), t2, const, True)[O.D_LIVE] == g["peak_live2_tp_d3"]
    assert est(cfg(L=3, method=2, d=1), t2, const, True)[O.D_LIVE] == g["peak_live2_tp_d1"]
    assert est(cfg(L=3, method=1, d=3), t2, const, True)[O.D_LIVE] == g["peak_live2_cdp"]
    # no events at all: the resident state is the peak
    assert est(cfg(L=3), T.ArchTable("none", (), ()), const, True)[O.D_LIVE] == g["peak_live_no_events"]


def test_embedding_count_leaves_out_the_head():
    """e_n of m_out (Sec. 4.2) counts the Embedding operators of the transformer part: a head that
    is declared as an Embedding-class tensor (a tied copy of the token embedding) is not one.
    Tiny table: a token embedding and such a head, no blocks: m_out = one hidden-state tensor."""
    P = T.ParamEntry
    t = T.ArchTable("tied", (P("tok", 1, ("V", "h"), "E", "EMBED_TOK", False), P("head", 1, ("V", "h"), "E", "LM_HEAD", False)), ())
    c = cfg(L=0, bs=4, sl=512, h=512, V=1000)
    assert est(c, t, T.Constants(m_base=0))[O.D_OUT] == 2 * 1024 * 1024          # 4 * 512 * 512 * 2 B = exactly one page


def test_event_lists_that_start_with_a_release():
    """The empty prefix counts (nothing is live before the first event): a list whose running
    totals never rise above zero has peaks of zero, in both pools."""
    assert O.event_list_peaks([]) == (0, 0)
    assert O.event_list_peaks([-600]) == (0, 0)
    assert O.event_list_peaks([-600, 100]) == (0, 0)
    # the total never rises above zero, but the small pool on its own reaches one block: one segment reserved
    assert O.event_list_peaks([-3_000_000, 100]) == (0, 2 * 1024 * 1024)


# ---------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------
def test_param_count_closed_forms():
    rng = random.Random(1)
    gpt, llama = T.gpt_table(), T.llama_table()
    for _ in range(50):
        h = 64 * rng.randint(1, 64)
        L, V, P = rng.randint(1, 48), rng.randint(1000, 130000), rng.randint(1, 4096)
        f = 4 * h
        tied = rng.random() < 0.5
        c = cfg(h=h, L=L, V=V, P=P, ffn=f, n_heads=h // 64, n_kv=h // 64,
                flags=G.FLAG_GRAD_ALIAS | (G.FLAG_TIED_LM_HEAD if tied else 0))
        n = V * h * (1 if tied else 2) + P * h + L * (12 * h * h + 13 * h) + 2 * h
        assert est(c, gpt)[O.D_NPARAMS] == n
        nkv = rng.choice((1, 2, 4, 8))
        nh = h // 64
        kv = nkv * 64
        f = rng.randint(1, 30000)
        c = cfg(h=h, L=L, V=V, P=0, ffn=f, n_heads=nh, n_kv=nkv)
        n = 2 * V * h + L * (2 * h * h + 2 * h * kv + 3 * h * f + 2 * h) + h
        assert est(c, llama)[O.D_NPARAMS] == n
    # the "125m" decoder: h=768, L=12, V=50272, 2050 positions, tied
    c = cfg(h=768, L=12, V=50272, P=2050, ffn=3072, n_heads=12, n_kv=12,
            flags=G.FLAG_GRAD_ALIAS | G.FLAG_TIED_LM_HEAD)
    assert est(c, T.opt_table())[O.D_NPARAMS] == 125_239_296


def test_swiglu_width_of_llama_grids():
    g = G.grid3(n=2000)
    expect = {2048: 5632, 4096: 11008, 5120: 13824, 8192: 22016}
    for h, f in zip(g["h"], g["ffn"]):
        assert expect[int(h)] == int(f)
    assert (g["n_heads"] * 128 == g["h"]).all()


def _aligned_table():
    """Only Embedding/Linear tensors, every one a whole number of pages in every
    byte width used: model states are then exact multiples of the element count."""
    P = T.ParamEntry
    return T.ArchTable("aligned", (
        P("emb", 1, ("V", "h"), "E", "EMBED_TOK", False),
        P("w1", 1, ("h", "ffn"), "L", "OTHER", True),
        P("w2", 1, ("ffn", "h"), "L", "OTHER", True),
    ), ())


def test_model_states_bytes_per_parameter():
    """Mixed-precision Adam: fp16 param (shared with fp16 grad) + fp32 master +
    momentum + variance = 14 B per element on the GPU; 16 B once gradients get
    their own space (Sec. 4.1; the well-known 16 B/param of mixed-precision Adam)."""
    t = _aligned_table()
    # h*ffn = 2^22 elements per matrix; V*h = 2^24; other_p = 2*L*2^22 = L * 2^23 = L chunks of 16 MiB
    for L in (1, 3, 8):
        c = cfg(h=1024, ffn=4096, V=16384, L=L, bs=1, sl=1, chunk_k=4)
        r = est(c, t)
        n = r[O.D_NPARAMS]
        assert n == 16384 * 1024 + 2 * L * 1024 * 4096
        states = r[O.D_PEAK] - r[O.D_OUT] - r[O.D_LM]
        assert states == 14 * n
        r2 = est(dict(c, flags=0), t)
        assert r2[O.D_PEAK] - r2[O.D_OUT] - r2[O.D_LM] == 16 * n
        assert r[O.D_GRAD] == 2 * n and r[O.D_PARAM] == 6 * n and r[O.D_OS] == 8 * n
        # ZeRO-3: fp16 params whole, the 12 B/element of fp32 master + Adam states shared out
        for d in (2, 4, 8):
            z = est(dict(c, method=1, d=d), t)
            assert z[O.D_PEAK] - z[O.D_OUT] - z[O.D_LM] == 2 * n + 12 * n // d
            tp = est(dict(c, method=2, d=d), t)
            assert tp[O.D_PEAK] - tp[O.D_OUT] - tp[O.D_LM] - tp[O.D_BACK] == 14 * n // d


def test_zero3_share_is_total_over_d():
    gpt = T.gpt_table()
    for d in range(1, 17):
        c = cfg(method=1, d=d, h=768, ffn=3072, L=12, V=50272, P=2048, n_heads=12, n_kv=12)
        z = est(c, gpt)
        s = est(dict(c, method=0), gpt)
        D = O.dim_vector(c)
        embed_p, lm_p, other_p, *_ = O.param_census(gpt, D, False)
        m_p, m_p16, m_p32 = O.param_memory(embed_p, other_p, O.chunk_elems(4), CU_P)
        x = m_p32 + s[O.D_OS]
        share = z[O.D_PEAK] - m_p16 - z[O.D_OUT] - z[O.D_LM]
        assert x <= share * d < x + 512 * d + d          # share in [x/d, x/d + 512 + 1)
        assert share % 512 == 0


def test_output_and_lm_terms_closed_form():
    """With page-aligned factors the ceilings vanish and the equations of Sec. 4.2
    reduce to plain products."""
    llama = T.llama_table()
    c = cfg(h=4096, L=32, n_heads=32, n_kv=8, ffn=11008, V=32768, P=0, bs=8, sl=1024,
            flags=G.FLAG_GRAD_ALIAS | G.FLAG_LOGITS_FP32)
    r = est(c, llama)
    assert r[O.D_OUT] == (1 + 32) * 8 * 1024 * 4096 * 2
    # logits 8*1024*32768*4 = 2^30; the shifted copies have 1023 rows: 8*1023*32768*4 = 1023 * 2^20
    # which is 511.5 pages -> 512 pages; lm_head 32768*4096*2 bytes
    assert r[O.D_LM] == 2**30 + 2 * 512 * CU_P + 32768 * 4096 * 2
    r2 = est(dict(c, flags=G.FLAG_GRAD_ALIAS), llama)      # 2-byte logits: half, shifted 255.75 -> 256 pages
    assert r2[O.D_LM] == 2**29 + 2 * 256 * CU_P + 32768 * 4096 * 2
    # bs = 16: one row of logits is exactly one page, so the shift by one position shows: 1023 pages
    r3 = est(dict(c, bs=16), llama)
    assert r3[O.D_LM] == 2**31 + 2 * 1023 * CU_P + 32768 * 4096 * 2
    # m_back^tp for d = 4: 32 * 2^25 elements * 2 B * 3/4 = 1.5 * 2^30 exactly
    assert est(dict(c, method=2, d=4), llama)[O.D_BACK] == 3 * 2**29


# ---------------------------------------------------------------------------
# special cases and invariants
# ---------------------------------------------------------------------------
def _random_cfgs(rng, n, family):
    if family == "llama":
        g = G.grid3(n=n, seed=rng.randint(0, 1 << 30))
    else:
        g = G.grid2(n=n, seed=rng.randint(0, 1 << 30))
    return [{k: int(v[i]) for k, v in g.items()} for i in range(n)]


@pytest.mark.parametrize("family", ["opt", "llama"])
def test_special_cases(family):
    rng = random.Random(2)
    t = T.FAMILIES[family]()
    for c in _random_cfgs(rng, 60, family):
        cdp = est(dict(c, method=0), t)
        tp1 = est(dict(c, method=2, d=1), t)
        assert tp1[O.D_PEAK] == cdp[O.D_PEAK] and tp1[O.D_BACK] == 0     # one GPU: TP is CDP
        z1 = est(dict(c, method=1, d=1), t)
        assert z1[O.D_PEAK] - cdp[O.D_PEAK] in (0, CU_P)                 # separate fp16/fp32 pages
        for d in (1, 5, 16):                                            # CDP ignores d
            assert est(dict(c, method=0, d=d), t)[O.D_PEAK] == cdp[O.D_PEAK]
        # sl = 1: the shifted copies vanish
        one = est(dict(c, sl=1), t)
        D = O.dim_vector(dict(c, sl=1))
        lm_p = O.param_census(t, D, False)[1]
        assert one[O.D_LM] == CU_P * -(-(c["bs"] * c["V"] * D["B_logits"]) // CU_P) + 2 * lm_p
        # the search's answer, given as a fixed chunk size, reproduces the search result
        s = est(dict(c, chunk_k=-1), t)
        f = est(dict(c, chunk_k=s[O.D_K]), t)
        assert s == f
        # least waste with ties to the smaller chunk == smallest chunk that holds t_max
        feasible = [k for k in range(2, 11) if s[O.D_TMAX] <= 2 ** (k + 19)]
        assert s[O.D_K] == (feasible[0] if feasible else 10)
        assert bool(s[O.D_FLAGS] & O.CHUNK_INFEASIBLE) == (not feasible)


@pytest.mark.parametrize("family", ["opt", "llama"])
def test_invariants(family):
    rng = random.Random(3)
    t = T.FAMILIES[family]()
    for c in _random_cfgs(rng, 40, family):
        r = est(c, t)
        # Algorithm 1 grows bs until the peak exceeds capacity: the peak must not fall with bs (or sl)
        assert est(dict(c, bs=c["bs"] + 1), t)[O.D_PEAK] >= r[O.D_PEAK]
        assert est(dict(c, sl=c["sl"] + 7), t)[O.D_PEAK] >= r[O.D_PEAK]
        cdp = est(dict(c, method=0), t)
        tp = est(dict(c, method=2), t)
        assert tp[O.D_PARAM] <= cdp[O.D_PARAM] and tp[O.D_OS] <= cdp[O.D_OS]
        # every term of the paper is whole pages, except lm_head bytes and the /d shards (512-blocks)
        D = O.dim_vector(c)
        lm_p = O.param_census(t, D, bool(c["flags"] & 2))[1]
        assert cdp[O.D_PARAM] % CU_P == 0 and cdp[O.D_OS] % CU_P == 0 and r[O.D_OUT] % CU_P == 0
        assert (r[O.D_LM] - 2 * lm_p) % CU_P == 0 and tp[O.D_BACK] % CU_P == 0
        assert (r[O.D_PEAK] - 2 * lm_p) % 512 == 0
        # larger partition degree never costs more under ZeRO-3
        z = [est(dict(c, method=1, d=d), t)[O.D_PEAK] for d in (1, 2, 4, 8, 16)]
        assert z == sorted(z, reverse=True)


def test_tp_cheaper_than_dp_for_large_models():
    """Sec. 1 / Sec. 7.4: TP lowers memory below DP when the model is large."""
    llama = T.llama_table()
    c = cfg(h=4096, L=32, n_heads=32, n_kv=8, ffn=11008, V=32000, P=0, bs=1, sl=512, d=4,
            flags=G.FLAG_GRAD_ALIAS | G.FLAG_LOGITS_FP32)
    cdp, z3, tp = (est(dict(c, method=m), llama)[O.D_PEAK] for m in (0, 1, 2))
    assert tp < z3 < cdp


def test_per_tensor_rounding_of_optimizer_states():
    """m_os rounds tensor by tensor: many sub-page tensors each cost a whole page."""
    P = T.ParamEntry
    t = T.ArchTable("small", (P("w", 1, ("h",), "L", "OTHER", True),
                              P("b", 1, ("h",), "B", "OTHER", True),
                              P("n", 1, ("h",), "N", "OTHER", True)), ())
    r = est(cfg(h=100, L=7), t)
    assert r[O.D_OS] == 7 * CU_P            # 7 Linear tensors of 800 B; Bias and LayerNorm are not counted
    assert r[O.D_NPARAMS] == 7 * 300


def test_degenerate_timeline_brackets_closed_form():
    """A timeline holding only what the paper's formula counts, releasing nothing,
    peaks within 4 pages below m_peak: block vs. page rounding of m_out and the three
    m_lm tensors is the only gap (conventional DP, hidden states a multiple of 512 B)."""
    rng = random.Random(4)
    for family in ("opt", "llama"):
        t = T.degenerate_table(T.FAMILIES[family]())
        for c in _random_cfgs(rng, 25, family):
            c = dict(c, method=0)
            r = est(c, t, T.Constants(m_base=12345), True)
            assert r[O.D_PEAK] - 4 * CU_P < r[O.D_LIVE] <= r[O.D_PEAK]
            # sharded methods: each separately sharded block adds at most one 512-byte round-up
            for m in (1, 2):
                q = est(dict(c, method=m, d=3), t, T.Constants(m_base=12345), True)
                assert q[O.D_PEAK] - q[O.D_BACK] - 4 * CU_P < q[O.D_LIVE] <= q[O.D_PEAK] - q[O.D_BACK] + 512 + 2


# ---------------------------------------------------------------------------
# brute-force allocator simulation
# ---------------------------------------------------------------------------
def _blocks(nbytes, block=512):
    """Number of `block`-byte blocks that cover [0, nbytes)."""
    return len(range(0, nbytes, block))


class BlockAllocator:
    """Keeps every live tensor as an explicit list of blocks; no running sums."""

    def __init__(self):
        self.live = []                      # one entry per live tensor: (pool, n_blocks)
        self.peak_total = 0
        self.peak_pool = {"small": 0, "large": 0}

    def _observe(self):
        tot = sum(n for _, n in self.live)
        self.peak_total = max(self.peak_total, tot)
        for pool in self.peak_pool:
            self.peak_pool[pool] = max(self.peak_pool[pool], sum(n for p, n in self.live if p == pool))

    def event(self, raw):
        n = _blocks(abs(raw))
        pool = "small" if n < 4096 else "large"          # 4096 blocks of 512 B = 2 MiB
        if raw >= 0:
            self.live.append((pool, n))
        else:
            self.live.remove((pool, n))                  # raises if no such tensor is live
        self._observe()


def test_event_list_peaks_against_block_simulation():
    rng = random.Random(5)
    edge = [1, 511, 512, 513, 2 * 1024 * 1024 - 513, 2 * 1024 * 1024 - 512, 2 * 1024 * 1024 - 511,
            2 * 1024 * 1024 - 1, 2 * 1024 * 1024, 2 * 1024 * 1024 + 1, 5_000_000, 0]
    for trial in range(200):
        live, events = [], []
        for _ in range(rng.randint(0, 50)):
            if live and rng.random() < 0.45:
                events.append(-live.pop(rng.randrange(len(live))))
            else:
                s = rng.choice(edge) if rng.random() < 0.6 else rng.randint(1, 6_000_000)
                live.append(s)
                events.append(s)
        sim = BlockAllocator()
        for e in events:
            sim.event(e)
        alloc, resv = O.event_list_peaks(events)
        assert alloc == sim.peak_total * 512
        seg = 4096
        want = sum(len(range(0, sim.peak_pool[p], seg)) for p in ("small", "large")) * seg * 512
        assert resv == want
        assert alloc <= resv and resv % (2 * 1024 * 1024) == 0
        # releasing later never lowers the peak
        if any(e < 0 for e in events):
            i = next(j for j, e in enumerate(events) if e < 0)
            later = events[:i] + events[i + 1:] + [events[i]]
            assert O.event_list_peaks(later)[0] >= alloc
    assert O.event_list_peaks([]) == (0, 0)
    # a release larger than anything in the other pool only touches its own pool
    a, r = O.event_list_peaks([3_000_000, 100, -3_000_000, 100])
    assert a == (_blocks(3_000_000) + 1) * 512
    assert r == 2 * 1024 * 1024 * (2 + 1)


def test_table_timeline_against_block_simulation():
    """Expand a small random table into the explicit event sequence of one
    iteration (A, F per block, H, B per block, Z) and let the block simulator find
    the peak; sizes are computed here from the raw table fields."""
    rng = np.random.default_rng(6)
    pyrng = random.Random(6)
    for trial in range(40):
        # random table whose frees always match an earlier allocation of the same segment
        evs = []
        for seg in T.SEGMENTS:
            open_ = []
            for _ in range(pyrng.randint(0, 6)):
                if open_ and pyrng.random() < 0.4:
                    e = open_.pop(pyrng.randrange(len(open_)))
                    evs.append(T.EventEntry("f", seg, -1, e.coef, e.dims, e.elem_bytes, e.methods, e.scale, e.times_L))
                else:
                    dims = tuple(pyrng.choice(("bs", "sl", "h", "one", "n_kv")) for _ in range(pyrng.randint(0, 3)))
                    e = T.EventEntry("a", seg, +1, pyrng.randint(1, 5), dims, pyrng.choice((1, 2, 4)),
                                     frozenset(m for m in (0, 1, 2) if pyrng.random() < 0.8),
                                     "tp_gather" if pyrng.random() < 0.2 else "none",
                                     pyrng.random() < 0.15 and seg in "AHZ")
                    open_.append(e)
                    evs.append(e)
        t = T.ArchTable("r", (), tuple(evs))
        c = cfg(bs=pyrng.randint(1, 3), sl=pyrng.randint(1, 40), h=pyrng.choice((16, 24, 100)),
                n_heads=2, n_kv=pyrng.randint(1, 3), L=pyrng.randint(0, 4), method=pyrng.randint(0, 2),
                d=pyrng.randint(1, 5))
        dims = dict(one=1, bs=c["bs"], sl=c["sl"], h=c["h"], n_kv=c["n_kv"])
        live_blocks, peak = [], 0

        def apply(e):
            nonlocal peak
            if c["method"] not in e.methods:
                return
            raw = e.coef * e.elem_bytes
            for dname in e.dims:
                raw *= dims[dname]
            if e.scale == "tp_gather":
                q, rem = divmod(raw * (c["d"] - 1), c["d"])
                raw = q + (1 if rem else 0)
            for _ in range(c["L"] if e.times_L else 1):
                if e.sign > 0:
                    live_blocks.append(_blocks(raw))
                else:
                    live_blocks.remove(_blocks(raw))
                # all copies of a times_L event happen at once: observe after the loop
            peak = max(peak, sum(live_blocks))

        seq = ["A"] + ["F"] * c["L"] + ["H"] + ["B"] * c["L"] + ["Z"]
        for s in seq:
            for e in evs:
                if e.seg == s:
                    apply(e)
        r = est(c, t, T.Constants(m_base=0), True)
        assert r[O.D_LIVE] == peak * 512, (trial, c)


@pytest.mark.parametrize("family", ("gpt", "llama"))
def test_family_timelines_with_and_without_checkpointing(family):
    """The family tables themselves, checkpointed and as the full traversal that keeps
    every saved forward output (Sec. 3.1): the block simulator walks the explicit event
    sequence of one iteration on top of the resident state; from two blocks on the full
    traversal never peaks below the checkpointed one, and its forward alone already holds L blocks'
    worth of saved tensors."""
    pyrng = random.Random(8)
    make = T.FAMILIES[family]
    for trial in range(6):
        h = pyrng.choice((64, 128))
        c = cfg(bs=pyrng.randint(1, 3), sl=pyrng.choice((1, 7, 33)), h=h, n_heads=h // 32, n_kv=pyrng.choice((1, 2)),
                ffn=pyrng.choice((96, 172)), V=pyrng.choice((50, 301)), P=pyrng.choice((0, 40)), L=pyrng.randint(0, 3),
                method=pyrng.randint(0, 2), d=pyrng.randint(1, 4), flags=pyrng.randint(0, 7))
        D = O.dim_vector(c)
        peaks = {}
        for checkpoint in (True, False):
            t = make(checkpoint=checkpoint)
            const = T.Constants(m_base=pyrng.choice((0, 5 * 512)))
            r = est(c, t, const, True)
            _, lm_p, _, _, _, _ = O.param_census(t, D, False)
            trainable_extra = r[O.D_PEAK] - (O.estimate_one(dict(c, flags=c["flags"] | G.FLAG_GRAD_ALIAS), [t], const, False)[O.D_PEAK])
            resident = const.m_base + r[O.D_PARAM] + r[O.D_OS] + lm_p * 2 + trainable_extra
            live_blocks, peak, after_forward = [], 0, None
            for s in ["A"] + ["F"] * c["L"] + ["H"] + ["B"] * c["L"] + ["Z"]:
                if s == "H" and after_forward is None:
                    after_forward = sum(live_blocks)
                for e in t.events:
                    if e.seg != s or c["method"] not in e.methods:
                        continue
                    raw = e.coef * e.elem_bytes
                    for dname in e.dims:
                        raw *= D[dname]
                    if e.scale == "tp_gather":
                        q, rem = divmod(raw * (c["d"] - 1), c["d"])
                        raw = q + (1 if rem else 0)
                    for _ in range(c["L"] if e.times_L else 1):
                        if e.sign > 0:
                            live_blocks.append(_blocks(raw))
                        else:
                            live_blocks.remove(_blocks(raw))
                    peak = max(peak, sum(live_blocks))
            assert not live_blocks
            assert r[O.D_LIVE] == resident + peak * 512, (trial, checkpoint, c)
            peaks[checkpoint] = (r[O.D_LIVE] - resident, after_forward * 512)
        if c["L"] >= 2:
            assert peaks[False][0] >= peaks[True][0]
            # saved tensors of every block are alive when the forward ends; a checkpointed block keeps one output
            x_bytes = _blocks(c["bs"] * c["sl"] * c["h"] * 2) * 512
            assert peaks[True][1] <= (c["L"] + 2) * x_bytes
            assert peaks[False][1] >= 10 * c["L"] * x_bytes


# ---------------------------------------------------------------------------
# error reporting of a single configuration
# ---------------------------------------------------------------------------
def test_invalid_configurations_are_flagged():
    gpt = T.gpt_table()
    cases = [(dict(arch_id=1), O.ERR_ARCH), (dict(method=3), O.ERR_METHOD), (dict(d=0), O.ERR_D),
             (dict(n_heads=0), O.ERR_HEADS), (dict(chunk_k=17), O.ERR_CHUNK), (dict(chunk_k=-2), O.ERR_CHUNK),
             (dict(d=0, method=7), O.ERR_D | O.ERR_METHOD)]
    for kw, flag in cases:
        r = est(cfg(**kw), gpt)
        assert r[O.D_PEAK] == -1 and r[O.D_FLAGS] == flag and sum(r[1:11]) == 0
    # no chunk candidate holds the largest tensor: k = 10 is used and the flag set
    big = est(cfg(h=32768, ffn=32768, n_heads=256, n_kv=256, chunk_k=-1), gpt)
    assert big[O.D_K] == 10 and big[O.D_FLAGS] == O.CHUNK_INFEASIBLE and big[O.D_PEAK] > 0


# ---------------------------------------------------------------------------
# the pins notice plausible mistakes: plant them in the oracle, on the CPU
# ---------------------------------------------------------------------------
def _suite(golden):
    test_worked_example(golden)
    test_worked_timeline(golden)
    test_model_states_bytes_per_parameter()
    test_output_and_lm_terms_closed_form()
    test_per_tensor_rounding_of_optimizer_states()
    test_param_count_closed_forms()
    test_event_list_peaks_against_block_simulation()
    test_embedding_count_leaves_out_the_head()
    test_event_lists_that_start_with_a_release()


def _wrong_census(t_max_over_all=False, layers_once=False, tied_counted=False, embeddings_all=False):
    def census(table, D, tied):
        L = D["L"]
        embed_p = lm_p = other_p = t_max = e_n = 0
        for p in table.params:
            t_p = O.monomial(p.coef, p.dims, D)
            count = L if (p.per_layer and not layers_once) else 1
            if p.role == "EMBED_TOK":
                embed_p += t_p * count
            elif p.role == "LM_HEAD":
                lm_p += t_p * count
            else:
                other_p += t_p * count
            if p.role == "OTHER" or t_max_over_all:
                t_max = max(t_max, t_p)
            if p.cls == "E" and (p.role != "LM_HEAD" or embeddings_all):
                e_n += 1
        n_params = embed_p + other_p + (lm_p if (tied_counted or not tied) else 0)
        return embed_p, lm_p, other_p, t_max, n_params, e_n
    return census


def _wrong_timeline(backward_once=False, without_resident=False, segment_ends_only=False, forward_last_block_first=False):
    def peak_of(table, D, method, prelude, align):
        by_seg = {s: [e for e in table.events if e.seg == s] for s in "AFHBZ"}
        live = prelude
        peak = 0 if without_resident else prelude
        order = ["A"] + ["F"] * D["L"] + ["H"] + ["B"] * (1 if backward_once else D["L"]) + ["Z"]
        for s in order:
            for e in by_seg[s]:
                live += O.event_value(e, D, method, align)
                if not segment_ends_only:
                    peak = max(peak, live)
            if segment_ends_only:
                peak = max(peak, live)
        return peak
    return peak_of


def _wrong_event_list(split_inclusive=False, pool_by_raw_size=False, reserved_of_sum=False, reserved_of_total=False,
                      unrounded=False, without_empty_prefix=False):
    def peaks(events):
        small = large = 0
        top_small = top_large = top = None if without_empty_prefix else 0
        for raw in events:
            raw = int(raw)
            r = abs(raw) if unrounded else O.up(abs(raw), O.EVENT_ALIGN)
            key = abs(raw) if pool_by_raw_size else r
            delta = r if raw >= 0 else -r
            if key < O.EVENT_SPLIT or (split_inclusive and key == O.EVENT_SPLIT):
                small += delta
            else:
                large += delta
            top_small = small if top_small is None else max(top_small, small)
            top_large = large if top_large is None else max(top_large, large)
            top = small + large if top is None else max(top, small + large)
        top_small, top_large, top = top_small or 0, top_large or 0, top or 0
        if reserved_of_total:
            return top, O.up(top, O.EVENT_SEGMENT)
        if reserved_of_sum:
            return top, O.up(top_small + top_large, O.EVENT_SEGMENT)
        return top, O.up(top_small, O.EVENT_SEGMENT) + O.up(top_large, O.EVENT_SEGMENT)
    return peaks


MUTANTS = {
    "floor instead of ceiling": ("cdiv", lambda a, b: a // b),
    "no page rounding": ("up", lambda a, u: a),
    "chunk holds fp32 values": ("chunk_elems", lambda k: (1 << k) * 1024 * 1024 // 4),
    "shifted copies counted once": ("lm_memory", lambda lm_p, D, cu_p: O.up(D["bs"] * D["sl"] * D["V"] * D["B_logits"], cu_p)
                                    + O.up(D["bs"] * D["sl_m1"] * D["V"] * D["B_logits"], cu_p) + lm_p * 2),
    "shift ignored": ("lm_memory", lambda lm_p, D, cu_p: 3 * O.up(D["bs"] * D["sl"] * D["V"] * D["B_logits"], cu_p) + lm_p * 2),
    "lm_head dropped": ("lm_memory", lambda lm_p, D, cu_p: O.up(D["bs"] * D["sl"] * D["V"] * D["B_logits"], cu_p)
                        + 2 * O.up(D["bs"] * D["sl_m1"] * D["V"] * D["B_logits"], cu_p)),
    "embeddings not kept": ("output_memory", lambda e_n, D, cu_p: O.up(D["L"] * D["bs"] * D["sl"] * D["h"] * 2, cu_p)),
    "m_os rounded once": ("optimizer_memory", lambda table, D, cu_p: O.up(sum(
        O.monomial(p.coef, p.dims, D) * 8 * (D["L"] if p.per_layer else 1)
        for p in table.params if p.cls in "EL" and p.role != "LM_HEAD"), cu_p)),
    "m_os over all classes": ("optimizer_memory", lambda table, D, cu_p: sum(
        O.up(O.monomial(p.coef, p.dims, D) * 8, cu_p) * (D["L"] if p.per_layer else 1)
        for p in table.params if p.role != "LM_HEAD")),
    "momentum only": ("optimizer_memory", lambda table, D, cu_p: sum(
        O.up(O.monomial(p.coef, p.dims, D) * 4, cu_p) * (D["L"] if p.per_layer else 1)
        for p in table.params if p.cls in "EL" and p.role != "LM_HEAD")),
    "tp buffer not scaled": ("tp_backward_memory", lambda D, d, cu_p: O.up(D["L"] * D["bs"] * D["sl"] * D["h"] * 2, cu_p)),
    "tp buffer over d": ("tp_backward_memory", lambda D, d, cu_p: O.up(O.cdiv(D["L"] * D["bs"] * D["sl"] * D["h"] * 2, d), cu_p)),
    "zero3 shards fp16 too": ("compose", lambda method, d, m_base, m_p, m_p16, m_p32, m_os, m_out, m_lm, m_back, align:
                              m_base + (m_p + m_os if method == 0 else O.up(O.cdiv(m_p + m_os, d), align)) + m_out + m_lm
                              + (m_back if method == 2 else 0)),
    "tp forgets m_back": ("compose", lambda method, d, m_base, m_p, m_p16, m_p32, m_os, m_out, m_lm, m_back, align:
                          m_base + m_out + m_lm + (m_p + m_os if method == 0 else
                                                   m_p16 + O.up(O.cdiv(m_p32 + m_os, d), align) if method == 1 else
                                                   O.up(O.cdiv(m_p + m_os, d), align))),
    "gradient always separate": ("gradient_terms", lambda method, d, trainable, grad_alias, cu_p, align:
                                 (trainable * 2, O.up(trainable * 2, cu_p))),
    "gradient shard not block-rounded": ("gradient_terms", lambda method, d, trainable, grad_alias, cu_p, align: (
        trainable * 2 if method == 0 else O.cdiv(trainable * 2, d),
        0 if grad_alias else O.up(trainable * 2, cu_p) if method == 0 else O.cdiv(O.up(trainable * 2, cu_p), d))),
    "gradient divided before page rounding": ("gradient_terms", lambda method, d, trainable, grad_alias, cu_p, align: (
        trainable * 2 if method == 0 else O.cdiv(trainable * 2, d),
        0 if grad_alias else O.up(trainable * 2, cu_p) if method == 0 else O.up(O.cdiv(trainable * 2, d), align))),
    "gradient shard page-rounded": ("gradient_terms", lambda method, d, trainable, grad_alias, cu_p, align: (
        trainable * 2 if method == 0 else O.cdiv(trainable * 2, d),
        0 if grad_alias else O.up(trainable * 2, cu_p) if method == 0 else O.up(O.cdiv(O.up(trainable * 2, cu_p), d), cu_p))),
    "gradient not shared out": ("gradient_terms", lambda method, d, trainable, grad_alias, cu_p, align: (
        trainable * 2 if method == 0 else O.cdiv(trainable * 2, d), 0 if grad_alias else O.up(trainable * 2, cu_p))),
    "logical gradient not shared out": ("gradient_terms", lambda method, d, trainable, grad_alias, cu_p, align: (
        trainable * 2, 0 if grad_alias else O.up(trainable * 2, cu_p) if method == 0
        else O.up(O.cdiv(O.up(trainable * 2, cu_p), d), align))),
    "logical gradient page-rounded": ("gradient_terms", lambda method, d, trainable, grad_alias, cu_p, align: (
        O.up(trainable * 2, cu_p) if method == 0 else O.cdiv(O.up(trainable * 2, cu_p), d),
        0 if grad_alias else O.up(trainable * 2, cu_p) if method == 0 else O.up(O.cdiv(O.up(trainable * 2, cu_p), d), align))),
    "os shard not rounded": ("resident_bytes", lambda method, d, m_p, m_p16, m_p32, m_os, align: (
        (m_p, m_os) if method == 0 else (m_p16 + O.up(O.cdiv(m_p32, d), align), O.cdiv(m_os, d)) if method == 1
        else (O.up(O.cdiv(m_p, d), align), O.cdiv(m_os, d)))),
    "os not shared out": ("resident_bytes", lambda method, d, m_p, m_p16, m_p32, m_os, align: (
        (m_p, m_os) if method == 0 else (m_p16 + O.up(O.cdiv(m_p32, d), align), m_os) if method == 1
        else (O.up(O.cdiv(m_p, d), align), m_os))),
    "TP param shard uses m_p16": ("resident_bytes", lambda method, d, m_p, m_p16, m_p32, m_os, align: (
        (m_p, m_os) if method == 0 else (m_p16 + O.up(O.cdiv(m_p32, d), align), O.up(O.cdiv(m_os, d), align)) if method == 1
        else (O.up(O.cdiv(m_p16, d), align), O.up(O.cdiv(m_os, d), align)))),
    "TP param shard not rounded": ("resident_bytes", lambda method, d, m_p, m_p16, m_p32, m_os, align: (
        (m_p, m_os) if method == 0 else (m_p16 + O.up(O.cdiv(m_p32, d), align), O.up(O.cdiv(m_os, d), align)) if method == 1
        else (O.cdiv(m_p, d), O.up(O.cdiv(m_os, d), align)))),
    "ZeRO-3 param shard includes fp16": ("resident_bytes", lambda method, d, m_p, m_p16, m_p32, m_os, align: (
        (m_p, m_os) if method == 0 else (O.up(O.cdiv(m_p, d), align), O.up(O.cdiv(m_os, d), align)))),
    "ZeRO-3 param shard not rounded": ("resident_bytes", lambda method, d, m_p, m_p16, m_p32, m_os, align: (
        (m_p, m_os) if method == 0 else (m_p16 + O.cdiv(m_p32, d), O.up(O.cdiv(m_os, d), align)) if method == 1
        else (O.up(O.cdiv(m_p, d), align), O.up(O.cdiv(m_os, d), align)))),
    "search prefers large chunks": ("chunk_search", lambda embed_p, other_p, t_max, cu_p: (10, True)),
    "events not rounded": ("event_value", lambda e, D, method, align: 0 if method not in e.methods else
                           e.sign * O.monomial(e.coef, e.dims, D) * e.elem_bytes * (D["L"] if e.times_L else 1)),
    "method mask ignored": ("event_value", lambda e, D, method, align:
                            e.sign * O.up(O.monomial(e.coef, e.dims, D) * e.elem_bytes, align) * (D["L"] if e.times_L else 1)),
    "all-gather buffer floored": ("event_value", lambda e, D, method, align: 0 if method not in e.methods else e.sign * O.up(
        (O.monomial(e.coef, e.dims, D) * e.elem_bytes * (D["d"] - 1) // D["d"]) if e.scale == "tp_gather"
        else O.monomial(e.coef, e.dims, D) * e.elem_bytes, align) * (D["L"] if e.times_L else 1)),
    "all-gather buffer whole": ("event_value", lambda e, D, method, align: 0 if method not in e.methods else e.sign * O.up(
        O.monomial(e.coef, e.dims, D) * e.elem_bytes, align) * (D["L"] if e.times_L else 1)),
    "per-block events summed before rounding": ("event_value", lambda e, D, method, align: 0 if method not in e.methods else e.sign * O.up(
        (O.cdiv(O.monomial(e.coef, e.dims, D) * e.elem_bytes * (D["d"] - 1), D["d"]) if e.scale == "tp_gather"
         else O.monomial(e.coef, e.dims, D) * e.elem_bytes) * (D["L"] if e.times_L else 1), align)),
    "backward walked once": ("timeline_peak", _wrong_timeline(backward_once=True)),
    "resident state alone not a peak": ("timeline_peak", _wrong_timeline(without_resident=True)),
    "peak taken at segment ends": ("timeline_peak", _wrong_timeline(segment_ends_only=True)),
    "largest tensor over all roles": ("param_census", _wrong_census(t_max_over_all=True)),
    "per-block tensors counted once": ("param_census", _wrong_census(layers_once=True)),
    "tied head counted": ("param_census", _wrong_census(tied_counted=True)),
    "lm_head counted among the embeddings": ("param_census", _wrong_census(embeddings_all=True)),
    "kv width from the model width": ("dim_vector", lambda c: dict(_REAL_DIM_VECTOR(c), kv_dim=c["n_kv"] * c["h"])),
    "shifted length not shortened": ("dim_vector", lambda c: dict(_REAL_DIM_VECTOR(c), sl_m1=c["sl"])),
    "pool split inclusive": ("event_list_peaks", _wrong_event_list(split_inclusive=True)),
    "pool chosen by raw size": ("event_list_peaks", _wrong_event_list(pool_by_raw_size=True)),
    "reserved rounds the sum of the pools": ("event_list_peaks", _wrong_event_list(reserved_of_sum=True)),
    "reserved from the total peak": ("event_list_peaks", _wrong_event_list(reserved_of_total=True)),
    "list events not rounded": ("event_list_peaks", _wrong_event_list(unrounded=True)),
    "empty prefix does not count": ("event_list_peaks", _wrong_event_list(without_empty_prefix=True)),
}
_REAL_DIM_VECTOR = O.dim_vector


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistakes(name, golden, monkeypatch):
    attr, wrong = MUTANTS[name]
    _suite(golden)                                   # passes on the real oracle
    monkeypatch.setattr(O, attr, wrong)
    with pytest.raises(AssertionError):
        _suite(golden)
