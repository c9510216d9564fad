"""Pins of CPU oracle A for the DP+TP estimate (Sec. 5) and the method decision
(Sec. 6, Algorithm 1): a hand-worked example (tests/golden), reductions to the
already pinned ZeRO-3 and TP estimates, an exhaustive search over batch sizes,
rational-arithmetic scores, and planted mistakes the pins must notice."""
import random
from fractions import Fraction

import pytest

from oracle import llmem_oracle as O
from workloads import tables as T
from workloads import grids as G

CONST0 = T.Constants(m_base=0)


def query(**kw):
    base = dict(arch_id=0, h=256, L=4, n_heads=4, n_kv=4, ffn=1024, V=8192, P=512, bs=64, sl=256,
                method=0, d=4, chunk_k=4, flags=G.FLAG_GRAD_ALIAS)
    base.update(kw)
    return base


def test_worked_decision(golden):
    g = golden("worked_decision_gpt_tiny.txt")
    gpt = [T.gpt_table()]
    for tp in (2, 4):
        r = O.method_peaks(query(bs=4), tp, gpt, CONST0)
        assert r[3] == g[f"hybrid_tp{tp}_bs4"]
        assert bool(r[4] & O.HYBRID_READINGS_DIFFER) == bool(g[f"hybrid_tp{tp}_readings_differ"])
        assert O.hybrid_peak(query(bs=4), tp, gpt, CONST0)[0] == g[f"hybrid_tp{tp}_bs4"]
    r = O.decide_one(query(), 2, gpt, CONST0, g["case1_m_total"])
    assert r[O.C_BS_CDP:O.C_BS_CDP + 4] == [g["case1_bs_cdp"], g["case1_bs_adp"], g["case1_bs_tp"], g["case1_bs_hybrid"]]
    assert r[O.C_SCORE2_CDP:O.C_SCORE2_CDP + 4] == [g["case1_score2_cdp"], g["case1_score2_adp"],
                                                   g["case1_score2_tp"], g["case1_score2_hybrid"]]
    assert (r[O.C_METHOD], r[O.C_BS], r[O.C_PEAK], r[O.C_FLAGS]) == (g["case1_method"], g["case1_bs"], g["case1_peak"], 0)
    r = O.decide_one(query(), 2, gpt, CONST0, g["case2_m_total"])
    assert r[O.C_BS_CDP:O.C_BS_CDP + 4] == [0, 0, g["case2_bs_tp"], g["case2_bs_hybrid"]]
    assert r[O.C_SCORE2_TP] == r[O.C_SCORE2_HYBRID] == 4          # the tie goes to TP
    assert (r[O.C_METHOD], r[O.C_BS], r[O.C_PEAK]) == (g["case2_method"], g["case2_bs"], g["case2_peak"])
    r = O.decide_one(query(), 2, gpt, CONST0, g["case3_m_total"])
    assert (r[O.C_METHOD], r[O.C_BS], r[O.C_PEAK], r[O.C_FLAGS]) == (g["case3_method"], g["case3_bs"], 0, 0)
    assert r[O.C_BS_CDP:O.C_SCORE2_HYBRID + 1] == [0] * 8
    r = O.decide_one(query(), 4, gpt, CONST0, g["case4_m_total"])
    assert (r[O.C_METHOD], r[O.C_BS]) == (g["case4_method"], g["case4_bs"])
    assert (r[O.C_BS_HYBRID], r[O.C_SCORE2_HYBRID]) == (g["case4_bs_hybrid"], g["case4_score2_hybrid"])
    assert bool(r[O.C_FLAGS] & O.FALLBACK_READINGS_DIFFER) == bool(g["case4_listing_and_prose_differ"])
    assert r[O.C_FLAGS] & O.HYBRID_READINGS_DIFFER


def _random_queries(rng, n, family):
    out = []
    for _ in range(n):
        if family == "gpt":
            h = rng.choice((128, 256, 512, 768))
            q = query(h=h, L=rng.randint(1, 8), n_heads=h // 64, n_kv=h // 64, ffn=4 * h,
                      V=rng.choice((1000, 8192, 32000)), P=rng.choice((0, 512, 2048)),
                      sl=rng.choice((1, 64, 256, 512)), chunk_k=rng.choice((-1, 2, 4, 6)),
                      flags=rng.randint(0, 7))
        else:
            h = rng.choice((512, 1024, 2048))
            q = query(h=h, L=rng.randint(1, 12), n_heads=h // 128, n_kv=rng.choice((1, 2, 4)),
                      ffn=rng.choice((1376, 2816, 5632)), V=rng.choice((32000, 128256)), P=0,
                      sl=rng.choice((128, 512, 2048)), chunk_k=rng.choice((-1, 3, 5, 8)),
                      flags=rng.randint(0, 7))
        g = rng.choice((1, 2, 3, 4, 6, 8, 12, 16))
        tp = rng.choice([t for t in range(1, g + 1) if g % t == 0])
        q["d"] = g
        out.append((q, tp))
    return out


@pytest.mark.parametrize("family", ("gpt", "llama"))
def test_hybrid_reduces_to_pinned_estimates(family):
    """m_peak^{dp+tp} against the pinned ZeRO-3 and TP estimates: what is added is
    exactly the TP all-gather buffer of a group of tp_n GPUs, what is removed is the
    stated share of param fp16."""
    rng = random.Random(5)
    table = T.gpt_table() if family == "gpt" else T.llama_table()
    for q, tp in _random_queries(rng, 60, family):
        q["bs"] = rng.randint(0, 9)
        g = q["d"]
        const = T.Constants(m_base=rng.choice((0, 12345 * 512)))
        hyb, flags = O.hybrid_peak(q, tp, [table], const)
        zero3 = O.estimate_one(dict(q, method=1), [table], const, False)
        tp_row = O.estimate_one(dict(q, method=2, d=tp), [table], const, False)     # buffer of a tp_n group
        # param fp16 bytes: ZeRO-3 keeps all of them next to the fp32 shard
        D = O.dim_vector(q)
        embed_p, _, other_p, _, _, _ = O.param_census(table, D, False)
        _, m_p16, m_p32 = O.param_memory(embed_p, other_p, O.chunk_elems(zero3[O.D_K]), const.cu_p)
        assert zero3[O.D_PARAM] == m_p16 + O.up(O.cdiv(m_p32, g), const.align)
        removed = zero3[O.D_PEAK] + tp_row[O.D_BACK] - hyb
        # the removed share is m_p16 * tp_n / gpu_n up to one 512-byte block
        assert 0 <= removed * g - m_p16 * tp < 512 * g
        assert removed % 512 == 0
        if tp == g:
            assert removed == m_p16                                   # all of param fp16 leaves the GPU
        if tp == 1:
            assert tp_row[O.D_BACK] == 0
        if (g, tp) == (4, 2):
            assert not flags & O.HYBRID_READINGS_DIFFER               # the paper's 2+2 case: both readings agree
        elif tp * tp != g * (tp - 1) and m_p16 > 512 * g * tp:
            assert flags & O.HYBRID_READINGS_DIFFER
        # never above ZeRO-3 plus the buffer; grows with bs
        assert hyb <= zero3[O.D_PEAK] + tp_row[O.D_BACK]
        assert O.hybrid_peak(dict(q, bs=q["bs"] + 1), tp, [table], const)[0] >= hyb


def test_method_peaks_are_the_single_method_estimates():
    rng = random.Random(6)
    table = T.llama_table()
    for q, tp in _random_queries(rng, 30, "llama"):
        q["bs"] = rng.randint(1, 5)
        r = O.method_peaks(q, tp, [table], CONST0)
        for m in (0, 1, 2):
            assert r[m] == O.estimate_one(dict(q, method=m), [table], CONST0, False)[O.D_PEAK]
        assert r[3] == O.hybrid_peak(q, tp, [table], CONST0)[0]
        assert O.method_peaks(q, 0, [table], CONST0)[3] == -1         # no DP+TP set-up


@pytest.mark.parametrize("family", ("gpt", "llama"))
def test_decision_against_exhaustive_search(family):
    """Batch sizes: the largest bs <= cap whose estimate fits, found by evaluating
    every bs (no early stop).  Scores and choice: rational arithmetic with the
    factor 1.5, a stable sort for the tie order."""
    rng = random.Random(7)
    table = T.gpt_table() if family == "gpt" else T.llama_table()
    seen = set()
    for q, tp in _random_queries(rng, 40, family):
        q["bs"] = cap = rng.randint(0, 12)
        tp_used = rng.choice((tp, tp, 0))
        mid = O.method_peaks(dict(q, bs=rng.randint(0, cap + 1)), tp, [table], CONST0)
        m_total = rng.choice((0, mid[rng.randint(0, 3)] + rng.choice((-1, 0, 1)), 1 << 60))
        row = O.decide_one(q, tp_used, [table], CONST0, m_total)
        best = [0, 0, 0, 0]
        for bs in range(1, cap + 1):
            r = O.method_peaks(dict(q, bs=bs), tp_used, [table], CONST0)
            for i in range(4 if tp_used else 3):
                if r[i] <= m_total:
                    best[i] = bs
        assert row[O.C_BS_CDP:O.C_BS_CDP + 4] == best
        g = q["d"]
        scores = [Fraction(3, 2) * best[0] * g, Fraction(best[1] * g), Fraction(best[2]),
                  Fraction(best[3] * (g // tp_used if tp_used else 0))]
        assert [Fraction(x, 2) for x in row[O.C_SCORE2_CDP:O.C_SCORE2_CDP + 4]] == scores
        order = sorted(range(4), key=lambda i: -scores[i])            # stable: ties keep CDP, ADP, TP, DP+TP
        if scores[2] != 0:
            want = (order[0], best[order[0]])
        else:
            want = (4, 0)
        assert (row[O.C_METHOD], row[O.C_BS]) == want
        if want[0] < 4:
            assert row[O.C_PEAK] == O.method_peaks(dict(q, bs=want[1]), tp_used, [table], CONST0)[want[0]]
            assert row[O.C_PEAK] <= m_total
        assert bool(row[O.C_FLAGS] & O.FALLBACK_READINGS_DIFFER) == (scores[2] == 0 and any(scores))
        seen.add(want[0])
    assert {0, 4} <= seen and len(seen) >= 3


def test_decision_limits():
    gpt = [T.gpt_table()]
    # capacity never binding: every method reaches the cap, CDP's factor 1.5 wins for any gpu_n
    for g, tp in ((1, 1), (4, 2), (8, 8)):
        r = O.decide_one(query(d=g, bs=7), tp, gpt, CONST0, 1 << 62)
        assert r[O.C_BS_CDP:O.C_BS_CDP + 4] == [7, 7, 7, 7] and (r[O.C_METHOD], r[O.C_BS]) == (0, 7)
    # nothing fits
    r = O.decide_one(query(), 2, gpt, CONST0, 0)
    assert (r[O.C_METHOD], r[O.C_BS]) == (4, 0) and not r[O.C_FLAGS] & O.FALLBACK_READINGS_DIFFER
    # cap 0: no batch size is tried
    r = O.decide_one(query(bs=0), 2, gpt, CONST0, 1 << 62)
    assert (r[O.C_METHOD], r[O.C_BS]) == (4, 0)
    # more capacity never lowers a batch size
    prev = [0, 0, 0, 0]
    for m_total in range(30 << 20, 400 << 20, 37 << 20):
        cur = O.decide_one(query(), 2, gpt, CONST0, m_total)[O.C_BS_CDP:O.C_BS_CDP + 4]
        assert all(c >= p for c, p in zip(cur, prev))
        prev = cur


def test_invalid_queries_are_flagged():
    gpt = [T.gpt_table()]
    for kw, tp, bit in ((dict(d=4), 3, O.ERR_TP), (dict(d=0), 1, O.ERR_D), (dict(n_heads=0), 1, O.ERR_HEADS),
                        (dict(arch_id=1), 1, O.ERR_ARCH), (dict(chunk_k=17), 1, O.ERR_CHUNK),
                        (dict(d=6, chunk_k=-2), 4, O.ERR_TP | O.ERR_CHUNK)):
        r = O.decide_one(query(**kw), tp, gpt, CONST0, 1 << 40)
        assert r[O.C_METHOD] == -1 and r[O.C_FLAGS] == bit and r[O.C_BS:O.C_FLAGS] == [0] * 10
        assert O.method_peaks(query(**kw), tp, gpt, CONST0) == [-1, -1, -1, -1, bit]
    # the method field of a query is not read
    assert O.decide_one(query(method=9), 2, gpt, CONST0, 1 << 28) == O.decide_one(query(method=0), 2, gpt, CONST0, 1 << 28)


# ---------------------------------------------------------------------------
# the pins notice plausible mistakes: plant them in the oracle, on the CPU
# ---------------------------------------------------------------------------
def _suite(golden):
    test_worked_decision(golden)
    test_hybrid_reduces_to_pinned_estimates("gpt")
    test_decision_against_exhaustive_search("gpt")
    test_decision_limits()


def _first_max_from_the_end(score2, bs_list):
    idx = max(range(len(score2)), key=lambda i: (score2[i], i))
    return (idx, bs_list[idx], False) if score2[2] != 0 else (4, 0, any(score2))


def _largest_batch_off_by_one(peak_of_bs, bs_cap, m_total):
    bs = 1
    while bs <= bs_cap and peak_of_bs(bs) <= m_total:
        bs += 1
    return min(bs, bs_cap), (peak_of_bs(min(bs, bs_cap)) if bs_cap else 0)


def _largest_batch_strict(peak_of_bs, bs_cap, m_total):
    bs, last = 1, 0
    while bs <= bs_cap and peak_of_bs(bs) < m_total:
        last = peak_of_bs(bs)
        bs += 1
    return bs - 1, last


MUTANTS = {
    "subtrahend is the other reading": ("hybrid_subtrahends", lambda m_p16, tp_n, gpu_n, align: (
        O.up(O.cdiv(m_p16 * (tp_n - 1), tp_n), align),) * 2),
    "subtrahend over tp_n": ("hybrid_subtrahends", lambda m_p16, tp_n, gpu_n, align: (
        O.up(O.cdiv(m_p16, tp_n), align), O.up(O.cdiv(m_p16 * (tp_n - 1), tp_n), align))),
    "subtrahend floors": ("hybrid_subtrahends", lambda m_p16, tp_n, gpu_n, align: (
        (m_p16 * tp_n // gpu_n) // align * align, O.up(O.cdiv(m_p16 * (tp_n - 1), tp_n), align))),
    "buffer of all gpu_n GPUs": ("hybrid_peak", lambda c, tp_n, tables, const: (
        O.estimate_one(dict(c, method=1), tables, const, False)[O.D_PEAK]
        - O.hybrid_subtrahends(_m_p16(c, tables, const), tp_n, c["d"], const.align)[0]
        + O.tp_backward_memory(O.dim_vector(c), c["d"], const.cu_p), 0)),
    "hybrid adds the share": ("hybrid_peak", lambda c, tp_n, tables, const: (
        O.estimate_one(dict(c, method=1), tables, const, False)[O.D_PEAK]
        + O.hybrid_subtrahends(_m_p16(c, tables, const), tp_n, c["d"], const.align)[0]
        + O.tp_backward_memory(O.dim_vector(c), tp_n, const.cu_p), 0)),
    "hybrid built on the TP estimate": ("hybrid_peak", lambda c, tp_n, tables, const: (
        O.estimate_one(dict(c, method=2), tables, const, False)[O.D_PEAK]
        - O.hybrid_subtrahends(_m_p16(c, tables, const), tp_n, c["d"], const.align)[0], 0)),
    "batch size one too large": ("largest_batch", _largest_batch_off_by_one),
    "capacity must not be reached": ("largest_batch", _largest_batch_strict),
    "CDP without the factor 1.5": ("scores_doubled", lambda bs, g, dp: [2 * bs[0] * g, 2 * bs[1] * g, 2 * bs[2], 2 * bs[3] * dp]),
    "factor 1.5 on ADP": ("scores_doubled", lambda bs, g, dp: [2 * bs[0] * g, 3 * bs[1] * g, 2 * bs[2], 2 * bs[3] * dp]),
    "TP scaled by gpu_n": ("scores_doubled", lambda bs, g, dp: [3 * bs[0] * g, 2 * bs[1] * g, 2 * bs[2] * g, 2 * bs[3] * dp]),
    "DP+TP scaled by gpu_n": ("scores_doubled", lambda bs, g, dp: [3 * bs[0] * g, 2 * bs[1] * g, 2 * bs[2], 2 * bs[3] * g]),
    "ties go to the last method": ("choose", _first_max_from_the_end),
    "fallback only when all scores are zero": ("choose", lambda s, b: (
        (max(range(4), key=lambda i: (s[i], -i)), b[max(range(4), key=lambda i: (s[i], -i))], False) if any(s) else (4, 0, False))),
    "fallback tested on CDP": ("choose", lambda s, b: (
        (max(range(4), key=lambda i: (s[i], -i)), b[max(range(4), key=lambda i: (s[i], -i))], False) if s[0] != 0
        else (4, 0, any(s)))),
}


def _m_p16(c, tables, const):
    table = tables[c["arch_id"]]
    D = O.dim_vector(c)
    embed_p, _, other_p, _, _, _ = O.param_census(table, D, False)
    k = O.estimate_one(dict(c, method=1), tables, const, False)[O.D_K]
    return O.param_memory(embed_p, other_p, O.chunk_elems(k), const.cu_p)[1]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistakes(name, golden, monkeypatch):
    attr, wrong = MUTANTS[name]
    _suite(golden)                                   # passes on the real oracle
    monkeypatch.setattr(O, attr, wrong)
    with pytest.raises(AssertionError):
        _suite(golden)
