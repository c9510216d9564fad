"""Operation census of the estimator: how many integer operations one configuration
costs in the leanest form of the definition, counted from the tables alone.

TEST AND MEASUREMENT INFRASTRUCTURE ONLY (the oracle's side of the roofline: the
benchmark divides this census by the measured time to say how fast the *method*
is being evaluated, next to the instructions the kernel actually issues).  It
knows nothing of any kernel: the counts follow from the equations of Sec. 4.2 and
Sec. 5, the chunk-size search of Sec. 4.1 and the traversal of Sec. 2.1 / Sec. 3.1
as `llmem_oracle.py` states them, with three algebraic facts applied that keep
every result the same integer:

  * tensors (and events) whose size is the same expression are evaluated once
    ("groups" of parameter entries, "size classes" of events);
  * the L equal blocks need one walk: repetition r of a segment shifts every
    prefix sum by r times the segment's net change, so the largest prefix over
    the repetitions lies in the first or the last one;
  * within a segment the live total can only peak right after an allocation that
    is followed by a release (or ends the segment), and a candidate whose vector
    of per-class event counts is nowhere above another candidate's can never
    exceed it, since sizes are not negative.

Operations are counted by kind and priced in 64-bit lane operations of a machine
without a native 64-bit multiplier or divider (gfx950's vector unit):
  add    64-bit add / subtract / shift                                   1
  mul32  32 x 32 -> 64-bit multiply(-add)                                1
  mul    64-bit value times 32-bit value                                 3
  up     round up to a power-of-two unit (add, and-not or two shifts)    3
  max    compare and select                                              3
  div    ceiling division by the partition degree (multiply-high)       12
"""
from __future__ import annotations

from typing import Dict

PRICE = {"add": 1, "mul32": 1, "mul": 3, "up": 3, "max": 3, "div": 12}
SEGMENTS = ("A", "F", "H", "B", "Z")


def _product(dims):
    return tuple(sorted(d for d in dims if d != "one"))


def lean_counts(table) -> Dict[str, int]:
    """Parameter groups, size classes, kept peak points and (class, count) terms of one
    architecture table, from its entries alone."""
    groups = {(p.coef, _product(p.dims)) for p in table.params}

    def key(e):
        return (e.coef, _product(e.dims), e.elem_bytes, e.times_L, e.scale == "tp_gather", frozenset(e.methods))

    classes = sorted({key(e) for e in table.events}, key=repr)
    terms = points = 0
    for seg in SEGMENTS:
        evs = [e for e in table.events if e.seg == seg]
        count, seen = {c: 0 for c in classes}, []
        for j, e in enumerate(evs):
            count[key(e)] += e.sign
            if e.sign > 0 and (j + 1 == len(evs) or evs[j + 1].sign < 0):
                seen.append(tuple(count[c] for c in classes))
        kept = []
        for j, v in enumerate(seen):
            dominated = any(k != j and all(a <= b for a, b in zip(v, w)) and (v != w or k < j)
                            for k, w in enumerate(seen))
            if not dominated:
                kept.append(v)
        points += len(kept)
        terms += sum(1 for v in kept + [tuple(count[c] for c in classes)] for x in v if x != 0)
    return dict(param_groups=len(groups), size_classes=len(classes), terms=terms, peak_points=points)


def _ops(**kinds) -> Dict[str, int]:
    out = {k: 0 for k in PRICE}
    out.update(kinds)
    return out


def _scaled(ops: Dict[str, int], times: int) -> Dict[str, int]:
    return {k: v * times for k, v in ops.items()}


def _sum(*parts: Dict[str, int]) -> Dict[str, int]:
    return {k: sum(p[k] for p in parts) for k in PRICE}


def estimate_census(table, n_candidates: int) -> Dict[str, object]:
    """One configuration through the whole path (closed forms, `n_candidates` chunk sizes, all
    detail columns, the timeline peak).  Returns the counts by kind, the priced total
    (`lane_ops`) and the table's lean counts."""
    lean = lean_counts(table)
    # a parameter group: its expression (two dimensions beyond the first product on average are
    # priced as one 32-bit and one wide multiply), its share of a role's sum (count * L multiply,
    # add), its optimizer-state pages (times 8, page round-up, times count, add), the largest tensor
    per_group = _ops(mul32=3, mul=3, add=3, up=1, max=1)
    # a size class: expression (one 32-bit, two wide multiplies), block round-up, store
    per_class = _ops(mul32=1, mul=2, up=1, add=1)
    per_term = _ops(mul=1, add=1)                      # count * value, accumulate
    per_point = _ops(max=1)
    # m_out and m_lm (Sec. 4.2), m_back^tp (Sec. 5), the gradient sizes (Sec. 4.1)
    fixed = _sum(_ops(mul=3, up=1), _ops(mul=4, up=2, add=3), _ops(mul=3, up=1, div=1), _ops(mul=2, div=1))
    # one chunk-size candidate: chunked count, m_p / m_p16 / m_p32, the shard, compose, waste, keep the best
    per_candidate = _ops(add=7, mul=3, up=4, div=1, max=2)
    # per-GPU parameter and optimizer bytes, closing five segments (L * net change, two maxima), resident sum
    tail = _sum(_ops(div=2, up=2), _scaled(_ops(mul=1, max=1, add=2), 5), _ops(add=4))
    total = _sum(_scaled(per_group, lean["param_groups"]), _scaled(per_class, lean["size_classes"]),
                 _scaled(per_term, lean["terms"]), _scaled(per_point, lean["peak_points"]), fixed,
                 _scaled(per_candidate, n_candidates), tail)
    return dict(ops=total, lane_ops=sum(PRICE[k] * v for k, v in total.items()), **lean)


def sweep_extra_census() -> Dict[str, object]:
    """What drawing a configuration of the Llama-style grids in registers and folding its results
    into the statistics adds: eight counter-based draws (splitmix64's finaliser: two 64 x 64-bit
    multiplies at 4 lane operations, three xor-shifts at 2, one add), four remainders by constants
    that are no powers of two (priced as divisions), the feed-forward width (one division, three
    adds), ten selections, score and packing (5), eight statistics with group and test (12)."""
    lane_ops = 8 * (1 + 3 * 2 + 2 * 4) + 4 * (12 + 1) + 4 * 2 + (4 + 2) + (12 + 3) + 10 + 5 + 12
    return dict(lane_ops=lane_ops)


def decide_census(table, probes: int) -> Dict[str, object]:
    """One query of Algorithm 1 (Sec. 6) in its leanest form: the parameter census by groups, the
    chunk size in closed form (the smallest feasible candidate is the least-waste one), the
    batch-independent parts of the four estimates, per method a bracket of the largest batch size
    from the estimate's linear growth (18 single-precision operations) and `probes` evaluations
    of the batch-dependent terms counted in 32-bit pages, scores, choice, the chosen estimate."""
    lean = lean_counts(table)
    per_group = _ops(mul32=3, mul=3, add=3, up=1, max=1)
    chunk = _ops(max=1, add=3)
    fixed = _sum(_scaled(_ops(mul=1, up=1), 3), _scaled(_ops(div=1, up=1), 2), _scaled(_ops(mul=1, div=1, up=1), 2),
                 _ops(add=22, mul=5))
    bracket = _ops(add=18)
    probe_plain = _ops(mul32=4, add=7, max=1)
    probe_gather = _sum(probe_plain, _ops(mul32=2, add=8))       # the all-gather buffer: a 32-bit division by t (5)
    tail = _sum(_ops(mul32=4, max=3, up=1, add=4), probe_gather)
    total = _sum(_scaled(per_group, lean["param_groups"]), chunk, fixed, _scaled(bracket, 4),
                 _scaled(_sum(_scaled(probe_plain, 2), _scaled(probe_gather, 2)), probes), tail)
    return dict(ops=total, lane_ops=sum(PRICE[k] * v for k, v in total.items()), **lean)
