"""Benchmark: configurations estimated per second on one MI355X.

A step is one pass of the whole hot path over the 10^7-configuration Llama-style
grid with chunk-size search: one llmem_estimate_ex launch producing m_peak and
all detail columns (component sizes, chosen chunk, timeline peak).  Inputs are
generated on the device beforehand and stay resident in HBM.  Reported
under "extra", each timed on its own: the explicit event-list kernel on the
10^5-list grid, the same grid with the table without gradient checkpointing, the
streaming sweep (draw, estimate, reduce in one kernel) and the method decision.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X nominal peaks used for the roofline fractions
PEAK_LANE_TOPS = 256 * 64 * 2.4e9 / 1e12       # 256 CUs x one 64-lane vector instruction per clock x 2.4 GHz
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs under profiles/, scaled by the
# plain-copy reference; None while the kernel has changed since the counters were taken
TRAFFIC_ESTIMATE = 1.3691e9     # 10^7 configurations, all detail columns, built-in compiled form (incl. 8 B/lane of spill scratch)
TRAFFIC_SPECIALIZED = 1.3503e9  # the same workload, kernel built at run time
TRAFFIC_SWEEP = 5.0558e7        # 10^7 configurations drawn and reduced in the kernel built at run time
TRAFFIC_TIMELINE = 8.0182e9     # 100 000 event lists, 1 000 110 810 events
TRAFFIC_DECIDE = 5.4027e8       # 4 000 000 queries, all decision columns (the search inside the kernel does not touch memory)
# Vector instructions issued per wave of 64 units (SQ_INSTS_VALU of the same runs), i.e. per unit and lane;
# with them `issued` = the share of the nominal vector issue slots the kernel fills, whatever the census says
VALU_ESTIMATE = 1815            # built-in compiled form, per configuration
VALU_SPECIALIZED = 1332         # kernel built at run time
VALU_SWEEP = 1483
VALU_DECIDE = 938.6             # per query


def issued(valu_per_unit, units_per_s):
    """Vector lane-instructions issued per second against the nominal issue rate (None: no counter for this kernel)."""
    if valu_per_unit is None:
        return None
    rate = valu_per_unit * units_per_s / 1e12
    return {"valu_per_unit": valu_per_unit, "achieved": rate, "frac": rate / PEAK_LANE_TOPS}


def algorithmic_lane_ops(forms, n_candidates):
    """Integer work of one configuration in 64-bit lane operations of the method itself, in its
    leanest known form (equal size expressions evaluated once, the L equal blocks collapsed, the
    timeline reduced to the peak points no other point dominates), priced in gfx950 vector
    instructions: add/sub 1, 32x32->64 multiply 1, multiply of a 64-bit value by a 32-bit one 3,
    round up to a power of two 3, compare-and-select (max) 3, ceil-divide by d 12.
    `forms` = llmem_kernel_forms of the tables."""
    ADD, MUL32, MUL, UP, MAX, DIV = 1, 1, 3, 3, 3, 12
    per_group = MUL32 + MUL + (MUL32 + MUL + ADD) + (ADD + UP + MUL32 + MUL + ADD) + MAX   # expression, role sum, m_os, t_max
    per_class = MUL32 + 2 * MUL + UP + ADD                                                 # expression, block round-up, store
    per_term = MUL + ADD
    per_point = MAX
    fixed = (2 * MUL + MUL + UP) + (2 * MUL + 2 * (MUL + UP) + 3 * ADD) + (3 * MUL + UP + DIV) + 2 * MUL + DIV
    per_candidate = 2 * ADD + 3 * (MUL + UP) + DIV + UP + 5 * ADD + 2 * MAX
    tail = 2 * (DIV + UP) + 5 * (MUL + MAX + 2 * ADD) + 4 * ADD
    return (forms["param_groups"] * per_group + forms["size_classes"] * per_class + forms["terms"] * per_term
            + forms["peak_points"] * per_point + fixed + n_candidates * per_candidate + tail)


def algorithmic_lane_ops_decide(n_param_groups, probes):
    """The method decision of one query in the same units, leanest known form: parameter census
    by groups of equal size expression, the chunk size in closed form (the smallest feasible
    candidate is the one with the least waste), the batch-independent parts of the four estimates,
    the per-page constants of the batch-dependent terms, then per method the bracket of the largest
    batch size in single precision (one reciprocal, two products, conversions and clamps) and
    `probes` estimates of the batch-dependent terms counted in 32-bit pages (one to check the
    bracket's lower end, the rest bisecting the bracket), scores, choice and the chosen estimate."""
    ADD, MUL32, MUL, UP, MAX, DIV, DIV32 = 1, 1, 3, 3, 3, 12, 5
    per_group = MUL32 + MUL + (MUL32 + MUL + ADD) + (ADD + UP + MUL32 + MUL + ADD) + MAX
    chunk = MAX + 3 * ADD                                        # bit length of t_max, clamp to 2..10
    fixed = 3 * (MUL + UP) + 2 * (DIV + UP) + 2 * (MUL + DIV + UP) + 12 * ADD + 5 * MUL + 10 * ADD
    bracket = 18                                                 # room in pages, growth, quotient, two clamped ends
    probe_plain = MUL32 + 3 * (MUL32 + ADD) + 4 * ADD + MAX      # shared whole pages; three remainders; compare, keep
    probe_gather = probe_plain + 2 * MUL32 + 2 * ADD + DIV32 + ADD   # plus the all-gather buffer, divided by t
    tail = 4 * MUL32 + 3 * MAX + probe_gather + UP + 4 * ADD
    return (n_param_groups * per_group + chunk + fixed + 4 * bracket
            + probes * (2 * probe_plain + 2 * probe_gather) + tail)


def algorithmic_lane_ops_sweep_extra():
    """What the streaming sweep adds per configuration of grid 4, same units: eight counter-based
    draws (the part of the hash input that all fields share, once; per draw one add and the
    splitmix64 finaliser: two 64 x 64-bit multiplies at 4 (two 32-bit products, one 32 x 32 -> 64
    multiply-add, one add), three xor-shifts at 2; then a remainder, priced like a division, 12, by
    a constant that is no power of two, else 1, and the offset), the SwiGLU width, the value
    selections, the score and the eight statistics."""
    ADD, MUL64, XORSHIFT, REM, DIV = 1, 4, 2, 12, 12
    draw = ADD + 3 * XORSHIFT + 2 * MUL64
    draws = 8 * draw + 4 * (REM + ADD) + 4 * (1 + ADD) + (MUL64 + 2 * ADD)
    shape = (DIV + 3 * ADD) + 10                  # ffn = 8h/3 rounded up to 256; table look-ups as selects
    fold = 3 + 2 + 8 + 4                          # score, packed best entry, eight statistics, group and test
    return draws + shape + fold


def timed_ms(fn, reps=3):
    """Mean duration of fn() in ms by HIP events on the current stream, after one untimed call."""
    import torch
    fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--n", type=int, default=10_000_000, help="configurations per step (default: the 10^7 grid)")
    ap.add_argument("--lists", type=int, default=100_000, help="event lists of the explicit-timeline grid (0: skip)")
    ap.add_argument("--full-traversal", type=int, default=10_000_000,
                    help="configurations timed with the table without gradient checkpointing (0: skip)")
    ap.add_argument("--sweep", type=int, default=10_000_000,
                    help="configurations of the streaming sweep (drawn, estimated and reduced in one kernel; 0: skip)")
    ap.add_argument("--queries", type=int, default=4_000_000, help="queries of the method-decision grid (0: skip)")
    ap.add_argument("--cpu-sample", type=int, default=600_000, help="configurations the CPU oracle is timed on (0: skip)")
    ap.add_argument("--kernel", choices=("specialized", "auto", "wave", "lane"), default="specialized",
                    help="estimator kernel: the lane kernel built at run time with the tables as constants (built "
                         "during warm-up, build time reported), the library's own choice among the built-in forms, "
                         "one wavefront or one lane per configuration")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy ten times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; nothing is sharded and there are no collectives "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2404_10933_amd as M
    from workloads import grids as G
    from workloads import tables as T

    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 27, dtype=torch.int64, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read": src.numel() * 8, "bytes_written": src.numel() * 8,
                                             "launches": 10}}))
        return
    const = T.Constants(m_base=256 << 20)
    table = T.llama_table()
    n = args.n
    dev = M.DeviceConfigs.empty(n)
    generators = {"grid4_ms": timed_ms(lambda: M.llmem_grid_generate(4, 0, 0, n, dev)), "grid4_configs": n}
    kernel = {"auto": 0, "wave": 1, "lane": 2, "specialized": 5}[args.kernel]
    tab = M.Tables([table], m_base=const.m_base, cu_p=const.cu_p, align=const.align, kernel=kernel)
    peaks = torch.empty(n, dtype=torch.int64, device="cuda")
    detail = torch.empty((M.NDETAIL, n), dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    build_s, kernel_note = None, args.kernel
    if args.kernel == "specialized":
        # the first call builds and loads the kernel for these tables; not part of the timed steps
        t0 = time.perf_counter()
        try:
            M.llmem_estimate_ex(dev, tab, peaks, detail, n=64)
            torch.cuda.synchronize()
            build_s = time.perf_counter() - t0
            kernel_note = (f"specialized (built at run time, or loaded from LLMEM_KERNEL_CACHE, before the warm-up: "
                           f"{build_s:.2f} s)")
        except M.LlmemError as e:
            kernel, kernel_note = 0, f"auto (the run-time build failed: {e})"
            tab = M.Tables([table], m_base=const.m_base, cu_p=const.cu_p, align=const.align, kernel=0)

    for _ in range(args.warmup):
        M.llmem_estimate_ex(dev, tab, peaks, detail)
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        starts[s].record()
        M.llmem_estimate_ex(dev, tab, peaks, detail)          # launched on torch's current stream
        stops[s].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = sum(a.elapsed_time(b) for a, b in zip(starts, stops)) / args.steps
    ms_per_step = wall * 1e3 / args.steps
    value = n / (ms_per_step * 1e-3)

    forms = M.llmem_kernel_forms(tab)
    ops = algorithmic_lane_ops(forms, 9)
    achieved = ops * n / (kernel_ms * 1e-3) / 1e12
    kernel_name = {1: "estimate_kernel<true>", 5: "llmem_specialized_detail"}.get(kernel, "estimate_batch_kernel<true, true, false>")
    bytes_per_cfg = M.llmem_config_bytes(1) + 8 + 8 * M.NDETAIL
    result = {
        "metric": "configs estimated/sec (bit-exact vs oracle)",
        "value": value, "unit": "configs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic",
        "config": {"workload": "g4: Llama-style grid with ZeRO-3 chunk-size search (9 candidates), "
                               "m_peak + all detail columns incl. timeline peak",
                   "n_configs": n, "table_params": len(table.params), "table_events": len(table.events),
                   "table_size_classes": forms["size_classes"], "table_peak_points": forms["peak_points"],
                   "table_terms": forms["terms"], "kernel": kernel_note, "seed": 0},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": PEAK_LANE_TOPS, "unit": "Tlane-op/s",
                     "frac": achieved / PEAK_LANE_TOPS,
                     "traffic": ({0: TRAFFIC_ESTIMATE, 5: TRAFFIC_SPECIALIZED}.get(kernel) if n == 10_000_000 else None),
                     "kernel": kernel_name, "kernel_ms": kernel_ms,
                     "algorithmic_lane_ops_per_config": ops,
                     "issued": issued({0: VALU_ESTIMATE, 5: VALU_SPECIALIZED}.get(kernel) if n == 10_000_000 else None,
                                      n / (kernel_ms * 1e-3)),
                     "hbm_gbs_algorithmic": bytes_per_cfg * n / (kernel_ms * 1e-3) / 1e9},
    }

    # sanity: the benchmark's own output on a slice equals the oracle (not timed)
    from oracle import oracle_c as B
    idx = np.arange(0, min(n, 4096))
    want_p, want_d = B.estimate(G.grid4(n=len(idx), seed=0), [table], const, threads=4)
    assert (peaks[:len(idx)].cpu().numpy() == want_p).all() and \
        (detail[:, :len(idx)].cpu().numpy().T == want_d).all(), "bench output differs from the oracle"
    result["verified_vs_oracle"] = int(len(idx))

    if kernel == 5:
        itab = M.Tables([table], m_base=const.m_base, cu_p=const.cu_p, align=const.align, kernel=0)
        for _ in range(2):
            M.llmem_estimate_ex(dev, itab, peaks, detail)
        torch.cuda.synchronize()
        reps = 10
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            M.llmem_estimate_ex(dev, itab, peaks, detail)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        i_achieved = ops * n / (ms * 1e-3) / 1e12
        assert (peaks[:len(idx)].cpu().numpy() == want_p).all() and \
            (detail[:, :len(idx)].cpu().numpy().T == want_d).all(), "built-in kernel's output differs from the oracle"
        result.setdefault("extra", {})["g4_built_in_kernel"] = {
            "workload": "the headline workload with the built-in compiled form (tables read from the kernel arguments)",
            "n_configs": n, "ms_per_launch": ms, "configs_per_s": n / (ms * 1e-3),
            "roofline": {"bound": "alu", "achieved": i_achieved, "peak": PEAK_LANE_TOPS, "unit": "Tlane-op/s",
                         "frac": i_achieved / PEAK_LANE_TOPS, "traffic": TRAFFIC_ESTIMATE if n == 10_000_000 else None,
                         "kernel": "estimate_batch_kernel<true, true, false>", "algorithmic_lane_ops_per_config": ops,
                         "issued": issued(VALU_ESTIMATE if n == 10_000_000 else None, n / (ms * 1e-3))},
            "verified_vs_oracle": int(len(idx))}

    if args.lists > 0:
        nl = args.lists
        counts = torch.empty(nl, dtype=torch.int64, device="cuda")
        M.llmem_events_count(0, 0, nl, counts)
        offsets = torch.zeros(nl + 1, dtype=torch.int64, device="cuda")
        offsets[1:] = torch.cumsum(counts, 0)
        total = int(offsets[-1].item())
        events = torch.empty(total, dtype=torch.int64, device="cuda")
        generators["event_lists_ms"] = timed_ms(lambda: M.llmem_events_generate(0, 0, nl, offsets, events))
        generators["event_lists"] = nl
        oa = torch.empty(nl, dtype=torch.int64, device="cuda")
        orv = torch.empty(nl, dtype=torch.int64, device="cuda")
        for _ in range(2):
            M.llmem_timeline_peaks(events, offsets, oa, orv)
        torch.cuda.synchronize()
        reps = 10
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            M.llmem_timeline_peaks(events, offsets, oa, orv)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        nbytes = 8 * total + 8 * (nl + 1) + 16 * nl
        gbs = nbytes / (ms * 1e-3) / 1e9
        result.setdefault("extra", {})["g5_event_lists"] = {
            "workload": "g5: explicit allocator event lists (~10^4 events each)", "n_lists": nl,
            "n_events": total, "ms_per_launch": ms, "lists_per_s": nl / (ms * 1e-3),
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": gbs / PEAK_HBM_GBS, "traffic": TRAFFIC_TIMELINE if nl == 100_000 else None,
                         "kernel": "timeline_kernel"}}
        from workloads import events as E
        ev_c, off_c = E.generate(64, seed=0, first=0)
        wa, wr = B.event_lists_peaks(ev_c, off_c)
        assert (oa[:64].cpu().numpy() == wa).all() and (orv[:64].cpu().numpy() == wr).all()
        del events

    if args.full_traversal > 0:
        nf = min(args.full_traversal, n)
        ftab = M.Tables([T.llama_table(checkpoint=False)], m_base=const.m_base + (64 << 20), cu_p=const.cu_p,
                        align=const.align, kernel=kernel)
        for _ in range(2):
            M.llmem_estimate_ex(dev, ftab, peaks, detail, n=nf)
        torch.cuda.synchronize()
        reps = 10
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            M.llmem_estimate_ex(dev, ftab, peaks, detail, n=nf)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        fforms = M.llmem_kernel_forms(ftab)
        f_ops = algorithmic_lane_ops(fforms, 9)
        f_achieved = f_ops * nf / (ms * 1e-3) / 1e12
        ns = min(4096, nf)
        fconst = T.Constants(m_base=const.m_base + (64 << 20), cu_p=const.cu_p, align=const.align)
        want_p, want_d = B.estimate(G.grid4(n=ns, seed=0), [T.llama_table(checkpoint=False)], fconst, threads=4)
        assert (peaks[:ns].cpu().numpy() == want_p).all() and (detail.view(-1)[:M.NDETAIL * nf].view(M.NDETAIL, nf)[:, :ns]
                                                                .cpu().numpy().T == want_d).all(), \
            "full-traversal output differs from the oracle"
        result.setdefault("extra", {})["g4_full_traversal"] = {
            "workload": "g4 with the Llama table without gradient checkpointing (every saved forward output alive "
                        "until its backward), 64 MiB allocator buffer added to m_base; all detail columns",
            "n_configs": nf, "ms_per_launch": ms, "configs_per_s": nf / (ms * 1e-3),
            "table_events": len(T.llama_table(checkpoint=False).events), "table_terms": fforms["terms"],
            "table_peak_points": fforms["peak_points"],
            "roofline": {"bound": "alu", "achieved": f_achieved, "peak": PEAK_LANE_TOPS, "unit": "Tlane-op/s",
                         "frac": f_achieved / PEAK_LANE_TOPS, "traffic": None, "kernel": kernel_name,
                         "algorithmic_lane_ops_per_config": f_ops},
            "verified_vs_oracle": ns}

    if args.sweep > 0:
        nsw, m_total = args.sweep, 64 << 30
        stats = torch.empty((M.NSWEEP, M.SWEEP_GROUPS), dtype=torch.int64, device="cuda")
        if kernel == 1:        # the sweep is a mode of the lane kernel: with --kernel wave the library chooses its form
            tab = M.Tables([table], m_base=const.m_base, cu_p=const.cu_p, align=const.align, kernel=0)
        for _ in range(2):
            M.llmem_sweep_reset(stats)
            M.llmem_sweep(4, 0, 0, nsw, tab, m_total, stats)
        torch.cuda.synchronize()
        reps = 10
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            M.llmem_sweep_reset(stats)
            M.llmem_sweep(4, 0, 0, nsw, tab, m_total, stats)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        s_ops = ops + algorithmic_lane_ops_sweep_extra()
        s_achieved = s_ops * nsw / (ms * 1e-3) / 1e12
        ns = min(100_000, nsw)
        head = torch.empty_like(stats)
        M.llmem_sweep_reset(head)
        M.llmem_sweep(4, 0, 0, ns, tab, m_total, head)
        want = B.sweep(G.grid4(n=ns, seed=0), 0, [table], const, m_total, threads=4)
        assert (head.cpu().numpy() == want).all(), "sweep statistics differ from the oracle"
        assert int(stats[0].sum().item()) == nsw
        result.setdefault("extra", {})["g4_streaming_sweep"] = {
            "workload": "g4 drawn in registers, estimated (all of the hot path) and folded into 8 statistics per "
                        "(method, gpu_n) against m_total 64 GiB; nothing per configuration touches HBM; reset + sweep",
            "n_configs": nsw, "ms_per_launch": ms, "configs_per_s": nsw / (ms * 1e-3),
            "configs_fitting": int(stats[1].sum().item()),
            "roofline": {"bound": "alu", "achieved": s_achieved, "peak": PEAK_LANE_TOPS, "unit": "Tlane-op/s",
                         "frac": s_achieved / PEAK_LANE_TOPS,
                         "traffic": TRAFFIC_SWEEP if (kernel == 5 and nsw == 10_000_000) else None,
                         "kernel": "llmem_specialized_sweep" if kernel == 5 else "estimate_batch_kernel<true, true, true>",
                         "algorithmic_lane_ops_per_config": s_ops,
                         "issued": issued(VALU_SWEEP if (kernel == 5 and nsw == 10_000_000) else None, nsw / (ms * 1e-3))},
            "verified_vs_oracle": ns}

    if args.queries > 0:
        nq, m_total = args.queries, 80 << 30
        del peaks, detail
        qdev = M.DeviceConfigs.empty(nq)
        tp = torch.empty(nq, dtype=torch.uint8, device="cuda")
        generators["queries_ms"] = timed_ms(lambda: M.llmem_queries_generate(0, 0, nq, qdev, tp))
        generators["queries"] = nq
        qtab = M.Tables([table], m_base=const.m_base, cu_p=const.cu_p, align=const.align)
        q_method = torch.empty(nq, dtype=torch.int32, device="cuda")
        q_bs = torch.empty(nq, dtype=torch.int32, device="cuda")
        q_det = torch.empty((M.NDECIDE, nq), dtype=torch.int64, device="cuda")
        for _ in range(2):
            M.llmem_decide(qdev, tp, qtab, m_total, q_method, q_bs, q_det)
        torch.cuda.synchronize()
        reps = 10
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            M.llmem_decide(qdev, tp, qtab, m_total, q_method, q_bs, q_det)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        # bracket check + one bisection step (brackets of <= 1 for this grid's models)
        q_ops = algorithmic_lane_ops_decide(M.llmem_kernel_forms(qtab)["param_groups"], 2)
        q_achieved = q_ops * nq / (ms * 1e-3) / 1e12
        q_bytes = 31 + 1 + 4 + 4 + 8 * M.NDECIDE                       # query columns, tp_n; method, bs, decision columns
        q_gbs = q_bytes * nq / (ms * 1e-3) / 1e9
        ns = min(2000, nq)
        qs, qs_tp = G.grid6(n=ns, seed=0)
        t1 = time.perf_counter()
        want = B.decide(qs, qs_tp, [table], const, m_total, threads=1)
        dt = time.perf_counter() - t1
        assert (q_det[:, :ns].cpu().numpy().T == want).all(), "decisions differ from the oracle"
        result.setdefault("extra", {})["g6_method_decision"] = {
            "workload": "g6: Algorithm 1 per query (Llama-style model, gpu_n, sl; batch sizes up to 4096; "
                        "m_total 80 GiB), method + bs + all decision columns",
            "n_queries": nq, "ms_per_launch": ms, "queries_per_s": nq / (ms * 1e-3),
            # 136 B per query at 8 TB/s take longer than the census at the vector issue rate: HBM bounds it
            "roofline": {"bound": "hbm", "achieved": q_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": q_gbs / PEAK_HBM_GBS,
                         "traffic": TRAFFIC_DECIDE if nq == 4_000_000 else None, "kernel": "decide_kernel<true>",
                         "algorithmic_bytes_per_query": q_bytes,
                         "alu": {"achieved": q_achieved, "peak": PEAK_LANE_TOPS, "unit": "Tlane-op/s",
                                 "frac": q_achieved / PEAK_LANE_TOPS, "algorithmic_lane_ops_per_query": q_ops,
                                 "issued": issued(VALU_DECIDE if nq == 4_000_000 else None, nq / (ms * 1e-3))}},
            "cpu_oracle": {"value": ns / dt, "unit": "queries/s", "cores": 1,
                           "sample": f"first {ns} queries, C oracle (one-by-one search), {dt:.1f} s"},
            "verified_vs_oracle": ns}

    if args.cpu_sample > 0:
        ns = min(args.cpu_sample, n)
        sample = G.grid4(n=ns, seed=0)
        t1 = time.perf_counter()
        B.estimate(sample, [table], const, timeline=True, threads=1)
        dt = time.perf_counter() - t1
        result["cpu_baseline"] = {"value": ns / dt, "unit": "configs/s", "cores": 1, "kind": "oracle",
                                  "sample": f"first {ns} configurations of the same grid, all detail columns, "
                                            f"C oracle single-threaded, {dt:.1f} s",
                                  "host_cores_visible": os.cpu_count()}
    # the seeded inputs are generated on the device before anything is timed; what generating them takes
    result["generators"] = generators
    print(json.dumps(result))


if __name__ == "__main__":
    main()
