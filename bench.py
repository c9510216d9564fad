"""Benchmark: configurations estimated per second on one MI355X.

A step is one pass of the whole hot path over the 10^7-configuration Llama-style
grid with chunk-size search: one llmem_estimate_ex launch producing m_peak and
all detail columns (component sizes, chosen chunk, timeline peak).  Inputs are
generated on the device beforehand and stay resident in HBM.  The explicit
event-list kernel is timed on its own 10^5-list grid and reported under "extra".

Prints ONE JSON line (see README / DESIGN for the fields).
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
PEAK_INT32_TOPS = 256 * 64 * 2.4e9 / 1e12      # 256 CUs x 64 lanes x 2.4 GHz simple int32 lane-ops
PEAK_HBM_GBS = 8000.0


def algorithmic_int32_ops(table, n_search_candidates):
    """Integer work per configuration of the estimator itself, in 32-bit lane
    operations (int64 add/compare/select/shift = 2, u64 x u32 multiply = 4,
    division by d via multiply-high = 16).  Census of the method with the L equal
    blocks collapsed; see the design doc for the derivation."""
    ADD, MUL, DIV = 2, 4, 16
    per_param = 4 * MUL + MUL + 3 * ADD + 2 * ADD + ADD          # monomial, x copies, page round-up, role sums, max
    per_event = 5 * MUL + 3 * ADD + 2 * ADD + ADD + ADD          # monomial*bytes, block round-up, sign/mask, prefix add, max
    fixed = 12 * MUL + 14 * ADD + 2 * DIV                        # m_out, m_lm (3 round-ups), m_back, gradient terms
    per_candidate = 3 * (MUL + 3 * ADD) + 3 * ADD + DIV + 3 * ADD + 6 * ADD   # m_p, m_p16, m_p32, compose, waste, compare
    tail = 3 * DIV + 10 * ADD + 2 * MUL + 12 * ADD                # resident bytes, layer closed form, prelude
    return (len(table.params) * per_param + len(table.events) * per_event + fixed
            + n_search_candidates * per_candidate + tail)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--n", type=int, default=10_000_000, help="configurations per step (default: the 10^7 grid)")
    ap.add_argument("--lists", type=int, default=100_000, help="event lists of the explicit-timeline grid (0: skip)")
    ap.add_argument("--cpu-sample", type=int, default=200_000, help="configurations the CPU oracle is timed on (0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; nothing is sharded and there are no collectives "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2404_10933_amd as M
    from workloads import grids as G
    from workloads import tables as T

    torch.cuda.set_device(0)
    const = T.Constants(m_base=256 << 20)
    table = T.llama_table()
    n = args.n
    dev = M.DeviceConfigs.empty(n)
    M.llmem_grid_generate(4, 0, 0, n, dev)
    tab = M.Tables([table], m_base=const.m_base, cu_p=const.cu_p, align=const.align)
    peaks = torch.empty(n, dtype=torch.int64, device="cuda")
    detail = torch.empty((M.NDETAIL, n), dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()

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

    ops = algorithmic_int32_ops(table, 9)
    achieved = ops * n / (kernel_ms * 1e-3) / 1e12
    bytes_per_cfg = M.llmem_config_bytes(1) + 8 + 8 * M.NDETAIL
    result = {
        "metric": "configs estimated/sec (bit-exact vs oracle)",
        "value": value, "unit": "configs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic",
        "config": {"workload": "g4: Llama-style grid with ZeRO-3 chunk-size search (9 candidates), "
                               "m_peak + all detail columns incl. timeline peak",
                   "n_configs": n, "table_params": len(table.params), "table_events": len(table.events),
                   "seed": 0},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": PEAK_INT32_TOPS, "unit": "Tint32op/s",
                     "frac": achieved / PEAK_INT32_TOPS, "traffic": None,
                     "kernel": "estimate_kernel<true>", "kernel_ms": kernel_ms,
                     "algorithmic_int32_ops_per_config": ops,
                     "hbm_gbs_algorithmic": bytes_per_cfg * n / (kernel_ms * 1e-3) / 1e9},
    }

    # sanity: the benchmark's own output on a slice equals the oracle (not timed)
    from oracle import oracle_c as B
    idx = np.arange(0, min(n, 4096))
    want_p, want_d = B.estimate(G.grid4(n=len(idx), seed=0), [table], const, threads=4)
    assert (peaks[:len(idx)].cpu().numpy() == want_p).all() and \
        (detail[:, :len(idx)].cpu().numpy().T == want_d).all(), "bench output differs from the oracle"
    result["verified_vs_oracle"] = int(len(idx))

    if args.lists > 0:
        nl = args.lists
        counts = torch.empty(nl, dtype=torch.int64, device="cuda")
        M.llmem_events_count(0, 0, nl, counts)
        offsets = torch.zeros(nl + 1, dtype=torch.int64, device="cuda")
        offsets[1:] = torch.cumsum(counts, 0)
        total = int(offsets[-1].item())
        events = torch.empty(total, dtype=torch.int64, device="cuda")
        M.llmem_events_generate(0, 0, nl, offsets, events)
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
        result["extra"] = {"g5_event_lists": {
            "workload": "g5: explicit allocator event lists (~10^4 events each)", "n_lists": nl,
            "n_events": total, "ms_per_launch": ms, "lists_per_s": nl / (ms * 1e-3),
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": gbs / PEAK_HBM_GBS, "traffic": None, "kernel": "timeline_kernel"}}}
        from workloads import events as E
        ev_c, off_c = E.generate(64, seed=0, first=0)
        wa, wr = B.event_lists_peaks(ev_c, off_c)
        assert (oa[:64].cpu().numpy() == wa).all() and (orv[:64].cpu().numpy() == wr).all()
        del events

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
    print(json.dumps(result))


if __name__ == "__main__":
    main()
