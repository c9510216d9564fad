"""Benchmark: configurations estimated per second on one MI355X.

A step is one pass of the whole hot path over the 10^7-configuration Llama-style
grid with chunk-size search: one llmem_estimate_ex launch producing m_peak and
all detail columns (component sizes, chosen chunk, timeline peak), with the
kernel the library chooses by itself (the specialized kernel built into it for
the Llama-style table).  Inputs are generated on the device beforehand and stay
resident in HBM.  Reported under "extra", each timed on its own: the literal
llmem_estimate call (m_peak only), grids 1 to 3, the same workload through the
other kernel forms, the explicit event-list kernel on the 10^5-list grid, the
table without gradient checkpointing, the streaming sweep and the method decision.

Roofline fractions of the integer-bound kernels are the share of the vector issue
slots the kernel fills: vector instructions per configuration as the hardware
counters gave them (profiles/counters.json, valid only while the kernel sources
are the ones that were profiled) times the measured rate, over the nominal issue
rate.  Next to it, "census": the operations of the method itself in its leanest
form, counted on the oracle's side from the tables alone and priced in 64-bit lane
operations, and how many instructions the kernel issues per such operation.

Prints ONE JSON line.  `--import-counters DIR` (no GPU needed) instead turns the
rocprofv3 counter files under DIR into profiles/counters.json.
"""
import argparse
import collections
import csv
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X nominal peaks used for the roofline fractions
PEAK_LANE_TOPS = 256 * 64 * 2.4e9 / 1e12       # 256 CUs x one 64-lane vector instruction per clock x 2.4 GHz
PEAK_HBM_GBS = 8000.0

COUNTERS_FILE = os.path.join(ROOT, "profiles", "counters.json")
CSRC = os.path.join("paper_2404_10933_amd", "csrc")
LANE_SOURCES = [os.path.join(CSRC, f) for f in ("estimate_batch.hip", "estimate_args.h", "wave.h", "grid_draws.h")] \
    + [os.path.join("include", "llmem.h"), os.path.join("workloads", "tables.py")]
# key -> (substring of the kernel's name, work-items of a launch over the whole workload: at least, below,
#         units per launch, sources the kernel is compiled from[, (i, of): the launches that match, in the order
#         they were made, fall into `of` equal runs and the i-th is this workload's])
PROFILED = {
    "g4_detail": ("llmem_aot_llama_detail", 2_000_000, 1 << 62, 10_000_000, LANE_SOURCES),
    "g4_peaks": ("llmem_aot_llama_peaks", 2_000_000, 1 << 62, 10_000_000, LANE_SOURCES),
    "g4_sweep": ("llmem_aot_llama_sweep", 1_000_000, 1 << 62, 10_000_000, LANE_SOURCES),
    "g4_full_traversal": ("llmem_aot_llama_full_detail", 2_000_000, 1 << 62, 10_000_000, LANE_SOURCES),
    "g4_compiled": ("estimate_batch_kernel<true, 1, false>", 2_000_000, 1 << 62, 10_000_000, LANE_SOURCES),
    "g3_detail": ("llmem_aot_llama_detail", 500_000, 2_000_000, 1_000_000, LANE_SOURCES),
    "g2_detail": ("llmem_aot_opt_detail", 50_000, 500_000, 100_000, LANE_SOURCES),
    "g5_lists": ("timeline_kernel", 0, 1 << 62, 100_000, [os.path.join(CSRC, "timeline.hip"), os.path.join(CSRC, "wave.h")]),
    "g6_decide": ("decide_kernel<true>", 0, 1 << 62, 4_000_000,
                  [os.path.join(CSRC, "decide.hip"), os.path.join(CSRC, "estimate_args.h"), os.path.join(CSRC, "wave.h")],
                  (0, 2)),                  # the second run of launches is the one without the decision columns
}


def source_checksum(paths):
    """Checksum of the kernel sources as the compiler sees them: comments and white space do not count."""
    h = hashlib.sha256()
    for p in paths:
        text = open(os.path.join(ROOT, p)).read()
        if p.endswith(".py"):
            text = re.sub(r"#[^\n]*", "", text)
        else:
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            text = re.sub(r"//[^\n]*", "", text)
        h.update(re.sub(r"\s+", " ", text).encode())
    return h.hexdigest()[:16]


def counters_for(key, units):
    """The profiled counters of a kernel, or None when the sources have changed since or the workload differs."""
    try:
        entry = json.load(open(COUNTERS_FILE))["kernels"][key]
    except (OSError, KeyError, ValueError):
        return None
    if entry["units"] != units or entry["checksum"] != source_checksum(PROFILED[key][4]):
        return None
    return entry


def import_counters(folder):
    """profiles/counters.json from rocprofv3 --pmc runs of this file under `folder`: sub-folders
    pmc_sq, pmc_fetch, pmc_write (this benchmark) and copy_fetch, copy_write (--calibrate-copy),
    each holding *_counter_collection.csv."""
    def read(sub, want, lo=0, hi=1 << 62, part=None):
        agg = collections.defaultdict(list)
        names = [f for f in os.listdir(os.path.join(folder, sub)) if f.endswith("counter_collection.csv")]
        rows = sorted(csv.DictReader(open(os.path.join(folder, sub, names[0]))), key=lambda r: int(r["Dispatch_Id"]))
        for r in rows:
            if want in r["Kernel_Name"] and lo <= int(r["Grid_Size"]) < hi:
                agg[r["Counter_Name"]].append(float(r["Counter_Value"]))
        if part is not None:
            agg = {k: v[len(v) * part[0] // part[1]: len(v) * (part[0] + 1) // part[1]] for k, v in agg.items()}
        return {k: sum(v) / len(v) for k, v in agg.items()}

    copy_fetch = read("copy_fetch", "copyBuffer")["FETCH_SIZE"]
    copy_write = read("copy_write", "copyBuffer")["WRITE_SIZE"]
    scale_f, scale_w = (1 << 20) / copy_fetch, (1 << 20) / copy_write        # a 1 GiB copy reads and writes 2^20 KiB
    out = {"note": "written by `python bench.py --import-counters DIR` from rocprofv3 --pmc runs of bench.py; "
                   "per launch over the whole workload; a kernel's entry is used only while `checksum` equals "
                   "the checksum of its sources (comments and white space aside)",
           "copy_reference": {"fetch_kib_per_gib_copied": copy_fetch, "write_kib_per_gib_copied": copy_write,
                              "fetch_scale": scale_f, "write_scale": scale_w},
           "kernels": {}}
    for key, (want, lo, hi, units, sources, *rest) in PROFILED.items():
        part = rest[0] if rest else None
        sq = read("pmc_sq", want, lo, hi, part)
        f = read("pmc_fetch", want, lo, hi, part).get("FETCH_SIZE")
        w = read("pmc_write", want, lo, hi, part).get("WRITE_SIZE")
        if not sq or f is None or w is None:
            print(f"{key}: not in the counter files, left out", file=sys.stderr)
            continue
        out["kernels"][key] = {
            "kernel": want, "units": units, "checksum": source_checksum(sources),
            "valu_per_unit": sq["SQ_INSTS_VALU"] * 64 / units, "salu_per_64_units": sq.get("SQ_INSTS_SALU", 0) * 64 / units,
            "lds_per_64_units": sq.get("SQ_INSTS_LDS", 0) * 64 / units,
            "valu_per_cu_clock": sq["SQ_INSTS_VALU"] / sq["SQ_BUSY_CU_CYCLES"] if sq.get("SQ_BUSY_CU_CYCLES") else None,
            "fetch_kib": f, "write_kib": w, "traffic_bytes": (f * scale_f + w * scale_w) * 1024}
    out["calibration"] = read_calibration()
    with open(COUNTERS_FILE, "w") as fh:
        json.dump(out, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print(f"{COUNTERS_FILE}: {sorted(out['kernels'])}")


def read_calibration():
    """What the stand-alone calibration program sustained on the box (profiles/calibrate_*.md): the mean
    issue rate of the 64-bit integer instructions the kernels are made of, per compute unit and nominal
    clock, and the best streaming read rate."""
    path = os.path.join(ROOT, "profiles", "calibrate_gfx950_instruction_rates.md")
    rates, reads, pattern = [], [], []
    try:
        for line in open(path):
            f = line.split()
            if f and f[0] in ("v_mad_u64_u32", "v_lshl_add_u64", "v_cmp_gt_i64", "v_cndmask_b32"):
                rates.append(float(f[-1]))
            if line.startswith("HBM streaming read"):
                reads.append(float(f[-2]))
            if line.startswith("estimate pattern 31 B in 104 out"):      # first the library's launch shape, then one batch per wavefront
                pattern.append(float(f[-2]))
    except OSError:
        return None
    if not rates or not reads:
        return None
    out = {"valu_per_cu_clock": sum(rates) / len(rates), "hbm_read_gbs": max(reads), "source": os.path.basename(path)}
    if pattern:
        out["estimate_pattern_gbs"] = pattern[0]
    return out


def calibration():
    try:
        return json.load(open(COUNTERS_FILE)).get("calibration")
    except (OSError, ValueError):
        return None


def alu_roofline(key, units, ms, kernel_name, census_ops=None):
    """Roofline object of an integer-bound kernel: issue-slot share from the counters, census beside it."""
    c = counters_for(key, units) if key in PROFILED else None
    rate = units / (ms * 1e-3)
    out = {"bound": "alu", "achieved": None, "peak": PEAK_LANE_TOPS, "unit": "Tlane-op/s", "frac": None,
           "basis": "vector instructions issued per unit (hardware counter) x units per second, against one 64-lane "
                    "instruction per compute unit and clock at 2.4 GHz: what 64-bit integer instructions sustain; plain "
                    "32-bit add/and/mov/xor issue at up to 1.6 per compute unit and clock (calibration program), so a "
                    "kernel rich in them - the sweep's draws - can pass 1.  null: no counters for this kernel and "
                    "workload, or its sources have changed since those in profiles/counters.json were taken",
           "traffic": None, "kernel": kernel_name, "kernel_ms": ms}
    if c is not None:
        out.update(achieved=c["valu_per_unit"] * rate / 1e12, frac=c["valu_per_unit"] * rate / 1e12 / PEAK_LANE_TOPS,
                   traffic=c["traffic_bytes"], valu_per_unit=c["valu_per_unit"])
        cal = calibration()
        if cal:         # against what the calibration program sustains for 64-bit integer instructions on the box
            out["calibrated"] = {"peak": PEAK_LANE_TOPS * cal["valu_per_cu_clock"],
                                 "frac": out["frac"] / cal["valu_per_cu_clock"]}
    if census_ops is not None:
        # context, not a fraction of any peak: a kernel that works in 32-bit pages and blocks issues fewer
        # instructions than the census prices in 64-bit operations
        out["census"] = {"lane_ops_per_unit": census_ops, "census_ops_per_s": census_ops * rate,
                         "issued_per_census_op": c["valu_per_unit"] / census_ops if c is not None else None,
                         "basis": "operations of the method in its leanest form, counted from the tables by "
                                  "oracle/census.py and priced in 64-bit lane operations"}
    return out


LEG_MS = {"warm": 60.0, "timed": 200.0}      # set from --leg-warm-ms and --leg-ms


def timed_ms(fn, reps=None, warm=None):
    """Mean duration of fn() in ms by HIP events on the current stream, after untimed calls.  The GPU
    raises its clock over the first tens of milliseconds of continuous work and drops it again when
    idle, so every leg warms up by itself: unless given, the untimed calls and the timed calls are as
    many as fill LEG_MS["warm"] and LEG_MS["timed"] milliseconds (at least 1 and 3).  The counts used
    are left in timed_ms.last."""
    import torch

    def run(count):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(count):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / count

    fn()
    torch.cuda.synchronize()
    estimate = max(run(2), 1e-3)
    if reps is None or warm is None:
        warm = min(max(int(LEG_MS["warm"] / estimate), 1), 20000) if warm is None else warm
        reps = min(max(int(LEG_MS["timed"] / estimate), 3), 50000) if reps is None else reps
    run(warm)
    timed_ms.last = (reps, warm)
    return run(reps)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=300, help="untimed steps before the timed ones (the GPU reaches its "
                                                            "clock under load after some 100 launches of 0.3 ms)")
    ap.add_argument("--leg-ms", type=float, default=200.0, help="timed milliseconds of every other workload (0: three calls)")
    ap.add_argument("--leg-warm-ms", type=float, default=60.0, help="untimed milliseconds before them (0: one call)")
    ap.add_argument("--n", type=int, default=10_000_000, help="configurations per step (default: the 10^7 grid)")
    ap.add_argument("--lists", type=int, default=100_000, help="event lists of the explicit-timeline grid (0: skip)")
    ap.add_argument("--full-traversal", type=int, default=10_000_000,
                    help="configurations timed with the table without gradient checkpointing (0: skip)")
    ap.add_argument("--sweep", type=int, default=10_000_000,
                    help="configurations of the streaming sweep (drawn, estimated and reduced in one kernel; 0: skip)")
    ap.add_argument("--queries", type=int, default=4_000_000, help="queries of the method-decision grid (0: skip)")
    ap.add_argument("--grids", type=int, default=1, help="also time grids 1 to 3 and the m_peak-only call (0: skip)")
    ap.add_argument("--forms", type=int, default=1, help="also time the other kernel forms on the headline workload (0: skip)")
    ap.add_argument("--cpu-sample", type=int, default=600_000, help="configurations the CPU oracle is timed on (0: skip)")
    ap.add_argument("--kernel", choices=("auto", "compiled", "runtime", "wave", "events"), default="auto",
                    help="estimator kernel of the headline: the library's own choice (the specialized kernel built into "
                         "it for the shipped tables), the lane kernel that reads the compiled tables from its arguments, "
                         "the specialized kernel built at run time (before the warm-up, build time reported), one "
                         "wavefront per configuration, one lane per configuration walking every event")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy ten times (reference for the HBM byte counters)")
    ap.add_argument("--import-counters", metavar="DIR", help="write profiles/counters.json from rocprofv3 output (no GPU)")
    args = ap.parse_args()
    LEG_MS["timed"], LEG_MS["warm"] = args.leg_ms, args.leg_warm_ms
    if args.import_counters:
        import_counters(args.import_counters)
        return
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
    # the oracle: checks of what is timed, the operation census, and the CPU baseline at the end
    from oracle import census as C
    from oracle import oracle_c as B

    const = T.Constants(m_base=256 << 20)
    table = T.llama_table()
    n = args.n
    dev = M.DeviceConfigs.empty(n)
    generators = {"grid4_ms": timed_ms(lambda: M.llmem_grid_generate(4, 0, 0, n, dev)), "grid4_configs": n}
    kernel = {"auto": 0, "wave": 1, "events": 3, "compiled": 4, "runtime": 6}[args.kernel]

    def tables_of(tabs, k=0, m_base=const.m_base):
        return M.Tables(tabs, m_base=m_base, cu_p=const.cu_p, align=const.align, kernel=k)

    tab = tables_of([table], kernel)
    forms = M.llmem_kernel_forms(tab)
    peaks = torch.empty(n, dtype=torch.int64, device="cuda")
    detail = torch.empty((M.NDETAIL, n), dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    kernel_note = {"auto": "auto: the specialized kernel built into the library for this table"
                           if forms["prebuilt"][1] else "auto: no built-in specialization matches, compiled form",
                   "compiled": "compiled tables read from the kernel arguments", "wave": "one wavefront per configuration",
                   "events": "one lane per configuration, every event walked"}.get(args.kernel)
    if args.kernel == "runtime":
        # the first call builds and loads the kernel for these tables; not part of the timed steps
        t0 = time.perf_counter()
        M.llmem_estimate_ex(dev, tab, peaks, detail, n=64)
        torch.cuda.synchronize()
        kernel_note = (f"specialized kernel built at run time, or loaded from LLMEM_KERNEL_CACHE, before the warm-up: "
                       f"{time.perf_counter() - t0:.2f} s")

    for _ in range(args.warmup):
        M.llmem_estimate_ex(dev, tab, peaks, detail)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for s in range(args.steps):
        M.llmem_estimate_ex(dev, tab, peaks, detail)          # launched on torch's current stream
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = start.elapsed_time(stop) / args.steps         # average launch, HIP events on the launch stream
    ms_per_step = wall * 1e3 / args.steps
    value = n / (ms_per_step * 1e-3)

    census = C.estimate_census(table, 9)
    assert {k: census[k] for k in ("param_groups", "size_classes", "terms", "peak_points")} \
        == {k: forms[k] for k in ("param_groups", "size_classes", "terms", "peak_points")}
    headline_key = {"auto": "g4_detail", "compiled": "g4_compiled"}.get(args.kernel, "none")
    kernel_name = {"auto": "llmem_aot_llama_detail" if forms["prebuilt"][1] else "estimate_batch_kernel<true, 1, false>",
                   "compiled": "estimate_batch_kernel<true, 1, false>", "runtime": "llmem_specialized_detail",
                   "wave": "estimate_kernel<true>", "events": "estimate_batch_kernel<true, 0, false>"}[args.kernel]
    bytes_per_cfg = M.llmem_config_bytes(1) + 8 + 8 * M.NDETAIL
    roofline = alu_roofline(headline_key, n, kernel_ms, kernel_name, census["lane_ops"])
    roofline["census"]["ops_by_kind"] = census["ops"]
    roofline["hbm_gbs_algorithmic"] = bytes_per_cfg * n / (kernel_ms * 1e-3) / 1e9
    # the other roof: by the published peaks the issue floor of this kernel lies above its HBM floor (hence "alu");
    # by what the box reaches the two are level - the launch's access pattern alone, without any arithmetic
    # (calibration program), takes nearly as long as the launch
    roofline["hbm"] = {"achieved": roofline["hbm_gbs_algorithmic"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": roofline["hbm_gbs_algorithmic"] / PEAK_HBM_GBS, "bytes_per_unit": bytes_per_cfg}
    cal = calibration()
    if cal and cal.get("estimate_pattern_gbs"):
        roofline["hbm"]["access_pattern_alone_gbs"] = cal["estimate_pattern_gbs"]
        roofline["hbm"]["frac_of_access_pattern_alone"] = roofline["hbm_gbs_algorithmic"] / cal["estimate_pattern_gbs"]
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
        "roofline": roofline,
    }
    extra = result.setdefault("extra", {})

    # sanity: the benchmark's own output on a slice equals the oracle (not timed)
    idx = np.arange(0, min(n, 4096))
    want_p, want_d = B.estimate(G.grid4(n=len(idx), seed=0), [table], const, threads=4)

    def same_as_oracle():
        return bool((peaks[:len(idx)].cpu().numpy() == want_p).all()
                    and (detail.view(-1)[:M.NDETAIL * n].view(M.NDETAIL, n)[:, :len(idx)].cpu().numpy().T == want_d).all())

    assert same_as_oracle(), "bench output differs from the oracle"
    result["verified_vs_oracle"] = int(len(idx))

    if args.grids:
        # the plain entry point: m_peak only, on the default stream (which is torch's current one here)
        assert torch.cuda.current_stream().cuda_stream == 0
        peaks.fill_(-7)
        ptab = tables_of([table])
        ms = timed_ms(lambda: M.llmem_estimate(dev, ptab, peaks))
        assert (peaks[:len(idx)].cpu().numpy() == want_p).all(), "llmem_estimate differs from the oracle"
        extra["g4_peaks_only"] = {
            "workload": "llmem_estimate(configs, n, method_tables, out_peaks): g4, m_peak only (39 B per configuration; "
                        "no timeline walk: peak_live is a detail column)",
            "n_configs": n, "ms_per_launch": ms, "timed_launches": timed_ms.last[0], "configs_per_s": n / (ms * 1e-3),
            "hbm_gbs_algorithmic": (M.llmem_config_bytes(1) + 8) * n / (ms * 1e-3) / 1e9,
            "roofline": alu_roofline("g4_peaks", n, ms, "llmem_aot_llama_peaks"), "verified_vs_oracle": int(len(idx))}
        for name, make, family, n_grid in (("g1", G.grid1, "gpt", 432), ("g2", G.grid2, "opt", 100_000),
                                           ("g3", G.grid3, "llama", 1_000_000)):
            gtab_py = T.FAMILIES[family]()
            gtab = tables_of([gtab_py])
            gdev = M.DeviceConfigs.empty(n_grid)
            M.llmem_grid_generate(int(name[1]), 0, 0, n_grid, gdev)
            gp = torch.empty(n_grid, dtype=torch.int64, device="cuda")
            gd = torch.empty((M.NDETAIL, n_grid), dtype=torch.int64, device="cuda")
            ms = timed_ms(lambda: M.llmem_estimate_ex(gdev, gtab, gp, gd))
            ns = min(n_grid, 4096)
            gcfg = make() if name == "g1" else make(n=ns, seed=0)
            wp, wd = B.estimate(gcfg, [gtab_py], const, threads=4)
            assert (gp[:ns].cpu().numpy() == wp).all() and (gd[:, :ns].cpu().numpy().T == wd).all(), name
            gcensus = C.estimate_census(gtab_py, 1)              # the chunk size is given in grids 1 to 3
            t1 = time.perf_counter()
            B.estimate(gcfg, [gtab_py], const, timeline=True, threads=1)
            dt = time.perf_counter() - t1
            extra[name] = {
                "workload": {"g1": "g1: tiny Cartesian grid, GPT-style table, all detail columns (a latency: two workgroups)",
                             "g2": "g2: 10^5 OPT-style configurations, all detail columns",
                             "g3": "g3: 10^6 Llama-style configurations, all detail columns"}[name],
                "n_configs": n_grid, "ms_per_launch": ms, "timed_launches": timed_ms.last[0], "configs_per_s": n_grid / (ms * 1e-3),
                "roofline": alu_roofline(name + "_detail", n_grid, ms, f"llmem_aot_{family}_detail", gcensus["lane_ops"]),
                "cpu_oracle": {"value": ns / dt, "unit": "configs/s", "cores": 1, "sample": f"first {ns} configurations, {dt:.2f} s"},
                "verified_vs_oracle": ns}
            del gdev, gp, gd

    if args.forms and args.kernel == "auto":
        for name, k, key, kname in (("g4_compiled_form", 4, "g4_compiled", "estimate_batch_kernel<true, 1, false>"),
                                    ("g4_built_at_run_time", 6, "none", "llmem_specialized_detail")):
            ftab = tables_of([table], k)
            t1 = time.perf_counter()
            try:
                M.llmem_estimate_ex(dev, ftab, peaks, detail, n=64)
                torch.cuda.synchronize()
            except M.LlmemError as e:                          # e.g. the run-time compiler inside a profiled process
                extra[name] = {"skipped": str(e)}
                continue
            first_call_s = time.perf_counter() - t1
            peaks.fill_(-7)
            ms = timed_ms(lambda: M.llmem_estimate_ex(dev, ftab, peaks, detail))
            assert same_as_oracle(), name
            extra[name] = {
                "workload": {4: "the headline workload with the lane kernel that reads the compiled tables from its arguments "
                                "(what tables without a built-in specialization get from LLMEM_KERNEL_AUTO)",
                             6: "the headline workload with the specialized kernel built at run time (hiprtc; "
                                "LLMEM_KERNEL_LANE_RUNTIME), first call incl. the build reported"}[k],
                "n_configs": n, "ms_per_launch": ms, "timed_launches": timed_ms.last[0], "configs_per_s": n / (ms * 1e-3), "first_call_s": first_call_s,
                "roofline": alu_roofline(key, n, ms, kname, census["lane_ops"]), "verified_vs_oracle": int(len(idx))}

    if args.forms:
        # a table with hundreds of distinct event sizes: no form with class slots takes it; the library's choice
        # (every event evaluated where it stands, one lane per configuration) against one wavefront per configuration
        wide = T.random_table(np.random.default_rng(11), 64, 700, "many sizes")
        nw = 1_000_000
        wcfg = G.random_configs(np.random.default_rng(12), nw, n_arch=1)
        wdev = M.DeviceConfigs.from_numpy(wcfg)
        wp = torch.empty(nw, dtype=torch.int64, device="cuda")
        wd = torch.empty((M.NDETAIL, nw), dtype=torch.int64, device="cuda")
        ns = 2048
        want_wp, want_wd = B.estimate(G.slice_configs(wcfg, np.arange(ns)), [wide], const, threads=4)
        entry = {"workload": "10^6 random configurations with a random table of 64 parameter entries and 700 events in "
                             f"{C.lean_counts(wide)['size_classes']} distinct sizes, all detail columns",
                 "n_configs": nw, "allowed_forms": M.llmem_kernel_forms(tables_of([wide]))["allowed"]}
        for label, k in (("auto_lane_direct", 0), ("wave", 1)):
            wtab = tables_of([wide], k)
            wp.fill_(-7)
            ms = timed_ms(lambda: M.llmem_estimate_ex(wdev, wtab, wp, wd))
            assert (wp[:ns].cpu().numpy() == want_wp).all() and (wd[:, :ns].cpu().numpy().T == want_wd).all(), label
            entry[label] = {"ms_per_launch": ms, "timed_launches": timed_ms.last[0], "configs_per_s": nw / (ms * 1e-3)}
        entry["speedup_over_wave"] = entry["wave"]["ms_per_launch"] / entry["auto_lane_direct"]["ms_per_launch"]
        entry["verified_vs_oracle"] = ns
        extra["many_size_classes"] = entry
        del wdev, wp, wd

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
        ms = timed_ms(lambda: M.llmem_timeline_peaks(events, offsets, oa, orv))
        nbytes = 8 * total + 8 * (nl + 1) + 16 * nl
        gbs = nbytes / (ms * 1e-3) / 1e9
        c = counters_for("g5_lists", nl)
        extra["g5_event_lists"] = {
            "workload": "g5: explicit allocator event lists (~10^4 events each)", "n_lists": nl,
            "n_events": total, "ms_per_launch": ms, "timed_launches": timed_ms.last[0], "lists_per_s": nl / (ms * 1e-3),
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": gbs / PEAK_HBM_GBS, "traffic": c["traffic_bytes"] if c else None,
                         "algorithmic_bytes": nbytes, "kernel": "timeline_kernel"}}
        if calibration():
            read = calibration()["hbm_read_gbs"]            # the calibration program's best streaming read
            extra["g5_event_lists"]["roofline"]["calibrated"] = {"peak": read, "frac": gbs / read}
        from workloads import events as E
        ev_c, off_c = E.generate(64, seed=0, first=0)
        wa, wr = B.event_lists_peaks(ev_c, off_c)
        assert (oa[:64].cpu().numpy() == wa).all() and (orv[:64].cpu().numpy() == wr).all()
        del events

    if args.full_traversal > 0:
        nf = min(args.full_traversal, n)
        full = T.llama_table(checkpoint=False)
        ftab = tables_of([full], kernel, const.m_base + (64 << 20))
        ms = timed_ms(lambda: M.llmem_estimate_ex(dev, ftab, peaks, detail, n=nf))
        fforms = M.llmem_kernel_forms(ftab)
        ns = min(4096, nf)
        fconst = T.Constants(m_base=const.m_base + (64 << 20), cu_p=const.cu_p, align=const.align)
        wp, wd = B.estimate(G.grid4(n=ns, seed=0), [full], fconst, threads=4)
        assert (peaks[:ns].cpu().numpy() == wp).all() and (detail.view(-1)[:M.NDETAIL * nf].view(M.NDETAIL, nf)[:, :ns]
                                                            .cpu().numpy().T == wd).all(), \
            "full-traversal output differs from the oracle"
        extra["g4_full_traversal"] = {
            "workload": "g4 with the Llama table without gradient checkpointing (every saved forward output alive "
                        "until its backward), 64 MiB allocator buffer added to m_base; all detail columns",
            "n_configs": nf, "ms_per_launch": ms, "timed_launches": timed_ms.last[0], "configs_per_s": nf / (ms * 1e-3),
            "table_events": len(full.events), "table_terms": fforms["terms"], "table_peak_points": fforms["peak_points"],
            "roofline": alu_roofline("g4_full_traversal" if kernel == 0 else "none", nf, ms,
                                     "llmem_aot_llama_full_detail" if kernel == 0 else kernel_name,
                                     C.estimate_census(full, 9)["lane_ops"]),
            "verified_vs_oracle": ns}

    if args.sweep > 0:
        nsw, m_total = args.sweep, 64 << 30
        stats = torch.empty((M.NSWEEP, M.SWEEP_GROUPS), dtype=torch.int64, device="cuda")
        stab = tables_of([table], 0 if kernel in (1, 3) else kernel)        # the sweep is a mode of the lane kernel

        def reset_and_sweep():
            M.llmem_sweep_reset(stats)
            M.llmem_sweep(4, 0, 0, nsw, stab, m_total, stats)

        ms = timed_ms(reset_and_sweep)
        ns = min(100_000, nsw)
        head = torch.empty_like(stats)
        M.llmem_sweep_reset(head)
        M.llmem_sweep(4, 0, 0, ns, stab, m_total, head)
        want = B.sweep(G.grid4(n=ns, seed=0), 0, [table], const, m_total, threads=4)
        assert (head.cpu().numpy() == want).all(), "sweep statistics differ from the oracle"
        assert int(stats[0].sum().item()) == nsw
        extra["g4_streaming_sweep"] = {
            "workload": "g4 drawn in registers, estimated (all of the hot path) and folded into 8 statistics per "
                        "(method, gpu_n) against m_total 64 GiB; nothing per configuration touches HBM; reset + sweep",
            "n_configs": nsw, "ms_per_launch": ms, "timed_launches": timed_ms.last[0], "configs_per_s": nsw / (ms * 1e-3),
            "configs_fitting": int(stats[1].sum().item()),
            "roofline": alu_roofline("g4_sweep" if kernel == 0 else "none", nsw, ms,
                                     "llmem_aot_llama_sweep" if kernel == 0 else "lane kernel, sweep mode",
                                     census["lane_ops"] + C.sweep_extra_census()["lane_ops"]),
            "verified_vs_oracle": ns}

    if args.queries > 0:
        nq, m_total = args.queries, 80 << 30
        del peaks, detail
        qdev = M.DeviceConfigs.empty(nq)
        tp = torch.empty(nq, dtype=torch.uint8, device="cuda")
        generators["queries_ms"] = timed_ms(lambda: M.llmem_queries_generate(0, 0, nq, qdev, tp))
        generators["queries"] = nq
        qtab = tables_of([table])
        q_method = torch.empty(nq, dtype=torch.int32, device="cuda")
        q_bs = torch.empty(nq, dtype=torch.int32, device="cuda")
        q_det = torch.empty((M.NDECIDE, nq), dtype=torch.int64, device="cuda")
        ms = timed_ms(lambda: M.llmem_decide(qdev, tp, qtab, m_total, q_method, q_bs, q_det))
        ms_short = timed_ms(lambda: M.llmem_decide(qdev, tp, qtab, m_total, q_method, q_bs, None), *timed_ms.last)   # as many launches
        # bracket check + one bisection step (brackets of <= 1 for this grid's models)
        q_census = C.decide_census(table, 2)
        q_bytes = 31 + 1 + 4 + 4 + 8 * M.NDECIDE                       # query columns, tp_n; method, bs, decision columns
        q_gbs = q_bytes * nq / (ms * 1e-3) / 1e9
        ns = min(2000, nq)
        qs, qs_tp = G.grid6(n=ns, seed=0)
        t1 = time.perf_counter()
        want = B.decide(qs, qs_tp, [table], const, m_total, threads=1)
        dt = time.perf_counter() - t1
        assert (q_det[:, :ns].cpu().numpy().T == want).all(), "decisions differ from the oracle"
        assert (q_method[:ns].cpu().numpy() == want[:, 0]).all() and (q_bs[:ns].cpu().numpy() == want[:, 1]).all()
        c = counters_for("g6_decide", nq)
        alu = alu_roofline("g6_decide", nq, ms, "decide_kernel<true>", q_census["lane_ops"])
        extra["g6_method_decision"] = {
            "workload": "g6: Algorithm 1 per query (Llama-style model, gpu_n, sl; batch sizes up to 4096; "
                        "m_total 80 GiB), method + bs + all decision columns",
            "n_queries": nq, "ms_per_launch": ms, "timed_launches": timed_ms.last[0], "queries_per_s": nq / (ms * 1e-3),
            # 136 B per query at 8 TB/s take longer than the census at the vector issue rate: HBM bounds it
            "roofline": {"bound": "hbm", "achieved": q_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": q_gbs / PEAK_HBM_GBS, "traffic": c["traffic_bytes"] if c else None,
                         "kernel": "decide_kernel<true>", "algorithmic_bytes_per_query": q_bytes, "alu": alu},
            "method_and_bs_only": {"workload": "the same queries, out_detail = NULL (40 B per query)", "ms_per_launch": ms_short, "timed_launches": timed_ms.last[0],
                                   "queries_per_s": nq / (ms_short * 1e-3),
                                   "hbm_gbs_algorithmic": 40 * nq / (ms_short * 1e-3) / 1e9},
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
    result["timing"] = {"headline": f"{args.warmup} untimed steps, then {args.steps} timed ones, one after the other on one stream",
                        "other_workloads": f"each: untimed launches for {args.leg_warm_ms:g} ms, then timed launches for {args.leg_ms:g} ms",
                        "why": "the GPU reaches its clock under load only after some tens of milliseconds of continuous work "
                               "and drops it when idle"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
