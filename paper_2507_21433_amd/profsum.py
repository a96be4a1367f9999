"""Profiler passes over ``bench.py`` and the short summaries kept under ``profiles/``.

    python3 -m paper_2507_21433_amd.profsum collect --workload 4 --passes A B C D E
    python3 -m paper_2507_21433_amd.profsum summarise --workload 4 --out profiles
    python3 -m paper_2507_21433_amd.profsum trace --out profiles
    python3 -m paper_2507_21433_amd.profsum table --json bench.json --out profiles

``collect`` runs, once per pass, ``rocprofv3 --pmc <counters of the pass> --kernel-trace --output-format csv
-d <dir>/pmc_w<N>_<pass> -- python3 bench.py --step-only 1 --workload N --steps 3 --warmup 1`` (one pass per run: the
profiler does not split a counter list over several runs of the kernels) and keeps, of the CSV files, only the rows of
this library's kernels and of the device copies.  ``summarise`` turns them into ``profiles/match_tile_kernel_<workload>.md``
(mean counter values per launch of the tile kernel, the figures derived from them, the commands) and enters the
workload's HBM traffic into ``profiles/hbm_traffic.json``, which ``bench.py`` reads for ``roofline.traffic``.

``trace`` runs ``rocprofv3 --kernel-trace --stats -- python3 bench.py ...`` on the timed step alone and on the headline
workload with its side measurements, and writes the per-kernel times of this library's kernels to
``profiles/bench_kernel_trace.md``; ``table`` condenses the JSON line of a default
``bench.py`` run into ``profiles/bench_all_workloads.md``.

FETCH_SIZE and WRITE_SIZE are scaled by what the same counters read, in the same run, for the 1 GiB device-to-device
copy that ``bench.py`` issues before anything else (the first device copy of the run): bytes = counter x (2^30 /
counter of that copy).  What the counters see is what leaves the L2 for the fabric: reads that the memory-side cache
serves are in it.
"""
import argparse
import csv
import glob
import hashlib
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KERNEL_SOURCES = ("paper_2507_21433_amd/csrc/rc_match.hip", "paper_2507_21433_amd/csrc/rc_common.hpp")
TILE_KERNEL = "match_tile_kernel"
COPY_KERNEL = "copyBuffer"
CAL_BYTES = 1 << 30

# per pass at most 8 SQ, 4 TCC (FETCH_SIZE takes 3, WRITE_SIZE 2), 4 TCP, 2 TA and 2 GRBM counters
PASSES = {
    "A": "SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_VALU_MFMA_BUSY_CYCLES SQ_WAIT_INST_LDS SQ_ACTIVE_INST_LDS "
         "SQ_LDS_BANK_CONFLICT SQ_INST_CYCLES_VMEM_RD GRBM_GUI_ACTIVE",
    "B": "SQ_LDS_IDX_ACTIVE SQ_LDS_ADDR_CONFLICT SQ_LDS_DATA_FIFO_FULL SQ_ACTIVE_INST_ANY SQ_WAIT_ANY SQ_INSTS_VMEM_RD "
         "SQ_INSTS_LDS SQ_INSTS_MFMA GRBM_GUI_ACTIVE",
    "C": "TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum TCC_EA0_RDREQ_sum TCP_TCC_READ_REQ_LATENCY_sum TCP_TCC_READ_REQ_sum "
         "TCP_PENDING_STALL_CYCLES_sum TCP_TCR_TCP_STALL_CYCLES_sum TA_BUSY_avr TA_ADDR_STALLED_BY_TC_CYCLES_sum "
         "GRBM_GUI_ACTIVE",
    "D": "FETCH_SIZE",
    "E": "WRITE_SIZE",
}
N_SIMD = 256 * 4          # 256 compute units x 4 SIMDs
N_XCD = 8


def bench_args(workload):
    return ["python3", "bench.py", "--step-only", "1", "--workload", str(workload), "--steps", "3", "--warmup", "1"]


def pass_command(workload, name, outdir):
    return ["rocprofv3", "--pmc"] + PASSES[name].split() + ["--kernel-trace", "--output-format", "csv", "-d",
                                                           os.path.join(outdir, f"pmc_w{workload}_{name}"), "--"] + bench_args(workload)


def kernel_source_hash():
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def collect(args):
    env = dict(os.environ, TMPDIR="/tmp")
    for name in args.passes:
        d = os.path.join(args.dir, f"pmc_w{args.workload}_{name}")
        subprocess.call(["rm", "-rf", d])
        cmd = ["timeout", "-s", "KILL", str(args.timeout)] + pass_command(args.workload, name, args.dir)
        print("[profsum] " + " ".join(cmd), flush=True)
        with open(d + ".json", "w") as out, open(d + ".err", "w") as err:
            rc = subprocess.call(cmd, cwd=ROOT, env=env, stdout=out, stderr=err)
        if rc != 0:
            print(f"[profsum] pass {name} failed with status {rc}", flush=True)
            sys.stdout.write(open(d + ".err").read()[-2000:])
            return rc
        for f in glob.glob(os.path.join(d, "*", "*_counter_collection.csv")) + glob.glob(os.path.join(d, "*", "*_kernel_trace.csv")):
            with open(f) as src:
                lines = src.readlines()
            keep = [lines[0]] + [ln for ln in lines[1:] if "rc::" in ln or COPY_KERNEL in ln]
            with open(f, "w") as dst:
                dst.writelines(keep)
        print(f"[profsum] pass {name} done", flush=True)
    return 0


def read_pass(d):
    """{kernel kind: {counter: [value per dispatch]}}, {kernel kind: [duration ns per dispatch]}, bench JSON or None."""
    files = sorted(glob.glob(os.path.join(d, "*", "*_counter_collection.csv")), key=os.path.getmtime, reverse=True)
    if not files:
        return None
    vals, durs = {}, {}
    for r in csv.DictReader(open(files[0])):
        k = r["Kernel_Name"]
        kind = "tile" if TILE_KERNEL in k else ("copy" if COPY_KERNEL in k else None)
        if kind is None:
            continue
        vals.setdefault(kind, {}).setdefault(r["Counter_Name"], {})[r["Dispatch_Id"]] = float(r["Counter_Value"])
        durs.setdefault(kind, {})[r["Dispatch_Id"]] = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    bench = None
    try:
        with open(d + ".json") as f:
            for ln in f:
                if ln.startswith("{"):
                    bench = json.loads(ln)
    except (OSError, ValueError):
        pass
    return vals, durs, bench


def mean(xs):
    xs = list(xs)
    return sum(xs) / len(xs) if xs else float("nan")


def summarise(args):
    wl = args.workload
    found = {}
    for name in PASSES:
        got = read_pass(os.path.join(args.dir, f"pmc_w{wl}_{name}"))
        if got and "tile" in got[0]:
            found[name] = got
    if not found:
        print(f"[profsum] no passes of workload {wl} under {args.dir}", file=sys.stderr)
        return 1
    bench = next((g[2] for g in found.values() if g[2]), None)
    wname = bench["config"]["workload"] if bench else f"cfg{wl}"
    roof = bench["roofline"] if bench else {}
    flop, alg_bytes = roof.get("algorithmic_flop"), roof.get("algorithmic_bytes")

    c = {}         # counter -> mean per launch of the tile kernel
    dur_ns = {}    # pass -> mean launch duration under that pass
    for name, (vals, durs, _) in found.items():
        for ctr, per in vals["tile"].items():
            c.setdefault(ctr, []).append(mean(per.values()))
        dur_ns[name] = mean(durs["tile"].values())
    launches = len(next(iter(found.values()))[1]["tile"])
    c = {k: mean(v) for k, v in c.items()}
    lines = [f"# match_tile_kernel on {wname}: hardware counters", ""]
    lines += ["Mean per launch of `rc::match_tile_kernel` (the kernel inside `rc_match_blocks`) over the "
              f"{launches} launches of one `bench.py --step-only 1` run per pass; one `rocprofv3 --pmc` run per pass, "
              "made with `python3 -m paper_2507_21433_amd.profsum collect` and condensed with its `summarise`.", ""]
    lines += ["Commands (from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", "", "```"]
    for name in found:
        lines.append(" ".join(pass_command(wl, name, args.dir)))
    lines += ["```", ""]
    if bench:
        lines += [f"`bench.py`'s own event timing of the launch during pass {next(iter(found))} (counters being collected): "
                  f"{roof.get('tflops', float('nan')):.0f} TFLOP/s = {roof.get('mfma_frac', float('nan')):.4f} of the "
                  f"2500 TFLOP/s MFMA peak, {roof.get('gb_per_s', float('nan')):.0f} GB/s of KV = "
                  f"{roof.get('hbm_frac', float('nan')):.4f} of the 8000 GB/s HBM peak "
                  f"({roof.get('flop_per_byte', float('nan')):.0f} FLOP per byte; the ridge is at "
                  f"{roof.get('ridge_flop_per_byte', float('nan')):.0f}).", ""]
    lines += ["| pass | launch under the profiler, ms |", "|---|---|"]
    lines += [f"| {n} | {dur_ns[n] / 1e6:.3f} |" for n in found]
    lines += ["", "| counter | mean per launch |", "|---|---|"]
    lines += [f"| {k} | {v:.6g} |" for k, v in sorted(c.items())]

    d = {}
    if "GRBM_GUI_ACTIVE" in c:
        any_pass = next(n for n in found if "GRBM_GUI_ACTIVE" in found[n][0]["tile"])
        gui = mean(found[any_pass][0]["tile"]["GRBM_GUI_ACTIVE"].values())
        d["clock_ghz"] = gui / N_XCD / dur_ns[any_pass]
        d["cycles_per_launch"] = gui / N_XCD
    if "SQ_VALU_MFMA_BUSY_CYCLES" in c and "A" in found:
        gui = mean(found["A"][0]["tile"]["GRBM_GUI_ACTIVE"].values())
        d["mfma_busy"] = c["SQ_VALU_MFMA_BUSY_CYCLES"] / (gui / N_XCD * N_SIMD)
        if flop:
            d["mfma_busy_cycles_expected"] = flop / 32768.0 * 32
    lines += ["", "## Derived", ""]
    if "clock_ghz" in d:
        lines.append(f"- Clock the chip granted: GRBM_GUI_ACTIVE / 8 XCDs / launch time = **{d['clock_ghz']:.3f} GHz** "
                     "(the peak figure assumes 2.4 GHz).")
    if "mfma_busy" in d:
        ceiling = 2500.0 * d["clock_ghz"] / 2.4
        lines.append(f"- MFMA pipes busy: SQ_VALU_MFMA_BUSY_CYCLES / (cycles x 1024 SIMDs) = **{100 * d['mfma_busy']:.1f} %** "
                     f"of the granted cycles.  (An MFMA of 32x32x16 holds its pipe 32 cycles: "
                     f"{d.get('mfma_busy_cycles_expected', float('nan')):.4g} busy cycles follow from the FLOP count, "
                     f"{c['SQ_VALU_MFMA_BUSY_CYCLES']:.4g} were counted.)")
        lines.append(f"- Ceiling at the granted clock (every pipe busy every cycle): 2500 x {d['clock_ghz']:.3f} / 2.4 = "
                     f"**{ceiling:.0f} TFLOP/s**; under the profiler the kernel reaches {100 * d['mfma_busy']:.1f} % of it.")
    if "SQ_WAVE_CYCLES" in c and "SQ_WAIT_INST_ANY" in c:
        lines.append(f"- Waves waiting on any counter (s_waitcnt): SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES = "
                     f"{100 * c['SQ_WAIT_INST_ANY'] / c['SQ_WAVE_CYCLES']:.1f} % of wave cycles; on LDS alone "
                     f"{100 * c.get('SQ_WAIT_INST_LDS', float('nan')) / c['SQ_WAVE_CYCLES']:.1f} %.")
    if "SQ_LDS_BANK_CONFLICT" in c and "SQ_ACTIVE_INST_LDS" in c:
        lines.append(f"- LDS: SQ_LDS_BANK_CONFLICT / SQ_ACTIVE_INST_LDS = {c['SQ_LDS_BANK_CONFLICT'] / c['SQ_ACTIVE_INST_LDS']:.2f} "
                     "conflict cycles per active LDS-instruction cycle (a 64-lane ds_read_b128 takes several passes by "
                     "construction; the counter calls the extra passes conflicts).")
    if "SQ_LDS_IDX_ACTIVE" in c and "SQ_LDS_ADDR_CONFLICT" in c:
        lines.append(f"- LDS address conflicts: {100 * c['SQ_LDS_ADDR_CONFLICT'] / c['SQ_LDS_IDX_ACTIVE']:.3f} % of the cycles the "
                     f"LDS index unit is active; data FIFO full {c.get('SQ_LDS_DATA_FIFO_FULL', float('nan')):.3g} cycles.")
    if "SQ_INSTS_MFMA" in c:
        lines.append(f"- Instruction mix per launch: {c['SQ_INSTS_MFMA']:.4g} MFMA, {c.get('SQ_INSTS_LDS', float('nan')):.4g} LDS, "
                     f"{c.get('SQ_INSTS_VMEM_RD', float('nan')):.4g} vector-memory reads"
                     + (f" ({flop / 32768.0:.4g} MFMA follow from the FLOP count)." if flop else "."))
    if "TCC_HIT_sum" in c and "TCC_MISS_sum" in c:
        lines.append(f"- L2: {100 * c['TCC_HIT_sum'] / (c['TCC_HIT_sum'] + c['TCC_MISS_sum']):.1f} % of {c.get('TCC_REQ_sum', float('nan')):.4g} "
                     f"requests hit; {c.get('TCC_EA0_RDREQ_sum', float('nan')):.4g} read requests leave the L2 for the fabric.")
    if "TCP_TCC_READ_REQ_LATENCY_sum" in c and "TCP_TCC_READ_REQ_sum" in c:
        lines.append(f"- Mean latency of an L1-to-L2 read request: {c['TCP_TCC_READ_REQ_LATENCY_sum'] / c['TCP_TCC_READ_REQ_sum']:.0f} cycles; "
                     f"L1 pending-request stalls {c.get('TCP_PENDING_STALL_CYCLES_sum', float('nan')):.4g} cycles summed over the L1s; "
                     f"texture-addresser stalled by the cache {c.get('TA_ADDR_STALLED_BY_TC_CYCLES_sum', float('nan')):.4g} cycles.")

    traffic = None
    if "D" in found and "E" in found:
        f_tile, w_tile = c["FETCH_SIZE"], c["WRITE_SIZE"]
        # the calibration copy is the first device copy of the run (the inputs are drawn after it)
        first = lambda per: per[min(per, key=int)]
        f_copy = first(found["D"][0]["copy"]["FETCH_SIZE"])
        w_copy = first(found["E"][0]["copy"]["WRITE_SIZE"])
        f_scale, w_scale = CAL_BYTES / f_copy, CAL_BYTES / w_copy
        traffic = {"fetch_counter": f_tile, "write_counter": w_tile, "copy_fetch_counter": f_copy, "copy_write_counter": w_copy,
                   "fetch_bytes": f_tile * f_scale, "write_bytes": w_tile * w_scale,
                   "hbm_bytes_per_launch": f_tile * f_scale + w_tile * w_scale, "algorithmic_bytes": alg_bytes,
                   "commands": [" ".join(pass_command(wl, n, args.dir)) for n in ("D", "E")]}
        lines.append(f"- HBM traffic: FETCH_SIZE {f_tile:.6g} and WRITE_SIZE {w_tile:.6g} per launch; the 1 GiB copy of the same runs "
                     f"reads {f_copy:.6g} and writes {w_copy:.6g}, so one count is {f_scale:.1f} bytes fetched, {w_scale:.1f} bytes "
                     f"written: **{traffic['fetch_bytes'] / 1e9:.2f} GB read + {traffic['write_bytes'] / 1e9:.3f} GB written per launch**"
                     + (f", {traffic['hbm_bytes_per_launch'] / alg_bytes:.2f} x the {alg_bytes / 1e9:.2f} GB of KV that the launch has to read once."
                        if alg_bytes else "."))
    os.makedirs(args.out, exist_ok=True)
    path = os.path.join(args.out, f"match_tile_kernel_{wname}.md")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(f"[profsum] wrote {path}")

    if traffic:
        tpath = os.path.join(args.out, "hbm_traffic.json")
        sha = kernel_source_hash()
        table = {"kernel_source_sha256": sha, "kernel_sources": list(KERNEL_SOURCES), "workloads": {}}
        try:
            with open(tpath) as f:
                old = json.load(f)
            if old.get("kernel_source_sha256") == sha:
                table = old
        except (OSError, ValueError):
            pass
        table["workloads"][wname] = traffic
        with open(tpath, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
            f.write("\n")
        print(f"[profsum] entered {wname} into {tpath}")
    return 0


TRACE_RUNS = {
    # the timed step of the headline workload and nothing else: every launch of the tile kernel is a launch of that step
    "step": ["--step-only", "1", "--steps", "10", "--warmup", "2"],
    # the headline workload with everything bench.py times beside the step
    "headline": ["--configs", "none"],
    # the default run: all five workloads (instantiations of the tile kernel are shared between workloads and with
    # the one-layer-per-call side measurement, so their averages mix shapes)
    "default": [],
}


def trace_command(outdir, run):
    return ["rocprofv3", "--kernel-trace", "--stats", "--output-format", "csv", "-d", os.path.join(outdir, f"trace_{run}"), "--",
            "python3", "bench.py"] + TRACE_RUNS[run]


def trace(args):
    """Per-kernel times of bench.py runs: collect (unless --no-run) and write profiles/bench_kernel_trace.md."""
    lines = ["# Kernel times of bench.py runs (rocprofv3 --kernel-trace --stats)", "",
             "Kernels of this library (`rc::`) and the device copies; the rest of a run is torch's input generation.  "
             "Commands from the repository root, after `cd /tmp && export TMPDIR=/tmp`."]
    for run in args.runs:
        d = os.path.join(args.dir, f"trace_{run}")
        if not args.no_run:
            subprocess.call(["rm", "-rf", d])
            cmd = ["timeout", "-s", "KILL", str(args.timeout)] + trace_command(args.dir, run)
            print("[profsum] " + " ".join(cmd), flush=True)
            with open(d + ".json", "w") as out, open(d + ".err", "w") as err:
                rc = subprocess.call(cmd, cwd=ROOT, env=dict(os.environ, TMPDIR="/tmp"), stdout=out, stderr=err)
            if rc != 0:
                print(f"[profsum] trace failed with status {rc}", flush=True)
                sys.stdout.write(open(d + ".err").read()[-2000:])
                return rc
            for f in glob.glob(os.path.join(d, "*", "*_kernel_trace.csv")):
                os.remove(f)     # per-dispatch rows of every torch kernel: large, and the stats file has what is kept
        files = sorted(glob.glob(os.path.join(d, "*", "*_kernel_stats.csv")), key=os.path.getmtime, reverse=True)
        if not files:
            print(f"[profsum] no kernel stats under {d}", file=sys.stderr)
            return 1
        rows = list(csv.DictReader(open(files[0])))
        bench = None
        try:
            with open(d + ".json") as f:
                for ln in f:
                    if ln.startswith("{"):
                        bench = json.loads(ln)
        except (OSError, ValueError):
            pass
        lines += ["", f"## `bench.py {' '.join(TRACE_RUNS[run])}`", "", "```", " ".join(trace_command(args.dir, run)), "```", "",
                  "| kernel | calls | average, ms | total, ms | share of GPU time |", "|---|---|---|---|---|"]
        for r in rows:
            name = r["Name"]
            if "rc::" not in name and COPY_KERNEL not in name:
                continue
            short = name.replace("(anonymous namespace)::", "")
            short = short[:short.index("(")] if "(" in short else short
            lines.append(f"| `{short}` | {r['Calls']} | {float(r['AverageNs']) / 1e6:.4f} | {float(r['TotalDurationNs']) / 1e6:.2f} | "
                         f"{float(r['Percentage']):.2f} % |")
        if run != "step":
            lines += ["", "In this run the tile kernel instantiation of the headline workload is launched by the timed step and "
                      "by the one-layer-per-call side measurement (a launch of one layer's tiles, 1/64 of the work), and the "
                      "layer-mean instantiation by its own measurement and by the steady-state loop: their averages mix "
                      "shapes.  The run of the timed step alone, above, is the one whose average is a launch of the step."]
        if bench and run == "step":
            k = bench["kernels"]["rc_match_blocks"]
            flop = bench["roofline"]["algorithmic_flop"]
            tile = next((r for r in rows if TILE_KERNEL in r["Name"]), None)
            lines += ["", f"`bench.py` timed `rc_match_blocks` of {bench['config']['workload']} with events at **{k['ms']:.3f} ms** per call in "
                      "this run (the tile kernel, the clearing of its schedule words and the selection kernel after it)"
                      + (f"; the profiler's average for the tile kernel is **{float(tile['AverageNs']) / 1e6:.3f} ms** over {tile['Calls']} "
                         f"launches, i.e. {flop / float(tile['AverageNs']) / 1e3:.0f} TFLOP/s." if tile else ".")]
    os.makedirs(args.out, exist_ok=True)
    path = os.path.join(args.out, "bench_kernel_trace.md")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(f"[profsum] wrote {path}")
    return 0


def table(args):
    """profiles/bench_all_workloads.md from the JSON line of one default bench.py run."""
    bench = None
    with open(args.json) as f:
        for ln in f:
            if ln.startswith("{"):
                bench = json.loads(ln)
    if not bench:
        print(f"[profsum] no JSON line in {args.json}", file=sys.stderr)
        return 1
    lines = ["# `bench.py` on the five workloads (one MI355X, one run)", "",
             "Command (from the repository root): `python3 bench.py` (2 warm-up steps, 10 timed steps per workload; the "
             "headline is cfg4).  A step = `rc_block_norms`(queries) + `rc_match_blocks` + `rc_remap_block_table` on all "
             "layers with the pool norms cached; pairs/s = L x P x Q / step time.  The roofline columns are the tile kernel "
             "inside `rc_match_blocks`, timed with events inside the run; `traffic` is what leaves the L2 per launch "
             "(`profiles/hbm_traffic.json`) over the KV bytes the launch has to read once.", "",
             "| workload | L x P x Q, dtype, mode | step, ms | pairs/s | binding roof | of that roof | TFLOP/s (of 2500) | KV GB/s (of 8000) "
             "| of the pure-MFMA rate this box sustains | traffic / algorithmic | query norms GB/s | remap, us | CPU oracle pairs/s (threads) |",
             "|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for name, b in bench["configs"].items():
        c, r, k = b["config"], b["roofline"], b["kernels"]
        cpu = b.get("cpu_baseline") or {}
        ceil = r.get("ceiling", {})
        tr = r.get("traffic")
        lines.append(
            f"| {name} | {c['layers']} x {c['pool_blocks_per_layer']} x {c['query_blocks_per_layer']}, {b['dtype']}, {c['mode']} "
            f"| {b['ms_per_step']:.3f} | {b['value']:.3g} | {r['bound']} | {r['frac']:.3f} | {r['tflops']:.0f} ({r['mfma_frac']:.3f}) "
            f"| {r['gb_per_s']:.0f} ({r['hbm_frac']:.3f}) | {ceil.get('frac_of_ceiling', float('nan')):.3f} "
            f"| {(tr / r['algorithmic_bytes']) if tr else float('nan'):.2f} | {k['rc_block_norms(queries)']['gb_per_s']:.0f} "
            f"| {k['rc_remap_block_table']['ms'] * 1e3:.0f} | {cpu.get('value', float('nan')):.3g} ({cpu.get('cores', '-')}) |")
    ceil = bench["roofline"].get("ceiling")
    if ceil:
        lines += ["", f"Pure-MFMA rate of this box in the same run: {ceil['pure_mfma_tflops']:.0f} TFLOP/s "
                  f"({ceil['what']}), i.e. a clock of {ceil['implied_clock_ghz']:.2f} GHz under matrix load."]
    lines += ["", f"Entry points timed beside the step on {bench['config']['workload']} (`kernels` of the same JSON line):", "",
              "| entry point | ms | figures |", "|---|---|---|"]
    for name, k in bench["kernels"].items():
        rest = ", ".join(f"{a} {b:.4g}" if isinstance(b, float) else f"{a} {b}" for a, b in k.items() if a not in ("ms", "sweep"))
        lines.append(f"| `{name}` | {k['ms']:.4f} | {rest} |")
    sweep = bench["kernels"]["rc_remap_block_table"].get("sweep")
    if sweep:
        lines += ["", "`rc_remap_block_table` on the table shape of cfg4 at growing layer counts, beside a device copy of the same bytes:", "",
                  "| layers | bytes | remap, ms | GB/s (of 8000) | copy, ms | remap rate / copy rate |", "|---|---|---|---|---|---|"]
        for e in sweep:
            lines.append(f"| {e['layers']} | {e['bytes']:.4g} | {e['ms']:.4f} | {e['gb_per_s']:.0f} ({e['hbm_frac']:.3f}) | "
                         f"{e['copy_same_bytes_ms']:.4f} | {e['frac_of_copy']:.3f} |")
    st = bench.get("streaming")
    if st:
        lines += ["", f"Steady-state loop ({st['what']}), pool {st['pool']}: {st['ms_per_step']:.2f} ms per step, "
                  f"{st['pairs_per_s']:.3g} pairs/s; per step {st['shared_per_step']} blocks shared, {st['evicted_per_step']} evicted, "
                  f"{st['admitted_per_step']} admitted."]
    os.makedirs(args.out, exist_ok=True)
    path = os.path.join(args.out, "bench_all_workloads.md")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(f"[profsum] wrote {path}")
    return 0


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("collect")
    a.add_argument("--workload", type=int, required=True)
    a.add_argument("--passes", nargs="+", default=list(PASSES), choices=list(PASSES))
    a.add_argument("--dir", default="prof_raw", help="directory of the raw profiler output")
    a.add_argument("--timeout", type=int, default=240, help="seconds per pass")
    b = sub.add_parser("summarise")
    b.add_argument("--workload", type=int, required=True)
    b.add_argument("--dir", default="prof_raw", help="directory of the raw profiler output")
    b.add_argument("--out", default="profiles")
    t = sub.add_parser("trace")
    t.add_argument("--runs", nargs="+", default=list(TRACE_RUNS), choices=list(TRACE_RUNS))
    t.add_argument("--dir", default="prof_raw", help="directory of the raw profiler output")
    t.add_argument("--out", default="profiles")
    t.add_argument("--timeout", type=int, default=600)
    t.add_argument("--no-run", action="store_true", help="summarise what an earlier run left under --dir")
    u = sub.add_parser("table")
    u.add_argument("--json", required=True, help="file holding the JSON line of a default bench.py run")
    u.add_argument("--out", default="profiles")
    args = ap.parse_args()
    sys.exit({"collect": collect, "summarise": summarise, "trace": trace, "table": table}[args.cmd](args))


if __name__ == "__main__":
    main()
