"""Profiler passes over ``bench.py`` and the short summaries kept under ``profiles/``.

    python3 -m paper_2507_21433_amd.profsum collect --workload 4 --passes A B C D E --dir gpurun_out
    python3 -m paper_2507_21433_amd.profsum summarise --workload 4 --dir gpurun_out --out profiles

``collect`` runs, once per pass, ``rocprofv3 --pmc <counters of the pass> --kernel-trace --output-format csv
-d <dir>/pmc_w<N>_<pass> -- python3 bench.py --step-only 1 --workload N --steps 3 --warmup 1`` (one pass per run: the
profiler does not split a counter list over several runs of the kernels) and keeps, of the CSV files, only the rows of
this library's kernels and of the device copies.  ``summarise`` turns them into ``profiles/match_tile_kernel_<workload>.md``
(mean counter values per launch of the tile kernel, the figures derived from them, the commands) and enters the
workload's HBM traffic into ``profiles/hbm_traffic.json``, which ``bench.py`` reads for ``roofline.traffic``.

FETCH_SIZE and WRITE_SIZE are scaled by what the same counters read, in the same run, for the 1 GiB device-to-device
copy that ``bench.py`` issues before anything else (the largest copy of the run): bytes = counter x (2^30 / counter of
that copy).
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
    files = glob.glob(os.path.join(d, "*", "*_counter_collection.csv"))
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
        lines.append(" ".join(pass_command(wl, name, "gpurun_out")))
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
        f_copy = max(found["D"][0]["copy"]["FETCH_SIZE"].values())
        w_copy = max(found["E"][0]["copy"]["WRITE_SIZE"].values())
        f_scale, w_scale = CAL_BYTES / f_copy, CAL_BYTES / w_copy
        traffic = {"fetch_counter": f_tile, "write_counter": w_tile, "copy_fetch_counter": f_copy, "copy_write_counter": w_copy,
                   "fetch_bytes": f_tile * f_scale, "write_bytes": w_tile * w_scale,
                   "hbm_bytes_per_launch": f_tile * f_scale + w_tile * w_scale, "algorithmic_bytes": alg_bytes,
                   "commands": [" ".join(pass_command(wl, n, "gpurun_out")) for n in ("D", "E")]}
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


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("collect")
    a.add_argument("--workload", type=int, required=True)
    a.add_argument("--passes", nargs="+", default=list(PASSES), choices=list(PASSES))
    a.add_argument("--dir", default="gpurun_out")
    a.add_argument("--timeout", type=int, default=240, help="seconds per pass")
    b = sub.add_parser("summarise")
    b.add_argument("--workload", type=int, required=True)
    b.add_argument("--dir", default="gpurun_out")
    b.add_argument("--out", default="profiles")
    args = ap.parse_args()
    sys.exit(collect(args) if args.cmd == "collect" else summarise(args))


if __name__ == "__main__":
    main()
