"""Turns rocprofv3 output of `bench.py` runs into the short summaries kept under profiles/.

    python -m paper_2103_07454_amd.rocprof_summary --config 5 --bench B.json \
        --trace DIR_T [--fetch DIR_F --write DIR_W] [--valu DIR_V] [--out profiles]

DIR_T  from  rocprofv3 --kernel-trace --stats --output-format csv -d DIR_T -o cfgC -- python3 bench.py --config C ...
DIR_F  from  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR_F -o cfgC -- python3 bench.py --config C ...
DIR_W  the same with WRITE_SIZE;  DIR_V the same with SQ_INSTS_VALU (and any other SQ counters)
B.json the JSON line an un-profiled `python bench.py --config C` printed in the same session

Writes, for the configuration's workload name W:
  profiles/evg_step_kernel_trace_W.md   per-kernel calls / average / min / max
  profiles/hbm_traffic_pmc_W.md         per-kernel HBM bytes per launch (when --fetch/--write are given)
  profiles/counters_W.json              the figures bench.py prints as roofline.traffic and as the
                                        VALU instruction count, with the run they were measured on

FETCH_SIZE and WRITE_SIZE are in KiB per dispatch and are calibrated on the library's own plain
copy kernel: at iteration 0 `k_copy` copies every chunk of x into both mailboxes, so it reads
P * sum(pad4(n_l)) * 4 bytes and writes twice that; true bytes = counter * 1024 * factor.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os

from . import inputs

KIB = 1024


def short(name: str) -> str:
    return name.split("(")[0].replace("void ", "")


def one(pattern: str) -> str:
    hits = sorted(glob.glob(pattern))
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[0]


def counter_rows(directory: str, counter: str):
    """{kernel name: [value per dispatch, in dispatch order]} for one counter."""
    by = collections.defaultdict(list)
    with open(one(os.path.join(directory, "*counter_collection.csv"))) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                by[r["Kernel_Name"]].append((int(r["Dispatch_Id"]), float(r["Counter_Value"])))
    return {k: [v for _, v in sorted(rows)] for k, rows in by.items()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--bench", required=True)
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--valu")
    ap.add_argument("--steps", type=int, default=100, help="--steps of the profiled bench.py runs")
    ap.add_argument("--warmup", type=int, default=3, help="--warmup of the profiled bench.py runs")
    ap.add_argument("--valu-steps", type=int, default=20)
    ap.add_argument("--valu-warmup", type=int, default=2)
    ap.add_argument("--out", default="profiles")
    a = ap.parse_args()
    w = inputs.config(a.config)
    c = a.config
    with open(a.bench) as f:
        b = json.loads([l for l in f if l.strip().startswith("{")][-1])
    if b["config"]["workload"] != w.name:
        raise SystemExit(f"{a.bench} is a run of {b['config']['workload']}, not of {w.name}")
    elems = w.P * w.N
    bench_cmd = f"python3 <repo>/bench.py --config {c} --steps {a.steps} --warmup {a.warmup} --no-cpu-baseline"

    # ---- kernel trace -----------------------------------------------------------------
    with open(one(os.path.join(a.trace, "*kernel_stats.csv"))) as f:
        rows = [r for r in csv.DictReader(f) if "evg::" in r["Name"]]
    rf = b["roofline"]
    out = [f"# rocprofv3 kernel trace of the whole evg_step pipeline, configuration {c} ({w.name})", "",
           "Command (on the MI355X box, after `cd /tmp && export TMPDIR=/tmp`):", "",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o cfg{c} -- {bench_cmd}", "",
           f"Launches per per-step kernel = {a.warmup} warm-up + the {a.steps} timed iterations + the same {a.steps} iterations",
           "again with the phase timers on. Times in microseconds.", "",
           "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    per_step = 0.0
    for r in rows:
        out.append(f"| {short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} "
                   f"| {float(r['MaxNs']) / 1e3:.1f} | {float(r['Percentage']):.2f} |")
        if int(r["Calls"]) >= a.steps:
            per_step += float(r["AverageNs"]) / 1e6
    out += ["", f"Sum of the per-step kernels' averages: {per_step:.3f} ms per iteration.", "",
            f"The un-profiled `python bench.py --config {c}` run of the same session printed:", "",
            f"    ms_per_step {b['ms_per_step']:.3f}, value {b['value']:.4e} elements/s, k_update avg launch "
            f"{rf['avg_launch_ms']:.3f} ms (HIP events on the library's stream),"]
    if rf["bound"] == "hbm":
        out.append(f"    roofline.achieved {rf['achieved']:.0f} GB/s = {rf['frac']:.3f} of 8 TB/s on "
                   f"{rf['algorithmic_bytes_per_launch'] / 1e9:.2f} GB algorithmic bytes per launch,")
    else:
        out.append(f"    roofline (bound: alu) {rf['achieved']:.1f} of {rf['peak']:.1f} T lane-instructions/s = {rf['frac']:.3f}; "
                   f"the same launches move their algorithmic bytes at {rf['hbm_achieved_GBps']:.0f} GB/s = {rf['hbm_frac']:.3f} of 8 TB/s,")
    out.append(f"    whole step {b['step_achieved_GBps']:.0f} GB/s = {b['step_frac_of_hbm_peak']:.3f} of peak on "
               f"{b['step_algorithmic_bytes_per_element']:.2f} B/element (f_full = {b['config']['fraction_fired_full']:.3f}, "
               f"f_topk = {b['config']['fraction_fired_topk']:.3f}).")
    os.makedirs(a.out, exist_ok=True)
    with open(os.path.join(a.out, f"evg_step_kernel_trace_{w.name}.md"), "w") as f:
        f.write("\n".join(out) + "\n")

    record = {"workload": w.name, "bench_command": bench_cmd, "steps": a.steps, "warmup": a.warmup,
              "fraction_fired_topk": b["config"]["fraction_fired_topk"],
              "fraction_fired_full": b["config"]["fraction_fired_full"], "kernels": {}}

    # ---- HBM traffic --------------------------------------------------------------------
    if a.fetch and a.write and not any("k_copy" in k for k in counter_rows(a.fetch, "FETCH_SIZE")):
        # cache-resident rings that send whole tensors never launch the copy kernel, and their
        # counters would mostly show cache hits anyway
        print(f"no k_copy launch in {a.fetch}: the counters cannot be calibrated, no traffic summary is written")
        a.fetch = a.write = None
    if a.fetch and a.write:
        fetch, write = counter_rows(a.fetch, "FETCH_SIZE"), counter_rows(a.write, "WRITE_SIZE")
        npad4 = sum((int(n) + 3) // 4 * 4 for n in w.layer_numel)
        copy_read = w.P * npad4 * 4
        copy_write = 2 * copy_read
        kc = [k for k in fetch if "k_copy" in k][0]
        f_fetch = copy_read / (max(fetch[kc]) * KIB)
        f_write = copy_write / (max(write[kc]) * KIB)
        record["calibration"] = {"kernel": short(kc), "read_bytes": copy_read, "write_bytes": copy_write,
                                 "fetch_factor": f_fetch, "write_factor": f_write}
        out = [f"# HBM traffic per kernel launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE), configuration {c} ({w.name})", "",
               "Commands (two runs, one counter each; on the MI355X box after `cd /tmp && export TMPDIR=/tmp`):", "",
               f"    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d <out> -o cfg{c} -- {bench_cmd}",
               f"    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d <out> -o cfg{c} -- {bench_cmd}", "",
               f"Counters are in KiB per dispatch. Calibration on the library's plain copy kernel `k_copy` at iteration 0, where it",
               f"copies every chunk of x into both mailboxes (reads {copy_read} B, writes {copy_write} B): FETCH_SIZE factor "
               f"{f_fetch:.4f}, WRITE_SIZE factor {f_write:.4f}", "(true bytes = counter x 1024 x factor).", "",
               f"Averages over the timed and the instrumented run of the {a.steps} iterations (warm-up launches dropped), GB per launch:", "",
               "| kernel | launches | fetch GB | write GB | total GB |", "|---|---|---|---|---|"]
        for k, fv in fetch.items():
            if "evg::" not in k:
                continue
            wv = write.get(k, [0.0])
            if len(fv) >= 2 * a.steps + a.warmup:
                fv, wv = fv[a.warmup:], wv[a.warmup:]
            af = sum(fv) / len(fv) * KIB * f_fetch
            aw = sum(wv) / len(wv) * KIB * f_write
            out.append(f"| {short(k)} | {len(fv)} | {af / 1e9:.3f} | {aw / 1e9:.3f} | {(af + aw) / 1e9:.3f} |")
            record["kernels"].setdefault(short(k).replace("evg::", "").split("<")[0], {}).update(
                fetch_bytes=af, write_bytes=aw, traffic_bytes=af + aw, launches=len(fv))
        upd = record["kernels"].get("k_update")
        if upd and rf["bound"] == "hbm":
            out += ["", f"`k_update`: {upd['traffic_bytes'] / 1e9:.2f} GB per launch = {upd['traffic_bytes'] / elems:.1f} B per element, against "
                    f"{rf['algorithmic_bytes_per_launch'] / 1e9:.2f} GB algorithmic"
                    + (f" and a line-granular floor of {rf['line_granular_floor_bytes_per_launch'] / 1e9:.2f} GB "
                       f"(dense arrays + messages + write-back of every 64-byte group that holds a sent entry)."
                       if "line_granular_floor_bytes_per_launch" in rf else ".")]
        with open(os.path.join(a.out, f"hbm_traffic_pmc_{w.name}.md"), "w") as f:
            f.write("\n".join(out) + "\n")

    # ---- SQ counters ------------------------------------------------------------------
    if a.valu:
        names = ["SQ_WAVES", "SQ_BUSY_CYCLES", "SQ_WAIT_INST_ANY", "SQ_ACTIVE_INST_VALU", "SQ_ACTIVE_INST_VMEM",
                 "SQ_ACTIVE_INST_LDS", "SQ_LDS_BANK_CONFLICT", "SQ_INSTS_VALU"]
        data = {n: counter_rows(a.valu, n) for n in names}
        drop = a.valu_warmup + 2                      # warm-up launches and the all-fire iterations 0, 1

        def avg(name, kernel):
            v = data[name].get(kernel, [])
            v = v[drop:] if len(v) > drop else v
            return sum(v) / len(v) if v else float("nan")

        sq_cmd = (f"rocprofv3 --pmc {' '.join(names)} --kernel-trace --output-format csv -d <out> -o cfg{c} -- "
                  f"python3 <repo>/bench.py --config {c} --steps {a.valu_steps} --warmup {a.valu_warmup} "
                  f"--no-cpu-baseline --no-phase-timers")
        out = [f"# SQ counters of the per-step kernels (rocprofv3 --pmc), configuration {c} ({w.name})", "",
               "Command (on the MI355X box, after `cd /tmp && export TMPDIR=/tmp`):", "", f"    {sq_cmd}", "",
               f"Averages per launch over iterations 2..{a.valu_steps - 1} (the all-fire iterations 0 and 1 dropped). The counters are sums",
               "over the chip's shader engines; they are given as ratios to SQ_BUSY_CYCLES of the same launch, which makes",
               "launches of different length comparable but is not a utilisation in percent (the counters' units differ).", "",
               "| kernel | waves | VALU-active / busy | VMEM-active / busy | LDS-active / busy | wait-any / busy | LDS bank conflict / busy | VALU wave-instructions |",
               "|---|---|---|---|---|---|---|---|"]
        for k in data["SQ_WAVES"]:
            if "evg::" not in k or avg("SQ_WAVES", k) < 1000:
                continue
            busy = avg("SQ_BUSY_CYCLES", k)
            out.append(f"| {short(k)} | {avg('SQ_WAVES', k):.0f} | {avg('SQ_ACTIVE_INST_VALU', k) / busy:.2f} | "
                       f"{avg('SQ_ACTIVE_INST_VMEM', k) / busy:.2f} | {avg('SQ_ACTIVE_INST_LDS', k) / busy:.2f} | "
                       f"{avg('SQ_WAIT_INST_ANY', k) / busy:.1f} | {avg('SQ_LDS_BANK_CONFLICT', k) / busy:.3f} | "
                       f"{avg('SQ_INSTS_VALU', k):.3g} |")
        ku = [k for k in data["SQ_INSTS_VALU"] if "k_update" in k]
        if ku:
            per_launch = avg("SQ_INSTS_VALU", ku[0])
            per_elem = per_launch * 64 / elems
            alu_ms = per_launch * 4 / 1024 / 2.4e9 * 1e3
            record["kernels"].setdefault("k_update", {}).update(
                valu_wave_instructions_per_launch=per_launch, valu_instructions_per_element=per_elem, valu_command=sq_cmd)
            out += ["", "A 64-lane wavefront occupies its SIMD for at least 4 cycles per vector instruction, and the chip has 256 CUs x 4 SIMDs",
                    f"at 2.4 GHz: the update pass executes {per_launch:.3g} wave-instructions per launch = {per_elem:.0f} per element, which the vector",
                    f"ALUs alone need {alu_ms:.2f} ms for (quarter-rate instructions such as 32-bit integer multiplies take longer), against "
                    f"{rf['avg_launch_ms']:.2f} ms per launch."]
        with open(os.path.join(a.out, f"sq_counters_{w.name}.md"), "w") as f:
            f.write("\n".join(out) + "\n")
    if record["kernels"]:                  # nothing to record from a kernel trace alone
        with open(os.path.join(a.out, f"counters_{w.name}.json"), "w") as f:
            json.dump(record, f, indent=1, sort_keys=True)
            f.write("\n")
    print(f"wrote summaries of {w.name} under {a.out}/")


if __name__ == "__main__":
    main()
