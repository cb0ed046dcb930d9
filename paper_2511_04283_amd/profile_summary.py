"""Turns the rocprofv3 output of profiled bench.py runs into the short summaries kept under profiles/.

    python -m paper_2511_04283_amd.profile_summary --config 3 --name cfg3_500k_sh3_1600x1064 \
        --stats DIR --fetch DIR --write DIR --sq DIR --bench bench_line.json --out profiles

DIRs are the `-d` folders of four rocprofv3 runs of the same bench.py command (kernel trace with --stats;
--pmc FETCH_SIZE; --pmc WRITE_SIZE; --pmc with the SQ counters below); the commands are written into the summary.
Outputs: profiles/<name>.md (per kernel: calls, average duration, HBM bytes, GB/s, vector-instruction and lane
utilisation; per kernel group: algorithmic work, achieved rate and fraction of the roofline) and
profiles/traffic_cfg<N>.json (HBM bytes per launch of every kernel group, with a digest of the kernel sources they were
measured on, which bench.py compares with the sources it runs).

Counter scaling: on this chip FETCH_SIZE reads half the bytes a plain copy of known size fetches and WRITE_SIZE reads
them exactly; both are checked in every run against the 256 MiB device copy that `bench.py --calibrate-copy` makes
(`__amd_rocclr_copyBuffer`) and the factors found there are the ones applied.
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import re
import sys
from collections import defaultdict

CLOCK_GHZ = 2.4
SIMDS = 256 * 4
SQ_COUNTERS = "SQ_WAVES SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_ACTIVE_INST_VALU SQ_THREAD_CYCLES_VALU SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE"
# kernel-name prefixes of every timing group of bench.py (`kernels_ms`), for the default step
GROUPS = {
    "preprocess": ["k_preprocess<"],
    "emit_pairs": ["k_tile_pairs<false, false>", "k_tile_pairs<true, false>", "k_tile_sum", "k_tile_scan"],
    "order_pairs": ["k_tile_pairs<false, true>", "k_tile_pairs<true, true>", "k_tile_sort<"],
    "render_fwd": ["k_render_fwd<true, true>"],
    "l1_grad": ["k_fold_tile_stats"],
    "render_bwd": ["k_render_bwd<false,", "k_render_bwd_splat<false,"],
    "preprocess_bwd": ["k_preprocess_bwd<"],
    "error_mask": ["k_err_mask_stats"],
    "score": ["k_score_bits<true>"],   # (the mask is made inside the count pass: fs_mask_score_fused)
}


def short(name: str) -> str:
    n = re.sub(r"\(anonymous namespace\)::", "", name)
    n = re.sub(r"\(.*", "", n).replace("void ", "").replace("fs::", "")
    return n[:48]


def one_csv(folder: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(folder, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit(f"no *{suffix} under {folder}")
    return hits[0]


def counters(folder: str):
    """{kernel: {counter: [values per dispatch]}}, {kernel: [durations ns per dispatch]}"""
    vals = defaultdict(lambda: defaultdict(list))
    durs = defaultdict(dict)
    for r in csv.DictReader(open(one_csv(folder, "counter_collection.csv"))):
        k = short(r["Kernel_Name"])
        vals[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
        durs[k][r["Dispatch_Id"]] = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    return vals, {k: list(d.values()) for k, d in durs.items()}


def mean(v):
    return sum(v) / len(v) if v else 0.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True)
    ap.add_argument("--name", required=True)
    ap.add_argument("--stats", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--sq")
    ap.add_argument("--bench", required=True, help="file with the JSON line bench.py printed in the --stats run")
    ap.add_argument("--bench-args", default="", help="bench.py arguments of the profiled runs besides --config (for the text)")
    ap.add_argument("--no-traffic", action="store_true",
                    help="write no traffic_cfg<N>.json (for runs of a variant, whose traffic bench.py must not pick up)")
    ap.add_argument("--out", default="profiles")
    a = ap.parse_args()

    bench = json.loads(open(a.bench).read().strip().splitlines()[-1])
    stats = {short(r["Name"]): r for r in csv.DictReader(open(one_csv(a.stats, "kernel_stats.csv")))}
    fv, fd = counters(a.fetch)
    wv, _ = counters(a.write)
    sv, sd = counters(a.sq) if a.sq else ({}, {})

    # calibration against the copy of known size
    copy = "__amd_rocclr_copyBuffer"
    known = 256 * 1024 * 1024
    f_scale = w_scale = None
    if copy in fv and fv[copy]["FETCH_SIZE"]:
        f_scale = known / (max(fv[copy]["FETCH_SIZE"]) * 1024.0)
    if copy in wv and wv[copy]["WRITE_SIZE"]:
        w_scale = known / (max(wv[copy]["WRITE_SIZE"]) * 1024.0)
    if not f_scale or not w_scale:
        raise SystemExit("no calibration copy in the counter runs: profile `bench.py --calibrate-copy`")

    rows = []
    per_kernel_bytes = {}
    for k, st in stats.items():
        if not (k.startswith("k_") or k == copy):
            continue
        fetch = mean(fv.get(k, {}).get("FETCH_SIZE", [])) * 1024.0 * f_scale
        write = mean(wv.get(k, {}).get("WRITE_SIZE", [])) * 1024.0 * w_scale
        if k == copy:
            fetch = max(fv[k]["FETCH_SIZE"]) * 1024.0 * f_scale
            write = max(wv[k]["WRITE_SIZE"]) * 1024.0 * w_scale
        avg_us = float(st["AverageNs"]) / 1e3
        row = dict(kernel=k, calls=int(st["Calls"]), avg_us=avg_us, min_us=float(st["MinNs"]) / 1e3, pct=float(st["Percentage"]),
                   fetch=fetch, write=write)
        per_kernel_bytes[k] = fetch + write
        if k in sv:
            c = {n: mean(v) for n, v in sv[k].items()}
            dur_s = mean(sd[k]) * 1e-9
            row["valu"] = c.get("SQ_INSTS_VALU", 0.0)
            row["lds"] = c.get("SQ_INSTS_LDS", 0.0)
            # a wave64 vector instruction occupies its SIMD for 4 cycles; fixed nominal clock; the dispatch's own duration
            # under the counters; not given for kernels under 30 us, whose ramp-up and tail dominate
            row["issue"] = c.get("SQ_INSTS_VALU", 0.0) * 4.0 / (dur_s * CLOCK_GHZ * 1e9 * SIMDS) if dur_s >= 30e-6 else None
            act = c.get("SQ_ACTIVE_INST_VALU", 0.0)
            row["lanes"] = c.get("SQ_THREAD_CYCLES_VALU", 0.0) / (act * 64.0) if act else None
            idx = c.get("SQ_LDS_IDX_ACTIVE", 0.0)
            row["conflict"] = c.get("SQ_LDS_BANK_CONFLICT", 0.0) / idx if idx else None
        rows.append(row)
    rows.sort(key=lambda r: -r["pct"])

    group_bytes = {}
    for grp, prefixes in GROUPS.items():
        total = sum(b for k, b in per_kernel_bytes.items() if any(k.startswith(p) for p in prefixes))
        if total > 0:
            group_bytes[grp] = int(total)

    from paper_2511_04283_amd.build import source_digest   # (the digest bench.py compares with)
    cmd = f"python3 bench.py --config {a.config} {a.bench_args}".strip() + " --steps 5 --warmup 2 --no-cpu-baseline --calibrate-copy"
    os.makedirs(a.out, exist_ok=True)
    tj = {"workload": bench["config"]["workload"], "kernel_source_digest": source_digest(),
          "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4), "bytes_per_launch": group_bytes,
          "command": f"rocprofv3 --pmc FETCH_SIZE (then WRITE_SIZE) --output-format csv -d <dir> -o p -- {cmd}",
          "summary": f"profiles/{a.name}.md"}
    suffix = "_wide_tail" if "wide_tail" in bench["config"]["workload"] else ""
    if not a.no_traffic:
        with open(os.path.join(a.out, f"traffic_cfg{a.config}{suffix}.json"), "w") as f:
            json.dump(tj, f, indent=1)
            f.write("\n")

    fmt = lambda v, p="{:.2f}": "—" if v is None else p.format(v)
    with open(os.path.join(a.out, a.name + ".md"), "w") as f:
        c = bench["config"]
        f.write(f"# rocprofv3 summary: {c['workload']} ({c['gaussians']} Gaussians, SH degree {c['sh_degree']}, "
                f"{c['image'][0]}x{c['image'][1]}, {c['pairs']} pairs)\n\n")
        f.write("Commands (MI355X box, repository root, after `python -m paper_2511_04283_amd.build`; one run each):\n\n")
        pre = "    cd /tmp && export TMPDIR=/tmp && cd $GRAFT_REPO_ROOT && rocprofv3 "
        f.write(f"{pre}--kernel-trace --stats --output-format csv -d gpurun_out/prof/stats -o p -- {cmd}\n")
        f.write(f"{pre}--pmc FETCH_SIZE --output-format csv -d gpurun_out/prof/fetch -o p -- {cmd}\n")
        f.write(f"{pre}--pmc WRITE_SIZE --output-format csv -d gpurun_out/prof/write -o p -- {cmd}\n")
        if a.sq:
            f.write(f"{pre}--pmc {SQ_COUNTERS} --output-format csv -d gpurun_out/prof/sq -o p -- {cmd}\n")
        f.write(f"    python -m paper_2511_04283_amd.profile_summary --config {a.config} --name {a.name} --stats ... --fetch ... "
                "--write ... --sq ... --bench <the line of the first run>\n\n")
        f.write(f"Durations: `*_kernel_stats.csv` of the first run (averages over all calls of the run).  HBM bytes per launch: "
                f"FETCH_SIZE x {f_scale:.3f} and WRITE_SIZE x {w_scale:.3f} (KiB -> bytes), the factors with which the 256 MiB "
                "`__amd_rocclr_copyBuffer` of the same runs reads as 256 MiB each way.  Vector-issue utilisation = SQ_INSTS_VALU x 4 cycles "
                f"/ (duration x {CLOCK_GHZ} GHz x {SIMDS} SIMDs), only for kernels of 30 us and more; lane utilisation = "
                "SQ_THREAD_CYCLES_VALU / (SQ_ACTIVE_INST_VALU x 64); LDS conflict rate = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE.  "
                "MB = 1e6 bytes.\n\n")
        f.write("| kernel | calls | avg us | min us | % GPU time | fetch MB | write MB | GB/s | VALU insts | issue util | lane util | LDS conflict |\n")
        f.write("|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|\n")
        for r in rows:
            if r["pct"] < 0.05 and r["kernel"] != copy:
                continue
            gbs = (r["fetch"] + r["write"]) / (r["avg_us"] * 1e-6) / 1e9 if r["avg_us"] > 0 else 0.0
            f.write(f"| {r['kernel']} | {r['calls']} | {r['avg_us']:.1f} | {r['min_us']:.1f} | {r['pct']:.2f} | {r['fetch'] / 1e6:.1f} | "
                    f"{r['write'] / 1e6:.1f} | {gbs:.0f} | {fmt(r.get('valu'), '{:.3g}')} | {fmt(r.get('issue'))} | {fmt(r.get('lanes'))} | "
                    f"{fmt(r.get('conflict'), '{:.3f}')} |\n")
        f.write("\nKernel groups of one step, from bench.py's line of the first run (HIP-event durations measured inside the "
                "library, algorithmic work per launch) beside the counter traffic above:\n\n")
        f.write("| group | kernels | ms (events) | bound | algorithmic work | achieved | peak | fraction | HBM traffic (counters) | traffic / algorithmic |\n")
        f.write("|---|---|---:|---|---:|---:|---:|---:|---:|---:|\n")
        for grp, ro in bench.get("rooflines", {}).items():
            amount = ro.get("flops_per_launch", ro.get("bytes_per_launch", 0))
            unit = "Gflop" if ro["bound"] == "alu" else "MB"
            amt = amount / 1e9 if ro["bound"] == "alu" else amount / 1e6
            tr = group_bytes.get(grp)
            ratio = f"{tr / amount:.2f}" if tr and ro["bound"] == "hbm" and amount else "—"
            f.write(f"| {grp} | {ro['kernel']} | {ro['avg_launch_ms']:.4f} | {ro['bound']} | {amt:.1f} {unit} | {ro['achieved']:.1f} {ro['unit']} | "
                    f"{ro['peak']:g} | {ro['frac']:.3f} | {fmt(tr / 1e6 if tr else None, '{:.1f} MB')} | {ratio} |\n")
        ro = bench["roofline"]
        f.write(f"\nbench.py of that run: ms_per_step = {bench['ms_per_step']}, value = {bench['value']} {bench['unit']}; dominant group "
                f"`{ro.get('group')}` ({ro.get('kernel')}): {ro.get('achieved')} {ro.get('unit')} = {ro.get('frac')} of {ro.get('peak')} "
                f"(event-timed {ro.get('avg_launch_ms')} ms per launch under the profiler).\n")
    print(f"wrote {a.out}/{a.name}.md" + ("" if a.no_traffic else f" and traffic_cfg{a.config}{suffix}.json"))
    return 0


if __name__ == "__main__":
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    sys.exit(main())
