#!/usr/bin/env python3
"""Counter and trace summaries of the hop kernel for bench.py's workloads.

    python bench_counters.py [--workloads 1 2 3 4] [--steps 10]

For each workload it runs `python3 bench.py --workload N` under rocprofv3, one pass
per counter set (rocprofv3 does not split counters over passes): a --kernel-trace
--stats pass for durations, then --pmc passes for FETCH_SIZE, WRITE_SIZE, the L2 hit and
miss counts and the occupancy.  It writes a short text summary per workload under
profiles/ (the figures, with the commands that made them) and records the hop kernel's
HBM bytes per launch in profiles/hop_traffic.json, which bench.py reports as
roofline.traffic while the workload and the library options are the same.

FETCH_SIZE and WRITE_SIZE are in KiB per dispatch; each is scaled by what the same
counter reads for the library's plain row copy (gp_copy_rows, which reads and writes
n*d*element bytes exactly) in the same run.

This script starts no GPU work of its own: every GPU process is a child
(`rocprofv3 ... -- python3 bench.py ...`), each under a time limit.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(os.environ.get("TMPDIR", "/tmp"), "gp_counters")   # raw rocprofv3 output and logs: scratch
PROFILES = os.path.join(ROOT, "profiles")
NAMES = {1: "config1_tiny", 2: "config2_chunglu_arxiv_like", 3: "config3_chunglu_mean_d100", 4: "config4_sbm_sum_d602"}
PMC_SETS = ["FETCH_SIZE", "WRITE_SIZE", "TCC_HIT_sum TCC_MISS_sum", "MeanOccupancyPerCU"]
HOP_KERNELS = ("gp_hop_segments", "gp_hop_cluster_lds", "gp_pack_strips")   # a hop's launches: the figures below are means over all of them


def run(cmd, log, limit):
    with open(log, "w") as f:
        rc = subprocess.call(["timeout", "-s", "KILL", str(limit)] + cmd, stdout=f, stderr=subprocess.STDOUT, cwd=ROOT,
                             env=dict(os.environ, TMPDIR="/tmp"))
    if rc != 0:
        tail = "".join(open(log).readlines()[-15:])
        sys.exit(f"bench_counters.py: {' '.join(cmd)} ended with {rc}; end of {log}:\n{tail}")


def kernel_of(name: str) -> str:
    m = re.search(r"(gp_[a-z_0-9]+|__amd_rocclr_\w+)", name)
    return m.group(1) if m else name[:40]


def per_kernel_means(csv_path):
    acc = collections.defaultdict(lambda: collections.defaultdict(float))
    kn = {}
    for r in csv.DictReader(open(csv_path)):
        acc[r["Dispatch_Id"]][r["Counter_Name"]] += float(r["Counter_Value"])
        kn[r["Dispatch_Id"]] = kernel_of(r["Kernel_Name"])
    per = collections.defaultdict(list)
    for d, c in acc.items():
        per[kn[d]].append(c)
    out = {k: {c: sum(x[c] for x in v) / len(v) for c in v[0]} for k, v in per.items()}
    hop = [c for k in HOP_KERNELS for c in per.get(k, [])]
    if hop:
        out["hop launches together"] = {c: sum(x[c] for x in hop) / len(hop) for c in hop[0]}
    return out


def main() -> int:
    global PROFILES
    ap = argparse.ArgumentParser()
    ap.add_argument("--workloads", type=int, nargs="+", default=[1, 2, 3, 4])
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE", help="passed on to bench.py")
    ap.add_argument("--out-dir", default=PROFILES, help="where the summaries and hop_traffic.json go (default: profiles/)")
    args = ap.parse_args()
    PROFILES = os.path.abspath(args.out_dir)
    os.makedirs(OUT, exist_ok=True)
    os.makedirs(PROFILES, exist_ok=True)
    opt = [x for o in args.option for x in ("--option", o)]
    traffic_path = os.path.join(PROFILES, "hop_traffic.json")
    try:
        traffic = json.load(open(traffic_path))
    except (OSError, ValueError):
        traffic = {}

    for wl in args.workloads:
        tag = NAMES.get(wl, f"config{wl}")
        bench = ["python3", "bench.py", "--no-cpu-baseline", "--workload", str(wl)] + opt
        lines = []
        # ---- durations ------------------------------------------------------------
        d = os.path.join(OUT, f"trace_w{wl}")
        shutil.rmtree(d, ignore_errors=True)
        cmd = ["rocprofv3", "--kernel-trace", "--stats", "-d", d, "-o", "t", "--output-format", "csv",
               "--"] + bench + ["--steps", str(args.steps)]
        log = os.path.join(OUT, f"trace_w{wl}.log")
        run(cmd, log, 600)
        rec = json.loads([l for l in open(log) if l.startswith("{")][-1])
        stats = list(csv.DictReader(open(glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True)[0])))
        shutil.rmtree(d, ignore_errors=True)
        lines += [f"# gp_hop_segments on {rec['config']['workload']}", "",
                  "rocprofv3 summaries for the hop kernel (gather / scale / accumulate) of `gp_propagate`, MI355X (gfx950), one GPU.",
                  f"n = {rec['config']['n']}, nnz = {rec['config']['nnz']}, d = {rec['config']['d']}, K = {rec['config']['K']}, "
                  f"{rec['config']['edge_blocks']} edge blocks, {rec['config']['segments']} segments, "
                  f"{rec['config']['partial_rows']} partial rows; work lists: {rec['config']['work_lists']}; "
                  f"options {json.dumps(rec['config']['options'])}.", "",
                  "## Kernel durations", "", "Command (from the repository root):", "", "    " + " ".join(cmd), "",
                  "| kernel | calls | average ns | % of GPU time | min ns | max ns |", "|---|---|---|---|---|---|"]
        # one row per kernel name (a hop may use two instantiations of the hop kernel: the launch over the
        # records that gather outside the row's cluster and the one over those that gather inside it)
        agg = collections.OrderedDict()
        for s in stats:
            k = kernel_of(s["Name"])
            a = agg.setdefault(k, {"calls": 0, "total": 0.0, "pct": 0.0, "min": None, "max": None, "kinds": 0})
            a["calls"] += int(s["Calls"])
            a["total"] += float(s["AverageNs"]) * int(s["Calls"])
            a["pct"] += float(s["Percentage"])
            a["min"] = int(s["MinNs"]) if a["min"] is None else min(a["min"], int(s["MinNs"]))
            a["max"] = int(s["MaxNs"]) if a["max"] is None else max(a["max"], int(s["MaxNs"]))
            a["kinds"] += 1
        for k, a in agg.items():
            note = f" ({a['kinds']} instantiations)" if a["kinds"] > 1 else ""
            lines.append(f"| {k}{note} | {a['calls']} | {a['total'] / a['calls']:.0f} | {a['pct']:.2f} | {a['min']} | {a['max']} |")
        hop_avg_ns = sum(agg[k]["total"] for k in HOP_KERNELS if k in agg) / sum(agg[k]["calls"] for k in HOP_KERNELS if k in agg)
        rl = rec["roofline"]
        if rl["launches_per_hop"] > 1:
            lines += ["", f"A hop is {rl['launches_per_hop']} launches here ({rl['kernel']}); every per-launch figure below is the mean "
                          f"over all of them ({hop_avg_ns:.0f} ns in the table above), a hop is {rl['launches_per_hop']} times that."]
        lines += ["", f"bench.py in the same run: {rec['value']} GEFU/s, {rec['ms_per_step']} ms per step; hop kernel timed with HIP "
                      f"events inside bench.py: {rl['avg_launch_us']} us per launch (rocprofv3 average above: {hop_avg_ns / 1e3:.1f} us).",
                  f"Algorithmic bytes per launch {rl['algorithmic_bytes_per_launch']} -> {rl['achieved']} GB/s = {rl['frac']} of the "
                  f"8 TB/s peak; fp32 vector arithmetic {rl['other_bounds']['alu']['achieved']} TFLOP/s = "
                  f"{rl['other_bounds']['alu']['frac']} of 157.3; gathered rows {rl['other_bounds']['gathered_rows']['achieved']} GB/s.", ""]
        # ---- counters ---------------------------------------------------------------
        means = {}
        cmds = []
        for cset in PMC_SETS:
            name = cset.replace(" ", "_")
            d = os.path.join(OUT, f"pmc_w{wl}_{name}")
            shutil.rmtree(d, ignore_errors=True)
            cmd = ["rocprofv3", "--pmc"] + cset.split() + ["--kernel-trace", "-d", d, "-o", "p",
                                                          "--output-format", "csv", "--"] + bench + ["--steps", "3", "--warmup", "1"]
            run(cmd, os.path.join(OUT, f"pmc_w{wl}_{name}.log"), 600)
            cmds.append("    " + " ".join(cmd))
            f = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)[0]
            for k, v in per_kernel_means(f).items():
                means.setdefault(k, {}).update(v)
            shutil.rmtree(d, ignore_errors=True)
        n, dd = rec["config"]["n"], rec["config"]["d"]
        copy_kib = n * dd * 4 / 1024.0
        cp, hop = means.get("gp_copy_rows", {}), means["hop launches together"]
        f_fetch = copy_kib / cp["FETCH_SIZE"] if cp.get("FETCH_SIZE") else 2.0
        f_write = copy_kib / cp["WRITE_SIZE"] if cp.get("WRITE_SIZE") else 1.0
        fetch_b = hop["FETCH_SIZE"] * f_fetch * 1024
        write_b = hop["WRITE_SIZE"] * f_write * 1024
        total = fetch_b + write_b
        alg = rl["algorithmic_bytes_per_launch"]
        hit, miss = hop.get("TCC_HIT_sum", 0.0), hop.get("TCC_MISS_sum", 0.0)
        lines += ["## HBM traffic, L2 hit rate and occupancy (mean per dispatch)", "", "Commands (one counter set per run):", ""] + cmds + ["",
                  f"Scale factors from the plain copy kernel of the same run (gp_copy_rows reads and writes n*d*4 B = {copy_kib:.1f} KiB): "
                  f"FETCH_SIZE reads {cp.get('FETCH_SIZE', float('nan')):.1f} -> factor {f_fetch:.4f}; "
                  f"WRITE_SIZE reads {cp.get('WRITE_SIZE', float('nan')):.1f} -> factor {f_write:.4f}.", "",
                  "| kernel | FETCH_SIZE (KiB) | WRITE_SIZE (KiB) | TCC_HIT_sum | TCC_MISS_sum | MeanOccupancyPerCU |", "|---|---|---|---|---|---|"]
        for k, v in sorted(means.items()):
            if k.startswith("gp_") or k.startswith("hop "):
                lines.append(f"| {k} | {v.get('FETCH_SIZE', 0):.1f} | {v.get('WRITE_SIZE', 0):.1f} | {v.get('TCC_HIT_sum', 0):.0f} | "
                             f"{v.get('TCC_MISS_sum', 0):.0f} | {v.get('MeanOccupancyPerCU', 0):.1f} |")
        lines += ["", f"Hop launches, scaled: fetch {fetch_b / 1e9:.4f} GB + write {write_b / 1e9:.4f} GB = **{total / 1e9:.4f} GB per launch** "
                      f"({total / (hop_avg_ns * 1e-9) / 1e12:.2f} TB/s over the {hop_avg_ns / 1e3:.1f} us launch).  Algorithmic (compulsory) bytes "
                      f"per launch: {alg / 1e9:.4f} GB; measured / algorithmic = {total / alg:.2f}.  All rows gathered: "
                      f"{rec['config']['nnz'] * dd * 4 / 1e9:.3f} GB per hop.  L2 hit rate over all requests (rows, ids, weights, "
                      f"stores): {100 * hit / max(hit + miss, 1):.1f} %.", ""]
        per_kernel = {k: {"fetch_bytes": int(means[k].get("FETCH_SIZE", 0.0) * f_fetch * 1024),
                          "write_bytes": int(means[k].get("WRITE_SIZE", 0.0) * f_write * 1024)} for k in HOP_KERNELS if k in means}
        lines += ["Per hop kernel, scaled the same way: " + "; ".join(
            f"{k} fetch {v['fetch_bytes'] / 1e9:.3f} GB + write {v['write_bytes'] / 1e9:.3f} GB" for k, v in per_kernel.items()) + ".", ""]
        traffic[str(wl)] = {"bytes_per_launch": int(total), "fetch_bytes": int(fetch_b), "write_bytes": int(write_b), "per_kernel": per_kernel,
                            "l2_hit_rate": round(hit / max(hit + miss, 1), 4), "options": rec["config"]["options"],
                            "work_lists": rec["config"]["work_lists"], "summary": f"profiles/gp_hop_segments_{tag}.md"}
        with open(os.path.join(PROFILES, f"gp_hop_segments_{tag}.md"), "w") as f:
            f.write("\n".join(lines))
        with open(traffic_path, "w") as f:
            json.dump(traffic, f, indent=1, sort_keys=True)
        print(f"workload {wl}: hop {hop_avg_ns / 1e3:.1f} us, {total / 1e9:.3f} GB per launch, L2 hit {100 * hit / max(hit + miss, 1):.1f} %", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
