#!/usr/bin/env python3
"""Summarise rocprofv3 output of a bench.py run into the short text files under profiles/.

    python -m paper_2511_10333_amd.profile_summary traffic --workload W --rank R \
        --fetch DIR --write DIR --cal-fetch DIR --cal-write DIR [--elements-per-launch N] --out profiles/traffic_W_rR.md
    python -m paper_2511_10333_amd.profile_summary kernels --trace DIR --title "..." --command "..." --out profiles/NAME.md

`traffic`: DIRs are the -d folders of four `rocprofv3 --pmc` runs (FETCH_SIZE and WRITE_SIZE of the
bench command, and of `bench.py --calibrate-copy`).  Both counters are in KiB per dispatch; the
calibration run (a plain device copy of 1 GiB per launch) gives the bytes one counted KiB stands
for.  The file ends with one `traffic_bytes_per_launch <kernel> <bytes>` line per kernel, which
bench.py reads for `roofline.traffic`.
`kernels`: DIR is the -d folder of a `rocprofv3 --kernel-trace --stats` run.
`counters`: DIR is the -d folder of any `rocprofv3 --pmc` run: mean of every counter per launch and kernel.
`cells`: the JSON line of `bench.py --workload cfg3_flat_1e9` as a table of its cells.
`bench`: the JSON line of a `bench.py` run, the headline figures and the other workloads as tables.
`rankcosts`: the JSON objects of `python -m paper_2511_10333_amd.calibrate` runs (one per line) as tables.
Kernels are named as bench.py names them (template arguments dropped, the whole-tile and
narrow forms of a pass under the pass's name).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import re
import sys

ALIASES = {"k_pass_p_deferred_full": "k_pass_p_deferred", "k_pass_p_deferred_narrow": "k_pass_p_deferred",
           "k_decompress_full": "k_decompress", "k_pass_q_full": "k_pass_q"}


def bench_name(kernel: str) -> str:
    k = re.sub(r"^void\s+", "", kernel).replace("(anonymous namespace)::", "")
    k = re.sub(r"\(.*$", "", k)
    full = k.replace("edgc::", "")
    base = re.sub(r"<.*$", "", full)
    return ALIASES.get(base, base), full


def find_csv(folder: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(folder, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit("no *%s under %s" % (suffix, folder))
    return hits[0]


def counter_per_launch(folder: str, counter: str):
    """{bench kernel name: (launches, mean counter value per launch, {variant: launches})}"""
    rows = list(csv.DictReader(open(find_csv(folder, "counter_collection.csv"))))
    tot = collections.defaultdict(float)
    disp = collections.defaultdict(set)
    var = collections.defaultdict(lambda: collections.defaultdict(set))
    for r in rows:
        if r["Counter_Name"] != counter:
            continue
        name, full = bench_name(r["Kernel_Name"])
        tot[name] += float(r["Counter_Value"])
        disp[name].add(r["Dispatch_Id"])
        var[name][full].add(r["Dispatch_Id"])
    return {k: (len(disp[k]), tot[k] / len(disp[k]), {v: len(d) for v, d in var[k].items()}) for k in tot}


def cmd_traffic(a) -> int:
    GiB = float(1 << 30)
    cal_f = counter_per_launch(a.cal_fetch, "FETCH_SIZE")
    cal_w = counter_per_launch(a.cal_write, "WRITE_SIZE")
    # the copy kernel of the calibration run: the one with the largest counter value
    cf = max(cal_f.values(), key=lambda t: t[1])
    cw = max(cal_w.values(), key=lambda t: t[1])
    f_factor = GiB / (cf[1] * 1024.0)      # bytes read per counted byte
    w_factor = GiB / (cw[1] * 1024.0)
    fetch = counter_per_launch(a.fetch, "FETCH_SIZE")
    write = counter_per_launch(a.write, "WRITE_SIZE")
    names = [k for k in fetch if k.startswith("k_")]
    names.sort(key=lambda k: -(fetch[k][1] + write.get(k, (0, 0.0, {}))[1]) * fetch[k][0])
    out = []
    out.append("# HBM-side traffic per launch — `%s`, rank %d (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)\n" % (a.workload, a.rank))
    out.append("Commands (each after `cd /tmp && export TMPDIR=/tmp`, from the repository root; `-d` names the output folder):\n")
    out.append("```")
    for c in a.command:
        out.append(c)
    out.append("python -m paper_2511_10333_amd.profile_summary traffic ...   # this file")
    out.append("```\n")
    out.append("Calibration, a plain device copy of 1 GiB per launch (`bench.py --calibrate-copy`): FETCH_SIZE reads "
               "%.4g KiB per launch (%d launches), WRITE_SIZE %.4g KiB: one counted KiB stands for %.3f KiB read and "
               "%.3f KiB written.\n" % (cf[1], cf[0], cw[1], f_factor, w_factor))
    out.append("| kernel | launches | FETCH_SIZE (KiB) | WRITE_SIZE (KiB) | bytes = %.2f x FETCH + %.2f x WRITE | forms seen |"
               % (f_factor, w_factor))
    out.append("|---|---|---|---|---|---|")
    lines = []
    for k in names:
        nf, f, forms = fetch[k]
        nw, w, _ = write.get(k, (0, 0.0, {}))
        b = (f * f_factor + w * w_factor) * 1024.0
        out.append("| `%s` | %d | %.4g | %.4g | %.1f MB | %s |" % (
            k, nf, f, w, b / 1e6, ", ".join("`%s` x %d" % (v, n) for v, n in sorted(forms.items()))))
        lines.append("traffic_bytes_per_launch %s %.6e" % (k, b))
    out.append("")
    out.append("The counters sit between the L2 caches and the memory fabric: bytes the 256 MB last-level cache behind "
               "that point serves are counted like HBM bytes.  A launch covers one group of the workload's matrices; "
               "the mean is over all launches of the run, the untimed warm-up steps included.\n")
    out.append("```")
    out.extend(lines)
    out.append("```")
    open(a.out, "w").write("\n".join(out) + "\n")
    print("\n".join(lines))
    return 0


def cmd_kernels(a) -> int:
    rows = list(csv.DictReader(open(find_csv(a.trace, "kernel_stats.csv"))))
    out = ["# %s\n" % a.title, "Command (after `cd /tmp && export TMPDIR=/tmp`, from the repository root):\n", "```"]
    out.extend(a.command)
    out.extend(["```\n", "| kernel (rocprofv3 name) | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"])
    for r in rows:
        name = r["Name"]
        if "edgc::" not in name and not name.startswith("k_"):
            continue
        full = bench_name(name)[1]
        out.append("| `%s` | %s | %.2f | %.2f | %.2f | %.2f |" % (
            full, r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
            float(r["Percentage"])))
    if a.note:
        out.append("")
        out.extend(a.note)
    open(a.out, "w").write("\n".join(out) + "\n")
    print("\n".join(out[-len(rows) - 4:]))
    return 0


def cmd_counters(a) -> int:
    rows = list(csv.DictReader(open(find_csv(a.dir, "counter_collection.csv"))))
    val = collections.defaultdict(lambda: collections.defaultdict(dict))     # kernel -> counter -> dispatch -> value
    names = []
    for r in rows:
        full = bench_name(r["Kernel_Name"])[1]
        if "k_" not in full:
            continue
        d = val[full][r["Counter_Name"]]
        d[r["Dispatch_Id"]] = d.get(r["Dispatch_Id"], 0.0) + float(r["Counter_Value"])
        if r["Counter_Name"] not in names:
            names.append(r["Counter_Name"])
    out = ["# %s\n" % a.title, "Command (after `cd /tmp && export TMPDIR=/tmp`, from the repository root):\n", "```"]
    out.extend(a.command)
    out.extend(["```\n",
                "Mean per launch over the launches that did work; `idle` counts launches whose first counter reads under "
                "1 % of the kernel's largest (a kernel queued behind the overflow gate of the one-read estimate returns at "
                "once).\n",
                "| kernel | launches | idle | " + " | ".join(names) + " |", "|---|---|---|" + "---|" * len(names)])
    def weight(k):
        return -max(val[k][names[0]].values() or [0.0])
    for k in sorted(val, key=weight):
        first = val[k][names[0]]
        top = max(first.values() or [0.0])
        live = [d for d, v in first.items() if v >= 0.01 * top] or list(first)
        cells = []
        for c in names:
            vs = [val[k][c].get(d, 0.0) for d in live]
            cells.append("%.4g" % (sum(vs) / len(vs)))
        out.append("| `%s` | %d | %d | %s |" % (k, len(live), len(first) - len(live), " | ".join(cells)))
    if a.note:
        out.append("")
        out.extend(a.note)
    open(a.out, "w").write("\n".join(out) + "\n")
    print("\n".join(out[-len(val) - 3 - len(a.note):]))
    return 0


def last_json_line(path: str):
    import json
    lines = [l for l in open(path) if l.startswith("{")]
    if not lines:
        sys.exit("no JSON line in %s" % path)
    return json.loads(lines[-1])


def cmd_cells(a) -> int:
    d = last_json_line(a.json)
    out = ["# %s\n" % a.title, "Command (from the repository root):\n", "```"]
    out.extend(a.command)
    out.extend(["```\n",
                "`ms`: one whole estimate, from a pair of events around back-to-back estimates.  `reads`: how often the "
                "estimate's kernels read the sample.  Kernel columns: microseconds per launch from a second pass with every "
                "launch between its own events (a kernel that only checks the overflow gate and returns reads about 1.6).\n",
                "| dtype | stride | bins | sampled | ms | reads | sample GB/s | buffer GB/s | kernels (us) |",
                "|---|---|---|---|---|---|---|---|---|"])
    for c in d["cells"]:
        ks = ", ".join("`%s` %.1f" % (k, v["avg_us"]) for k, v in c["kernels"].items() if v["avg_us"] >= 4.0)
        out.append("| %s | %d | %d | %d | %.4f | %d | %.0f | %.0f | %s |" % (
            c["dtype"], c["stride"], c["bins"], c["n_sampled"], c["ms"], c["reads_of_sample"], c["sample_gbs"],
            c["gradient_gbs"], ks))
    pk = d.get("device_peaks_measured") or {}
    out.append("")
    out.append("Measured on the same device in the same run: plain copy %s GB/s, plain read %s GB/s." % (
        pk.get("copy_gbs"), pk.get("read_gbs")))
    if d.get("roofline"):
        out.append("Roofline object of the line: `%s`." % d["roofline"])
    if d.get("cpu_baseline"):
        out.append("CPU baseline of the line: `%s`." % d["cpu_baseline"])
    if a.note:
        out.append("")
        out.extend(a.note)
    open(a.out, "w").write("\n".join(out) + "\n")
    print("wrote", a.out, len(d["cells"]), "cells")
    return 0


def cmd_bench(a) -> int:
    import json
    d = last_json_line(a.json)
    out = ["# %s\n" % a.title, "Command (from the repository root):\n", "```"]
    out.extend(a.command)
    out.extend(["```\n"])
    head = {k: d[k] for k in ("metric", "value", "unit", "ms_per_step", "steps", "warmup", "dtype", "arithmetic") if k in d}
    out.append("Headline: `%s`\n" % json.dumps(head))
    out.append("Workload: `%s`\n" % json.dumps(d.get("config")))
    out.append("Roofline: `%s`\n" % json.dumps(d.get("roofline")))
    out.append("CPU baseline: `%s`\n" % json.dumps(d.get("cpu_baseline")))
    out.append("Measured device ceilings: `%s`\n" % json.dumps(d.get("device_peaks_measured")))
    if d.get("kernels"):
        out.extend(["| kernel | launches per step | us per launch | GB/s (algorithmic bytes) | TFLOP/s | of the plain kernel of its traffic mix |",
                    "|---|---|---|---|---|---|"])
        for k, v in d["kernels"].items():
            frac = next((("%s %.3f" % (kk[len("frac_of_measured_"):], vv)) for kk, vv in v.items()
                         if kk.startswith("frac_of_measured_")), "")
            out.append("| `%s` | %s | %.2f | %s | %s | %s |" % (k, v.get("launches_per_step"), v["avg_us"], v.get("gbs"),
                                                               v.get("tflops"), frac))
        out.append("")
    if d.get("mfma"):
        out.append("MFMA: `%s`\n" % json.dumps(d["mfma"]))
    if d.get("other_workloads"):
        out.extend(["| workload | rank | ms per step | gradient GB/s | dominant kernel | its GB/s | of 8 TB/s |", "|---|---|---|---|---|---|---|"])
        for o in d["other_workloads"]:
            out.append("| `%s` | %s | %s | %s | `%s` | %s | %s |" % (
                o.get("workload"), o.get("rank"), o.get("ms_per_step"), o.get("gradient_gbs"), o.get("dominant_kernel"),
                o.get("dominant_gbs"), o.get("dominant_frac_of_hbm_peak")))
        out.append("")
    if d.get("dynamic"):
        dy = dict(d["dynamic"])
        out.append("Dynamic-rate run: `%s`\n" % json.dumps(dy))
    if a.note:
        out.extend(a.note)
    open(a.out, "w").write("\n".join(out) + "\n")
    print("wrote", a.out)
    return 0


def cmd_rankcosts(a) -> int:
    import json
    objs = [json.loads(l) for l in open(a.json) if l.startswith("{")]
    out = ["# %s\n" % a.title, "Commands (each prints one JSON object; the tables below are those numbers):\n", "```"]
    out.extend(a.command)
    out.extend(["```\n",
                "Times are sums over the four matrices of one transformer block (QKV, attention projection, MLP up, MLP down), "
                "one matrix at a time on one stream, each call between HIP events, mean over the rounds.  D_compressed = "
                "(m + n) r 4 bytes summed over the matrices; T_com = T_compress + T_decompress + D_compressed / B "
                "(Sec. IV-D-1).\n"])
    for d in objs:
        out.append("## hidden %d, %s gradients, %s residual: D_original = %.1f MB\n" % (
            d["hidden"], d["dtype"], d["residual"], d["bytes_original"] / 1e6))
        bws = d["bandwidths"]
        out.append("| rank | T_compress us | T_decompress us | D_compressed MB | " +
                   " | ".join("T_com @%g Gbit/s us" % b["gbps"] for b in bws) + " |")
        out.append("|---|---|---|---|" + "---|" * len(bws))
        for i, c in enumerate(d["costs"]):
            out.append("| %d | %.1f | %.1f | %.3f | %s |" % (
                c["rank"], c["t_compress_us"], c["t_decompress_us"], c["bytes_compressed"] / 1e6,
                " | ".join("%.0f" % b["t_com_us"][i] for b in bws)))
        out.append("")
        out.append("| bandwidth Gbit/s | D_original/B us | r_max | r_min | eta us per rank | MAPE % |")
        out.append("|---|---|---|---|---|---|")
        for b in bws:
            out.append("| %g | %.0f | %d | %d | %s | %s |" % (
                b["gbps"], b["t_uncompressed_us"], b["r_max"], b["r_min"],
                "-" if b["eta_us"] is None else "%.2f" % b["eta_us"],
                "-" if b["mape_percent"] is None else "%.1f" % b["mape_percent"]))
        out.append("")
    out.extend(a.note)
    open(a.out, "w").write("\n".join(out) + "\n")
    print("wrote", a.out)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("traffic")
    t.add_argument("--workload", required=True)
    t.add_argument("--rank", type=int, required=True)
    for k in ("fetch", "write", "cal-fetch", "cal-write", "out"):
        t.add_argument("--" + k, required=True)
    t.add_argument("--command", action="append", default=[])
    k = sub.add_parser("kernels")
    k.add_argument("--trace", required=True)
    k.add_argument("--title", required=True)
    k.add_argument("--out", required=True)
    k.add_argument("--command", action="append", default=[])
    k.add_argument("--note", action="append", default=[])
    c = sub.add_parser("counters")
    c.add_argument("--dir", required=True)
    for name in ("cells", "bench", "rankcosts"):
        j = sub.add_parser(name)
        j.add_argument("--json", required=True, help="file holding the JSON line bench.py printed")
        for q in (j,):
            pass
    for q in (c, sub.choices["cells"], sub.choices["bench"], sub.choices["rankcosts"]):
        q.add_argument("--title", required=True)
        q.add_argument("--out", required=True)
        q.add_argument("--command", action="append", default=[])
        q.add_argument("--note", action="append", default=[])
    a = ap.parse_args()
    return {"traffic": cmd_traffic, "kernels": cmd_kernels, "counters": cmd_counters, "cells": cmd_cells,
            "bench": cmd_bench, "rankcosts": cmd_rankcosts}[a.cmd](a)


if __name__ == "__main__":
    sys.exit(main())
