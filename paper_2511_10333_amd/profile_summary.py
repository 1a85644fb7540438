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
           "k_decompress_full": "k_decompress"}


def bench_name(kernel: str) -> str:
    k = re.sub(r"^void\s+", "", kernel)
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
    a = ap.parse_args()
    return cmd_traffic(a) if a.cmd == "traffic" else cmd_kernels(a)


if __name__ == "__main__":
    sys.exit(main())
