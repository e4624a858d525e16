"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python profile_summary.py stats <..._kernel_stats.csv> <..._kernel_trace.csv> <out.txt> --cmd "<command>"
    python profile_summary.py traffic <fetch_counter_collection.csv> <write_counter_collection.csv>
           <out.txt> --cmd "<command>" [--launches-per-step 53] [--copy-bytes 268435456]

`stats`: per-kernel call count and durations of the whole run, and the kernels of the last full
pass (between the last two launches of the input quantization).
`traffic`: HBM bytes per launch of the matrix-core convolution kernels from the FETCH_SIZE and
WRITE_SIZE counters (KiB per dispatch), each scaled by what the same counter reads for the copy
probe of known size that `bench.py --copy-probe` runs (concat_kernel: reads and writes
--copy-bytes each).  Averages are taken over the last --launches-per-step launches, i.e. one pass
at the benchmark's batch size.
"""
from __future__ import annotations

import argparse
import collections
import csv
import re


def short(name: str) -> str:
    name = name.replace("dfq::(anonymous namespace)::", "dfq::").replace("void ", "")
    name = re.sub(r"\(.*", "", name)
    return name[:86]


def is_conv(name: str) -> bool:
    return "conv_mfma_kernel" in name or "conv_pw_kernel" in name


def cmd_stats(a):
    rows = list(csv.DictReader(open(a.stats_csv)))
    out = ["rocprofv3 kernel statistics", "command (run from /tmp with TMPDIR=/tmp on the MI355X box):", "  " + a.cmd, ""]
    out.append(f"{'kernel':88s} {'calls':>6s} {'total_us':>10s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}")
    agg = collections.OrderedDict()
    for r in rows:
        k = short(r["Name"])
        e = agg.setdefault(k, [0, 0.0, 1e30, 0.0, 0.0])
        e[0] += int(r["Calls"]); e[1] += float(r["TotalDurationNs"]); e[2] = min(e[2], float(r["MinNs"]))
        e[3] = max(e[3], float(r["MaxNs"])); e[4] += float(r["Percentage"])
    for k, e in agg.items():
        out.append(f"{k:88s} {e[0]:6d} {e[1] / 1e3:10.1f} {e[1] / e[0] / 1e3:9.2f} {e[2] / 1e3:9.2f} {e[3] / 1e3:9.2f} {e[4]:6.2f}")
    out.append("")
    out.append("The totals include the untimed calibration pass, plan set-up and warm-up of the same command.")
    tr = list(csv.DictReader(open(a.trace_csv)))
    tr.sort(key=lambda r: int(r["Start_Timestamp"]))
    starts = [i for i, r in enumerate(tr) if "quantize_vec4" in r["Kernel_Name"]]
    big = max(int(tr[i]["Grid_Size_X"]) for i in starts)
    starts = [i for i in starts if int(tr[i]["Grid_Size_X"]) == big]
    if len(starts) >= 2:
        seg = tr[starts[-2]:starts[-1]]
        seg = [r for r in seg if "at::" not in r["Kernel_Name"]]          # the spin kernel ahead of an instrumented pass
        busy = sum(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in seg)
        per = collections.OrderedDict()
        for r in seg:
            k = short(r["Kernel_Name"])
            e = per.setdefault(k, [0, 0])
            e[0] += 1; e[1] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
        out.append("")
        out.append(f"One pass (the launches between the last two input quantizations): {len(seg)} kernels, GPU busy {busy / 1e3:.1f} us")
        for k, e in sorted(per.items(), key=lambda kv: -kv[1][1]):
            out.append(f"  {e[1] / 1e3:9.1f} us {e[0]:4d} launches  avg {e[1] / 1e3 / e[0]:8.2f} us  {k}")
        conv = [(n, e) for n, e in per.items() if is_conv(n)]
        n = sum(e[0] for _, e in conv); t = sum(e[1] for _, e in conv)
        if n:
            out.append(f"  matrix-core convolution kernels together: {n} launches, {t / 1e3:.1f} us, average {t / 1e3 / n:.2f} us per launch")
    open(a.out, "w").write("\n".join(out) + "\n")


def per_dispatch(path, counter):
    d = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        key = int(r["Dispatch_Id"])
        e = d.setdefault(key, [r["Kernel_Name"], 0.0])
        e[1] += float(r["Counter_Value"])
    return [d[k] for k in sorted(d)]


def cmd_traffic(a):
    out = ["HBM traffic of the matrix-core convolution kernels from rocprofv3 counters",
           "commands (run from /tmp with TMPDIR=/tmp on the MI355X box), one counter per run:", "  " + a.cmd.replace("COUNTER", "FETCH_SIZE"),
           "  " + a.cmd.replace("COUNTER", "WRITE_SIZE"), ""]
    total = 0.0
    for path, counter, label in ((a.fetch_csv, "FETCH_SIZE", "read"), (a.write_csv, "WRITE_SIZE", "written")):
        disp = per_dispatch(path, counter)
        copies = [v for n, v in disp if "concat_kernel" in n]
        convs = [v for n, v in disp if is_conv(n)][-a.launches_per_step:]
        copy_kib = sum(copies) / len(copies)
        factor = (a.copy_bytes / 1024.0) / copy_kib
        conv_kib = sum(convs) / len(convs)
        total += conv_kib * factor * 1024.0
        out.append(f"{counter}: copy probe ({len(copies)} launches, {a.copy_bytes} bytes {label} each) reads {copy_kib:.0f} KiB per launch "
                   f"-> scale factor {factor:.4f}")
        out.append(f"{counter}: convolution kernels, last {len(convs)} launches: {conv_kib:.0f} KiB per launch raw, "
                   f"{conv_kib * factor:.0f} KiB scaled")
    out.append("")
    out.append(f"hbm_bytes_per_launch = {total:.0f}")
    open(a.out, "w").write("\n".join(out) + "\n")


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    s = sub.add_parser("stats")
    s.add_argument("stats_csv"); s.add_argument("trace_csv"); s.add_argument("out"); s.add_argument("--cmd", required=True)
    t = sub.add_parser("traffic")
    t.add_argument("fetch_csv"); t.add_argument("write_csv"); t.add_argument("out"); t.add_argument("--cmd", required=True)
    t.add_argument("--launches-per-step", type=int, default=53)
    t.add_argument("--copy-bytes", type=int, default=256 << 20)
    a = ap.parse_args()
    (cmd_stats if a.what == "stats" else cmd_traffic)(a)


if __name__ == "__main__":
    main()
