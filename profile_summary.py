"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python profile_summary.py stats <..._kernel_stats.csv> <..._kernel_trace.csv> <out.txt> --cmd "<command>"
    python profile_summary.py traffic <fetch_counter_collection.csv> <write_counter_collection.csv>
           <out.txt> --cmd "<command>" --classes <launch_classes.json> [--copy-bytes 268435456]
    python profile_summary.py counters <out.txt> <counter_collection.csv> ... --cmd "<command>" [--cmd ...]
    python profile_summary.py layers <out.txt> <bench_layers.json> ... --cmd "<command>" [--cmd ...]
    python profile_summary.py variants <out.txt> <bench.log> ... --cmd "<command>" [--cmd ...]
    python profile_summary.py npnet <out.txt> <bench.log> --cmd "<command>"

`stats`: per-kernel call count and durations of the whole run, and the kernels of the last full
pass (between the last two launches of the input quantization).
`traffic`: HBM bytes per launch of the matrix-core convolution kernels from the FETCH_SIZE and
WRITE_SIZE counters (KiB per dispatch), each scaled by what the same counter reads for the copy
probe of known size that `bench.py --copy-probe` runs (concat_kernel: reads and writes
--copy-bytes each).  Averages are taken over the last --launches-per-step launches, i.e. one pass
at the benchmark's batch size, separately for the launches that the HBM roofline bounds and for those that
the matrix-core roofline bounds (`bench.py --launch-classes` writes which launch of a pass is which).
`layers`: the JSON lines of `bench.py --layers` runs as one table.
`counters`: per kernel, the average per dispatch of every counter found in the given collection files
(one file per `rocprofv3 --pmc` run), and the ratios the design notes quote.
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
    return "conv_mfma_kernel" in name or "conv_pw_kernel" in name or "conv_fc_kernel" in name


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
    if a.no_pass:
        out.append("The totals include set-up and warm-up launches of the same command (the minima of the convolution kernels are the")
        out.append("calibration launches on 8 images).")
        open(a.out, "w").write("\n".join(out) + "\n")
        return
    out.append("The totals include the untimed calibration pass, plan set-up and warm-up of the same command.")
    tr = list(csv.DictReader(open(a.trace_csv)))
    tr.sort(key=lambda r: int(r["Start_Timestamp"]))
    # a pass begins with the conversion of the input images: a kernel of its own, or the first layer's kernel where that
    # takes the float images itself (the launches with the largest grid are the full-batch ones)
    first = "conv_stem_pool_kernel" if any(re.search(r"conv_stem_pool_kernel<\d+, \d+, true", r["Kernel_Name"]) for r in tr) else "quantize_vec4"
    starts = [i for i, r in enumerate(tr) if first in r["Kernel_Name"]]
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
        out.append(f"One pass (from one full-batch launch of {first} to the next): {len(seg)} kernels, GPU busy {busy / 1e3:.1f} us")
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
    import json
    classes = json.load(open(a.classes))                     # per-pass order of the matrix-core launches
    n = len(classes)
    out = ["HBM traffic of the matrix-core convolution kernels from rocprofv3 counters",
           "commands (run from /tmp with TMPDIR=/tmp on the MI355X box), one counter per run:", "  " + a.cmd.replace("COUNTER", "FETCH_SIZE"),
           "  " + a.cmd.replace("COUNTER", "WRITE_SIZE"),
           f"launches of one pass: {n} ({sum(1 for c in classes if c['bound'] == 'hbm')} bound by the HBM roofline at the published peaks, "
           f"{sum(1 for c in classes if c['bound'] == 'mfma')} by the matrix-core roofline)", ""]
    total = {"hbm": 0.0, "mfma": 0.0, "all": 0.0}
    for path, counter, label in ((a.fetch_csv, "FETCH_SIZE", "read"), (a.write_csv, "WRITE_SIZE", "written")):
        disp = per_dispatch(path, counter)
        copies = [v for nm, v in disp if "concat_kernel" in nm]
        convs = [v for nm, v in disp if is_conv(nm)][-n:]
        assert len(convs) == n, "fewer convolution dispatches than one pass has launches"
        copy_kib = sum(copies) / len(copies)
        factor = (a.copy_bytes / 1024.0) / copy_kib
        out.append(f"{counter}: copy probe ({len(copies)} launches, {a.copy_bytes} bytes {label} each) reads {copy_kib:.0f} KiB per launch "
                   f"-> scale factor {factor:.4f}")
        for c in ("hbm", "mfma", "all"):
            sel = [v for v, k in zip(convs, classes) if c == "all" or k["bound"] == c]
            kib = sum(sel) / max(len(sel), 1)
            total[c] += kib * factor * 1024.0
            out.append(f"{counter}: {len(sel):3d} launches ({c:4s}): {kib:.0f} KiB per launch raw, {kib * factor:.0f} KiB scaled")
    out.append("")
    out.append(f"hbm_bytes_per_launch_hbm_bound = {total['hbm']:.0f}")
    out.append(f"hbm_bytes_per_launch_mfma_bound = {total['mfma']:.0f}")
    out.append(f"hbm_bytes_per_launch = {total['all']:.0f}")
    open(a.out, "w").write("\n".join(out) + "\n")


def cmd_counters(a):
    per = collections.OrderedDict()         # kernel -> counter -> [sum over dispatches, dispatches]
    for path in a.csvs:
        seen = collections.OrderedDict()
        for r in csv.DictReader(open(path)):
            key = (int(r["Dispatch_Id"]), r["Counter_Name"])
            e = seen.setdefault(key, [short(r["Kernel_Name"]), 0.0])
            e[1] += float(r["Counter_Value"])
        for (_, counter), (kernel, v) in seen.items():
            if a.only and a.only not in kernel:
                continue
            e = per.setdefault(kernel, collections.OrderedDict()).setdefault(counter, [0.0, 0])
            e[0] += v; e[1] += 1
    out = ["rocprofv3 counters per kernel (average per dispatch over all dispatches of the run)",
           "commands (run from /tmp with TMPDIR=/tmp on the MI355X box), one counter group per run:"]
    out += ["  " + c for c in a.cmd]
    out.append("")
    for kernel, ctr in per.items():
        if max(e[1] for e in ctr.values()) < a.min_dispatches:
            continue                          # (calibration launches of the general epilogue and the like)
        out.append(kernel)
        avg = {c: e[0] / e[1] for c, e in ctr.items()}
        for c, e in ctr.items():
            out.append(f"    {c:32s} {avg[c]:16.1f}   ({e[1]} dispatches)")
        if "SQ_BUSY_CYCLES" in avg and "SQ_VALU_MFMA_BUSY_CYCLES" in avg and avg["SQ_BUSY_CYCLES"] > 0:
            out.append(f"    matrix pipe busy / SQ busy cycles        {avg['SQ_VALU_MFMA_BUSY_CYCLES'] / avg['SQ_BUSY_CYCLES']:.3f}")
        if "SQ_WAVE_CYCLES" in avg and avg["SQ_WAVE_CYCLES"] > 0:
            for c in ("SQ_WAIT_INST_LDS", "SQ_WAIT_INST_ANY", "SQ_WAIT_ANY", "SQ_ACTIVE_INST_LDS", "SQ_ACTIVE_INST_VALU", "SQ_INST_CYCLES_VMEM"):
                if c in avg:
                    out.append(f"    {c} / SQ_WAVE_CYCLES{'':10s} {avg[c] / avg['SQ_WAVE_CYCLES']:.3f}")
        if "SQ_LDS_BANK_CONFLICT" in avg and avg.get("SQ_LDS_IDX_ACTIVE", 0) > 0:
            out.append(f"    LDS bank conflict cycles / active        {avg['SQ_LDS_BANK_CONFLICT'] / avg['SQ_LDS_IDX_ACTIVE']:.4f}")
        out.append("")
    open(a.out, "w").write("\n".join(out) + "\n")


def cmd_layers(a):
    import json
    out = ["standalone layer timings (bench.py --layers: formats from the library's own calibration of each layer, four rotating",
           "buffer sets per layer, HIP events over the launches)", "commands:"]
    out += ["  " + c for c in a.cmd]
    for path in a.jsons:
        d = json.loads([x for x in open(path) if x.startswith("{")][-1])
        out += ["", d["metric"]]
        out.append(f"  {'layer':20s} {'shape':34s} {'kernel':10s} {'us':>7s} {'TOPS':>8s} {'GB/s':>8s} {'%mfma':>6s} {'%hbm':>6s} {'%roof':>6s}")
        for r in d["layers"]:
            num = lambda k, w: (f"{r[k]:{w}.1f}" if k in r else " " * (w - 1) + "-")
            out.append(f"  {r['layer']:20s} {r['shape']:34s} {r['kernel']:10s} {r['us']:7.1f} {num('tops', 8)} {num('gbs', 8)} "
                       f"{num('pct_mfma_peak', 6)} {num('pct_hbm_peak', 6)} {num('pct_roofline', 6)}"
                       + (f"   (as separate calls: {r['two_calls_us']:.1f} us)" if "two_calls_us" in r else ""))
    open(a.out, "w").write("\n".join(out) + "\n")


def cmd_variants(a):
    import json
    out = ["bench.py lines of the benchmark's variants (same box, back to back), the fields that differ", "commands:"]
    out += ["  " + c for c in a.cmd]
    out.append("")
    for path in a.logs:
        d = json.loads([x for x in open(path) if x.startswith("{")][-1])
        r, o = d.get("roofline", {}), d.get("roofline_other_class", {})
        out.append(f"weight formats: {d.get('weight_formats')}; joins: {d.get('joins')}")
        out.append(f"  {d['ms_per_step']:.4f} ms per step, {d['value']:.1f} {d['unit']}, {d.get('images_per_s', 0):.0f} images/s")
        out.append(f"  parity_checked: {d.get('parity_checked')}")
        out.append(f"  roofline ({r.get('bound')}): {r.get('achieved')} {r.get('unit')} = {r.get('frac')} of {r.get('peak')}; other class ({o.get('bound')}): "
                   f"{o.get('achieved')} {o.get('unit')} = {o.get('frac')} of {o.get('peak')}")
        out.append("")
    open(a.out, "w").write("\n".join(out) + "\n")


def cmd_npnet(a):
    import json
    d = json.loads([x for x in open(a.log) if x.startswith("{")][-1])
    out = ["bench.py line of the network pass on (8, 4) codes", "command:", "  " + a.cmd[0], "", d["metric"],
           f"  {d['ms_per_step']:.4f} ms per step, {d['value']:.1f} {d['unit']}, {d.get('images_per_s', 0):.0f} images/s; launch: {d['launch']}",
           f"  parity_checked: {d.get('parity_checked')}", f"  cpu_baseline: {d.get('cpu_baseline')}",
           f"  roofline: {d['roofline']['achieved']} {d['roofline']['unit']} = {d['roofline']['frac']} of {d['roofline']['peak']} ({d['roofline']['note']})",
           "", "library calls of one pass (event intervals on the launch stream, launched call by call):"]
    for k, v in d["calls"].items():
        out.append(f"  {k:24s} {v['calls']:3d} calls {v['us']:9.1f} us")
    out += ["", f"  {'layer':12s} {'us':>7s} {'TOPS':>8s} {'int8 matrix TOPS':>17s}"]
    for r in d["conv_layers"]:
        out.append(f"  {r['layer']:12s} {r['us']:7.1f} {r['tops']:8.1f} {r['int8_matrix_tops']:17.1f}")
    open(a.out, "w").write("\n".join(out) + "\n")


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    s = sub.add_parser("stats")
    s.add_argument("stats_csv"); s.add_argument("trace_csv"); s.add_argument("out"); s.add_argument("--cmd", required=True)
    s.add_argument("--no-pass", action="store_true", help="the command is not the network benchmark: no per-pass section")
    t = sub.add_parser("traffic")
    t.add_argument("fetch_csv"); t.add_argument("write_csv"); t.add_argument("out"); t.add_argument("--cmd", required=True)
    t.add_argument("--classes", required=True)
    t.add_argument("--copy-bytes", type=int, default=256 << 20)
    c = sub.add_parser("counters")
    c.add_argument("out"); c.add_argument("csvs", nargs="+"); c.add_argument("--cmd", action="append", required=True)
    c.add_argument("--only", default="conv_", help="keep kernels whose name contains this")
    c.add_argument("--min-dispatches", type=int, default=3, help="skip kernels launched fewer times than this")
    l = sub.add_parser("layers")
    l.add_argument("out"); l.add_argument("jsons", nargs="+"); l.add_argument("--cmd", action="append", required=True)
    v = sub.add_parser("variants")
    v.add_argument("out"); v.add_argument("logs", nargs="+"); v.add_argument("--cmd", action="append", required=True)
    n = sub.add_parser("npnet")
    n.add_argument("out"); n.add_argument("log"); n.add_argument("--cmd", action="append", required=True)
    a = ap.parse_args()
    {"npnet": cmd_npnet, "stats": cmd_stats, "traffic": cmd_traffic, "counters": cmd_counters, "layers": cmd_layers, "variants": cmd_variants}[a.what](a)


if __name__ == "__main__":
    main()
