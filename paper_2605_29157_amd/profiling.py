"""Turn rocprofv3 CSV output into the short summaries kept under profiles/.

Nothing here touches the GPU or the library: it reads the CSV files that
`rocprofv3 --output-format csv ...` writes and prints Markdown / writes the key = value file
from which bench.py takes `roofline.traffic`.

    python3 -m paper_2605_29157_amd.profiling trace <..._kernel_trace.csv> [--kernel NAME --last K]
        per kernel: calls, mean / median / min / max duration. With --kernel and --last, also the
        statistics of the LAST K dispatches of the kernels whose name contains NAME -- bench.py
        puts its timed launches last (behind pre-roll and warm-up), so these are the launches
        its own figure comes from.
    python3 -m paper_2605_29157_amd.profiling counters <..._counter_collection.csv> [more.csv ...]
        per kernel and counter: mean value per dispatch.
    python3 -m paper_2605_29157_amd.profiling traffic --fetch F.csv --write W.csv --kernel NAME
            --copy-bytes N --key KEY --out profiles/hbm_traffic.txt
        HBM bytes per launch of the kernels whose name contains NAME: FETCH_SIZE and WRITE_SIZE
        (KiB per dispatch), each scaled by what the same counter reads for `util_copy_kernel`
        copying N bytes each way in the same run; stored as `KEY = bytes` in the output file
        (other keys in the file are kept).
"""
from __future__ import annotations

import argparse
import csv
import os
import statistics
import sys
from collections import defaultdict


def _short(name: str) -> str:
    name = name.replace("plx::", "")
    cut = name.find("(")
    return name if cut < 0 else name[:cut]


def read_trace(path):
    """{kernel name: [durations in us, in dispatch order]} from a kernel_trace.csv."""
    rows = []
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((int(r["Start_Timestamp"]), _short(r["Kernel_Name"]),
                         (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3))
    rows.sort()
    out = defaultdict(list)
    for _, name, us in rows:
        out[name].append(us)
    return out


def read_counters(paths):
    """{kernel name: {counter: [value per dispatch]}} from counter_collection.csv files."""
    out = defaultdict(lambda: defaultdict(lambda: defaultdict(float)))
    for path in paths:
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                # one row per (dispatch, counter [, dimension instance]): sum the instances
                out[_short(r["Kernel_Name"])][r["Counter_Name"]][(path, r["Dispatch_Id"])] += float(r["Counter_Value"])
    return {k: {c: list(v.values()) for c, v in cs.items()} for k, cs in out.items()}


def _stats_row(name, us):
    return "| `%s` | %d | %.2f | %.2f | %.2f | %.2f |" % (
        name, len(us), statistics.fmean(us), statistics.median(us), min(us), max(us))


def cmd_trace(opt):
    tr = read_trace(opt.csv)
    total = sum(sum(v) for v in tr.values())
    print("| kernel | calls | mean us | median us | min us | max us |")
    print("|---|---|---|---|---|---|")
    for name, us in sorted(tr.items(), key=lambda kv: -sum(kv[1])):
        if sum(us) >= 0.005 * total:
            print(_stats_row(name, us))
    if opt.kernel:
        for name, us in tr.items():
            if opt.kernel in name:
                last = us[-opt.last:] if opt.last else us
                print()
                print("last %d dispatches of `%s` (the timed launches): mean %.2f us, median %.2f us, "
                      "min %.2f us, max %.2f us" % (len(last), name, statistics.fmean(last),
                                                    statistics.median(last), min(last), max(last)))


def cmd_counters(opt):
    cs = read_counters(opt.csv)
    print("| kernel | counter | dispatches | mean per dispatch |")
    print("|---|---|---|---|")
    for name in sorted(cs):
        if opt.kernel and opt.kernel not in name:
            continue
        for c in sorted(cs[name]):
            v = cs[name][c]
            print("| `%s` | %s | %d | %.1f |" % (name, c, len(v), statistics.fmean(v)))


def read_traffic_file(path):
    vals = {}
    if os.path.exists(path):
        with open(path) as f:
            for line in f:
                line = line.split("#", 1)[0].strip()
                if "=" in line:
                    k, v = line.split("=", 1)
                    vals[k.strip()] = int(float(v))
    return vals


def cmd_traffic(opt):
    def mean_kib(path, counter, needle):
        cs = read_counters([path])
        hits = [v[counter] for k, v in cs.items() if needle in k and counter in v]
        if not hits:
            raise SystemExit("no %s for a kernel named *%s* in %s" % (counter, needle, path))
        vals = [x for h in hits for x in h]
        return statistics.fmean(vals), len(vals)

    copy_kib = opt.copy_bytes / 1024.0
    f_copy, _ = mean_kib(opt.fetch, "FETCH_SIZE", "util_copy_kernel")
    w_copy, _ = mean_kib(opt.write, "WRITE_SIZE", "util_copy_kernel")
    f_k, n_f = mean_kib(opt.fetch, "FETCH_SIZE", opt.kernel)
    w_k, n_w = mean_kib(opt.write, "WRITE_SIZE", opt.kernel)
    f_scale, w_scale = copy_kib / f_copy, copy_kib / w_copy
    rd, wr = f_k * f_scale * 1024.0, w_k * w_scale * 1024.0
    print("| kernel | FETCH_SIZE (KiB / dispatch) | WRITE_SIZE (KiB / dispatch) |")
    print("|---|---|---|")
    print("| `util_copy_kernel` (%d bytes each way) | %.1f | %.1f |" % (opt.copy_bytes, f_copy, w_copy))
    print("| `*%s*` (%d / %d dispatches) | %.1f | %.1f |" % (opt.kernel, n_f, n_w, f_k, w_k))
    print()
    print("scale factors: FETCH_SIZE x %.4f, WRITE_SIZE x %.4f" % (f_scale, w_scale))
    print("HBM read %.0f B + written %.0f B = %.0f B per launch" % (rd, wr, rd + wr))
    if opt.out:
        vals = read_traffic_file(opt.out)
        vals[opt.key] = int(round(rd + wr))
        with open(opt.out, "w") as f:
            f.write("# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE from rocprofv3 --pmc, each scaled by the same\n"
                    "# counter's reading for a plain copy of known size); written by\n"
                    "# `python3 -m paper_2605_29157_amd.profiling traffic`, read by bench.py (roofline.traffic)\n")
            for k in sorted(vals):
                f.write("%s = %d\n" % (k, vals[k]))


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("csv")
    t.add_argument("--kernel", default="")
    t.add_argument("--last", type=int, default=0)
    c = sub.add_parser("counters")
    c.add_argument("csv", nargs="+")
    c.add_argument("--kernel", default="")
    h = sub.add_parser("traffic")
    h.add_argument("--fetch", required=True)
    h.add_argument("--write", required=True)
    h.add_argument("--kernel", required=True)
    h.add_argument("--copy-bytes", type=int, default=1 << 30)
    h.add_argument("--key", required=True)
    h.add_argument("--out", default="")
    opt = ap.parse_args(argv)
    {"trace": cmd_trace, "counters": cmd_counters, "traffic": cmd_traffic}[opt.cmd](opt)


if __name__ == "__main__":
    main(sys.argv[1:])
