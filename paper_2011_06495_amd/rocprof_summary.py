"""Turns the CSV files rocprofv3 writes for a run of bench.py into the short text tables kept
under profiles/ (the raw output stays where rocprofv3 put it).

  python -m paper_2011_06495_amd.rocprof_summary trace    DIR BENCH_JSON --command "..." --out FILE
  python -m paper_2011_06495_amd.rocprof_summary hbm      FETCH_DIR WRITE_DIR BENCH_JSON --command "..." --out FILE
  python -m paper_2011_06495_amd.rocprof_summary counters DIR [DIR ...] --command "..." --out FILE

DIR is what rocprofv3 was given as `-d` with `-o bench --output-format csv`; BENCH_JSON is the file
bench.py's standard output of the same run was sent to.  `--command` is repeated once per command
line to be quoted in the summary.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os

HBM_PEAK_GBS = 8000.0


def short_name(name: str) -> str:
    return name.replace("void ", "").split("(")[0].split("<")[0].split("::")[-1]


def ours(name: str) -> bool:
    return name.startswith("mv_") or name.startswith("codec_") or name.startswith("quant_")


def find_csv(dirn: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(dirn, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, dirn))
    return hits[0]


def bench_line(path: str) -> dict:
    lines = [l for l in open(path).read().strip().splitlines() if l.startswith("{")]
    return json.loads(lines[-1])


def kernel_stats(dirn: str):
    """[(kernel, calls, avg_ns, min_ns, max_ns)] in launch order of first appearance, ours only."""
    rows = list(csv.DictReader(open(find_csv(dirn, "kernel_stats.csv"))))
    order = launch_order(dirn)
    out = []
    for r in rows:
        k = short_name(r["Name"])
        if ours(k):
            out.append((k, int(r["Calls"]), float(r["AverageNs"]), int(float(r["MinNs"])), int(float(r["MaxNs"]))))
    out.sort(key=lambda s: order.get(s[0], 1 << 30))
    return out


def launch_order(dirn: str) -> dict:
    try:
        path = find_csv(dirn, "kernel_trace.csv")
    except SystemExit:
        return {}
    first = {}
    for r in csv.DictReader(open(path)):
        k = short_name(r["Kernel_Name"])
        t = int(r["Start_Timestamp"])
        if k not in first or t < first[k]:
            first[k] = t
    return first


def counter_table(dirn: str):
    """{counter: {kernel: [values per dispatch]}} for our kernels, kernels in order of first dispatch."""
    acc = collections.OrderedDict()
    for r in csv.DictReader(open(find_csv(dirn, "counter_collection.csv"))):
        k = short_name(r["Kernel_Name"])
        if not ours(k):
            continue
        acc.setdefault(r["Counter_Name"], collections.OrderedDict()).setdefault(k, []).append(float(r["Counter_Value"]))
    return acc


def avg(a):
    return sum(a) / len(a)


def dominant(j: dict) -> dict:
    """bench.py's roofline entry; for a run without the library's events (--profile-level 0) the
    same figures from the workload: the streaming kernel reads g and e and writes e once."""
    if j.get("roofline"):
        return j["roofline"]
    c = j["config"]
    per = 10 if "grads=bf16" in c["workload"] else 12
    return {"kernel": "mv_stream_collect", "algorithmic_bytes_per_launch": per * c["N"] * c["d"],
            "algorithmic_bytes_rule": "%d B x %d x %s" % (per, c["N"], format(c["d"], ","))}


def header(title, commands):
    L = [title, "", "commands (from the repository root, after `python -c 'import __graft_entry__ as g; g.build()'`;",
         "rocprofv3 wants `cd /tmp && export TMPDIR=/tmp` first and paths to the repository made absolute):"]
    for c in commands:
        L.append("  " + c)
    L.append("")
    return L


def describe(j: dict) -> str:
    c = j["config"]
    return "%s (N=%d, d=%s, K=%s; %s)" % (c["workload"].split(":")[0], c["N"], format(c["d"], ","), format(c["K"], ","),
                                           c["scheme"])


def cmd_trace(a):
    j = bench_line(a.bench_json)
    rows = kernel_stats(a.dir)
    r = j["roofline"]
    L = header("rocprofv3 kernel trace of the vote step, workload %s, one MI355X" % describe(j), a.command)
    L.append("bench.py's own line in the same run: ms_per_step = %.4f (wall), median of the per-step HIP events = %.4f," %
             (j["ms_per_step"], j["ms_per_step_median_of_events"]))
    L.append("roofline.avg_kernel_ms (HIP events around %s inside the timed region) = %.4f," % (r["kernel"], r["avg_kernel_ms"]))
    L.append("roofline.achieved = %.1f GB/s, frac = %.4f" % (r["achieved"], r["frac"]))
    L.append("")
    L.append("kernel_stats.csv, this library's kernels in launch order (calls include warm-up and the oracle-check steps):")
    L.append("%-28s %6s %12s %10s %10s" % ("kernel", "calls", "avg_ns", "min_ns", "max_ns"))
    tot, nk, dom = 0.0, 0, None
    for s in rows:
        L.append("%-28s %6d %12.1f %10d %10d" % s)
        if s[0] != "mv_probe_copy_kernel":
            tot += s[2]
            nk += 1
        if s[0] == r["kernel"]:
            dom = s
    L.append("sum of the %d step kernels' averages: %.1f ns (they run back to back on one stream)" % (nk, tot))
    L.append("")
    alg = r["algorithmic_bytes_per_launch"]
    if dom:
        L.append("%s: %s algorithmic bytes per launch (%s);" % (dom[0], format(int(alg), ","), r.get("algorithmic_bytes_rule", "")))
        L.append("  at the trace's average %.1f us that is %.1f GB/s = %.3f of the %d GB/s HBM peak" %
                 (dom[2] / 1e3, alg / dom[2], alg / dom[2] / HBM_PEAK_GBS, HBM_PEAK_GBS))
        L.append("  (HIP events in bench.py: %.1f us; the two agree within %.1f %%)" %
                 (r["avg_kernel_ms"] * 1e3, abs(r["avg_kernel_ms"] * 1e6 / dom[2] - 1) * 100))
    for s in rows:
        if s[0] == "mv_probe_copy_kernel" and "copy_probe_bytes_each_way" in j:
            b = j["copy_probe_bytes_each_way"]
            L.append("mv_probe_copy_kernel (plain copy, %s B read + %s B written): %.1f us = %.1f GB/s" %
                     (format(b, ","), format(b, ","), s[2] / 1e3, 2 * b / s[2]))
    open(a.out, "w").write("\n".join(L) + "\n")


def cmd_hbm(a):
    j = bench_line(a.bench_json)
    f = counter_table(a.fetch_dir)["FETCH_SIZE"]
    w = counter_table(a.write_dir)["WRITE_SIZE"]
    copy_kib = j["copy_probe_bytes_each_way"] / 1024.0
    sf = copy_kib / avg(f["mv_probe_copy_kernel"])
    sw = copy_kib / avg(w["mv_probe_copy_kernel"])
    r = dominant(j)
    L = header("HBM traffic of the vote step's kernels from rocprofv3 counters, workload %s" % describe(j), a.command)
    L.append("calibration: mv_probe_copy_kernel reads %s B and writes %s B (= %.2f KiB each)" %
             (format(j["copy_probe_bytes_each_way"], ","), format(j["copy_probe_bytes_each_way"], ","), copy_kib))
    L.append("  FETCH_SIZE reads %.1f per dispatch -> scale %.4f to KiB;  WRITE_SIZE reads %.1f -> scale %.4f" %
             (avg(f["mv_probe_copy_kernel"]), sf, avg(w["mv_probe_copy_kernel"]), sw))
    L.append("")
    L.append("%-24s %4s %14s %14s %14s %14s" % ("kernel", "n", "FETCH_SIZE", "WRITE_SIZE", "read_MB", "written_MB"))
    tot, dom = 0.0, None
    for k in f:
        if k == "mv_probe_copy_kernel" or k not in w:
            continue
        rb, wb = avg(f[k]) * sf * 1024, avg(w[k]) * sw * 1024
        tot += rb + wb
        L.append("%-24s %4d %14.1f %14.1f %14.2f %14.2f" % (k, len(f[k]), avg(f[k]), avg(w[k]), rb / 1e6, wb / 1e6))
        if k == r["kernel"]:
            dom = (rb, wb)
    alg = r["algorithmic_bytes_per_launch"]
    L.append("")
    L.append("%s: %d B read + %d B written per launch" % (r["kernel"], dom[0], dom[1]))
    L.append("traffic_bytes_per_launch = %d" % (dom[0] + dom[1]))
    L.append("algorithmic_bytes_per_launch = %d   (%s)" % (alg, r.get("algorithmic_bytes_rule", "")))
    L.append("traffic / algorithmic = %.4f" % ((dom[0] + dom[1]) / alg))
    L.append("whole step, all kernels above: %d B = %.4f x algorithmic" % (tot, tot / alg))
    open(a.out, "w").write("\n".join(L) + "\n")


def cmd_counters(a):
    tables = collections.OrderedDict()
    for d in a.dirs:
        for c, per_kernel in counter_table(d).items():
            tables[c] = per_kernel
    kernels = []
    for per_kernel in tables.values():
        for k in per_kernel:
            if k not in kernels and k != "mv_probe_copy_kernel":
                kernels.append(k)
    L = header(a.title, a.command)
    L.append("average per dispatch over the run's dispatches of each kernel (n = dispatches counted)")
    names = list(tables)
    for i in range(0, len(names), 4):
        part = names[i:i + 4]
        L.append("")
        L.append("%-22s %4s " % ("kernel", "n") + " ".join("%26s" % c for c in part))
        for k in kernels:
            n = max(len(tables[c].get(k, [])) for c in part)
            L.append("%-22s %4d " % (k, n) +
                     " ".join("%26.1f" % avg(tables[c][k]) if k in tables[c] else "%26s" % "-" for c in part))
    if a.note:
        L.append("")
        L.extend(a.note)
    open(a.out, "w").write("\n".join(L) + "\n")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    t = sub.add_parser("trace")
    t.add_argument("dir")
    t.add_argument("bench_json")
    h = sub.add_parser("hbm")
    h.add_argument("fetch_dir")
    h.add_argument("write_dir")
    h.add_argument("bench_json")
    c = sub.add_parser("counters")
    c.add_argument("dirs", nargs="+")
    c.add_argument("--title", required=True)
    c.add_argument("--note", action="append", default=[])
    for p in (t, h, c):
        p.add_argument("--command", action="append", default=[])
        p.add_argument("--out", required=True)
    a = ap.parse_args()
    {"trace": cmd_trace, "hbm": cmd_hbm, "counters": cmd_counters}[a.what](a)


if __name__ == "__main__":
    main()
