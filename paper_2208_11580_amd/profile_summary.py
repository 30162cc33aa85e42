"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2208_11580_amd.profile_summary stats   <kernel_stats.csv> <passes> <title> <command> > profiles/<name>.md
    python -m paper_2208_11580_amd.profile_summary traffic <fetch_counter_collection.csv> <write_counter_collection.csv> \
                                                           <workload> <command> > profiles/<name>.txt

    python -m paper_2208_11580_amd.profile_summary counters <title> <command> <counter_collection.csv>... > profiles/<name>.txt

`counters` lists, per kernel, every counter found in the given runs (one run per counter set):
percent-type derived metrics (names ending in Util / Busy / Stalled) are averaged over the launches,
everything else is summed.

`traffic` scales the FETCH_SIZE / WRITE_SIZE counters (KiB per dispatch) by what the same counter
reads for the plain 1 GiB device copy that `bench.py --calib-copy` appends to the run (the copy
reads 1 GiB and writes 1 GiB), and reports the HBM bytes per launch of every row-solver kernel.
"""
from __future__ import annotations

import collections
import csv
import sys

GIB_KIB = 1048576.0


def _short(name: str) -> str:
    n = name.replace("(anonymous namespace)::", "").replace("obc_blocked::", "").replace("void ", "")
    if n.startswith("Cijk"):
        return "Cijk_... (torch matmul of the input generator)"
    if "at::native" in n:
        return "torch elementwise (input generator)"
    return n.split("(")[0]


def stats(path, passes, title, command):
    rows = list(csv.DictReader(open(path)))
    out = ["# %s" % title, "", "Command (run from /tmp on the MI355X box):", "", "    " + command, "",
           "Durations are rocprofv3's; `per pass` = total / %d passes of the path." % passes, "",
           "| kernel | calls | total ms | avg us | per pass ms | % |", "|---|---:|---:|---:|---:|---:|"]
    for r in rows[:18]:
        out.append("| `%s` | %s | %.3f | %.2f | %.3f | %.2f |" % (
            _short(r["Name"])[:70], r["Calls"], float(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3,
            float(r["TotalDurationNs"]) / 1e6 / passes, float(r["Percentage"])))
    print("\n".join(out))


def _load(path, counter):
    agg = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        k = _short(r["Kernel_Name"])
        a = agg.setdefault(k, [0, 0.0, 0.0, 0.0])
        v = float(r["Counter_Value"])
        a[0] += 1
        a[1] += v
        a[2] += (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6
        a[3] = max(a[3], v)
    return agg


def traffic(fetch_csv, write_csv, workload, command):
    f = _load(fetch_csv, "FETCH_SIZE")
    w = _load(write_csv, "WRITE_SIZE")
    copy = "__amd_rocclr_copyBuffer"
    fscale = GIB_KIB / f[copy][3]      # the 1 GiB copy is the largest copyBuffer dispatch
    wscale = GIB_KIB / w[copy][3]
    print("HBM traffic of the row-solver kernels, workload %s" % workload)
    print("commands (one run per counter, from /tmp on the MI355X box):")
    print("    " + command.replace("<COUNTER>", "FETCH_SIZE"))
    print("    " + command.replace("<COUNTER>", "WRITE_SIZE"))
    print("calibration: the plain 1 GiB copy reads FETCH_SIZE = %.0f KiB, WRITE_SIZE = %.0f KiB" % (f[copy][3], w[copy][3]))
    print("             -> scale factors %.3f (fetch), %.3f (write)" % (fscale, wscale))
    print("%-34s %7s %14s %14s %14s %9s" % ("kernel", "launches", "fetch GB", "write GB", "bytes/launch", "ms total"))
    fam = collections.OrderedDict()
    for k in f:
        family = next((t for t in ("flush_kernel", "panel_kernel", "rows_rank1_kernel") if t in k), None)
        if family is None:
            continue
        fb = f[k][1] * 1024.0 * fscale
        wb = w.get(k, [0, 0.0])[1] * 1024.0 * wscale
        print("%-34s %7d %14.3f %14.3f %14.0f %9.3f" % (k[:34], f[k][0], fb / 1e9, wb / 1e9, (fb + wb) / f[k][0], f[k][2]))
        a = fam.setdefault(family, [0, 0.0, 0.0])
        a[0] += f[k][0]
        a[1] += fb + wb
        a[2] += f[k][2]
    print("per kernel family (all template variants together):")
    for family, a in fam.items():
        print("family %s launches=%d traffic_bytes_per_launch=%.0f hbm_GBps=%.1f" % (
            family, a[0], a[1] / a[0], a[1] / (a[2] * 1e-3) / 1e9))


def counters(title, command, paths):
    per = collections.OrderedDict()          # kernel -> counter -> [n, sum]
    launches = collections.OrderedDict()     # kernel -> (dispatch ids, ms)
    names = []
    for path in paths:
        seen = set()
        for r in csv.DictReader(open(path)):
            k = _short(r["Kernel_Name"])
            c = r["Counter_Name"]
            if c not in names:
                names.append(c)
            a = per.setdefault(k, {}).setdefault(c, [0, 0.0])
            a[0] += 1
            a[1] += float(r["Counter_Value"])
            if path == paths[0] and (k, r["Dispatch_Id"]) not in seen:
                seen.add((k, r["Dispatch_Id"]))
                l = launches.setdefault(k, [0, 0.0])
                l[0] += 1
                l[1] += (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6
    print(title)
    print("commands (one run per counter set, from /tmp on the MI355X box):")
    for c in command.split(" ;; "):
        print("    " + c)
    print("percent-type metrics are averaged over the launches, the others summed; ms is the first run's")
    print("%-40s %8s %9s " % ("kernel", "launches", "ms") + " ".join("%16s" % n[-16:] for n in names))
    for k, cs in per.items():
        if k not in launches:
            continue
        vals = []
        for n in names:
            if n not in cs:
                vals.append("%16s" % "-")
            elif n.endswith(("Util", "Busy", "Stalled")):
                vals.append("%16.2f" % (cs[n][1] / cs[n][0]))
            else:
                vals.append("%16.4g" % cs[n][1])
        print("%-40s %8d %9.3f " % (k[:40], launches[k][0], launches[k][1]) + " ".join(vals))


if __name__ == "__main__":
    if len(sys.argv) >= 6 and sys.argv[1] == "stats":
        stats(sys.argv[2], int(sys.argv[3]), sys.argv[4], sys.argv[5])
    elif len(sys.argv) >= 5 and sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3], sys.argv[4:])
    elif len(sys.argv) >= 6 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5])
    else:
        sys.exit(__doc__)
