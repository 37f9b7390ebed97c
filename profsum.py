"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

  python profsum.py stats <..._kernel_stats.csv>
      rows of `rocprofv3 --kernel-trace --stats --output-format csv` for this library's kernels
      (and the runtime's copy kernel): calls, average / min / max duration.

  python profsum.py gaps <..._kernel_trace.csv>
      from the per-dispatch begin/end stamps of the same run: for every launch shape of the streaming
      kernel, its mean duration and the mean idle time between the end of the previous dispatch and
      its own begin (only where the previous dispatch is the streaming kernel too, i.e. inside a
      replayed step), and the two sums per step.

  python profsum.py pmc <..._counter_collection.csv> --copy-kib 1048576
      per kernel and launch shape, the mean of the collected counter (FETCH_SIZE or WRITE_SIZE, KiB
      per dispatch), the calibration factor (known KiB of bench.py's plain 1 GiB copy / what the same
      counter shows for it) and the scaled value.
"""
import argparse
import collections
import csv
import re

csv.field_size_limit(1 << 30)


def short(name):
    name = re.sub(r"\(.*$", "", name)
    m = re.match(r"_ZN5itq3s(\d+)", name)  # a name the profiler left mangled
    if m:
        name = name[len(m.group(0)) : len(m.group(0)) + int(m.group(1))]
    return name.replace("void ", "").replace("itq3s::", "")


def ours(name):
    return "itq3s" in name or "copyBuffer" in name


def stats(path):
    print("%-44s %7s %12s %10s %10s" % ("kernel", "calls", "avg_ns", "min_ns", "max_ns"))
    for r in csv.DictReader(open(path)):
        if ours(r["Name"]):
            print("%-44s %7d %12.1f %10d %10d" % (short(r["Name"])[:44], int(r["Calls"]), float(r["AverageNs"]), int(r["MinNs"]), int(r["MaxNs"])))


def gaps(path):
    rows = []
    for r in csv.DictReader(open(path)):
        rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), short(r["Kernel_Name"]), int(r.get("Grid_Size", r.get("Grid_Size_X", 0)) or 0)))
    rows.sort()
    # A dispatch counts as "inside a replayed step" if the dispatch before it is the streaming kernel
    # too and ended less than 5 us earlier; launches of one template and grid that follow different
    # launches (o after q+k+v, down after gate+up) are different shapes and are listed apart.
    agg = collections.defaultdict(lambda: [0, 0.0, 0.0])  # calls, duration, gap
    alone = collections.defaultdict(lambda: [0, 0.0])
    prev = None
    for st, en, name, grid in rows:
        if "gemv_kernel" in name:
            if prev is not None and "gemv_kernel" in prev[2] and 0 <= st - prev[1] < 5000:
                a = agg[(name, grid, prev[2], prev[3])]
                a[0] += 1
                a[1] += en - st
                a[2] += st - prev[1]
            else:
                alone[(name, grid)][0] += 1
                alone[(name, grid)][1] += en - st
        prev = (st, en, name, grid)
    print("%-30s %8s  %-30s %8s %7s %11s %11s" % ("kernel", "threads", "follows", "threads", "calls", "avg_ns", "avg_gap_ns"))
    tot_d = tot_g = 0.0
    for (name, grid, pname, pgrid), (calls, dur, gap) in sorted(agg.items()):
        if calls < 8:
            continue
        print("%-30s %8d  %-30s %8d %7d %11.1f %11.1f" % (name[:30], grid, pname[:30], pgrid, calls, dur / calls, gap / calls))
        tot_d += dur / calls
        tot_g += gap / calls
    print("one launch of each shape inside a replayed step: %.1f ns of kernel time + %.1f ns idle in front of them" % (tot_d, tot_g))
    for (name, grid), (calls, dur) in sorted(alone.items()):
        print("launched on its own (the timed passes: the host waits for every kernel): %-30s %8d %7d calls avg %.1f ns" % (name[:30], grid, calls, dur / calls))


def pmc(path, copy_kib):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if ours(r["Kernel_Name"]):
            agg[(short(r["Kernel_Name"]), int(r["Grid_Size"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    big = [(sum(v) / len(v), k) for k, v in agg.items() if "copyBuffer" in k[0]]
    factor = None
    if big and copy_kib:
        measured = max(big)[0]
        factor = copy_kib / measured if measured > 0 else None
    print("calibration: plain copy of %s KiB shows %s -> factor %s" % (copy_kib, ("%.1f" % max(big)[0]) if big else "n/a", ("%.4f" % factor) if factor else "n/a"))
    print("%-36s %9s %-11s %7s %14s %14s" % ("kernel", "threads", "counter", "calls", "mean_KiB", "scaled_KiB"))
    for (name, grid, ctr), v in sorted(agg.items()):
        mean = sum(v) / len(v)
        print("%-36s %9d %-11s %7d %14.1f %14s" % (name[:36], grid, ctr, len(v), mean, ("%.1f" % (mean * factor)) if factor else "n/a"))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("mode", choices=["stats", "gaps", "pmc"])
    ap.add_argument("csv")
    ap.add_argument("--copy-kib", type=float, default=0.0, help="known KiB the calibration copy reads (= writes)")
    a = ap.parse_args()
    if a.mode == "stats":
        stats(a.csv)
    elif a.mode == "gaps":
        gaps(a.csv)
    else:
        pmc(a.csv, a.copy_kib)


if __name__ == "__main__":
    main()
