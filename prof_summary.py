"""Condense rocprofv3 CSV output into the short text tables kept under profiles/.

    python prof_summary.py trace  <dir>/p_kernel_trace.csv
    python prof_summary.py pmc    <dir>/p_counter_collection.csv [...]

`trace` prints calls / average / min / max duration per (kernel, number of workgroups); `pmc` prints the
average counter value per dispatch for the same grouping.  Reads files only; runs nothing on the GPU.
"""
import collections
import csv
import sys


def _short(name: str) -> str:
    name = name.replace("void ", "").replace("ssv::", "")
    return name.split("(")[0][:64]


def trace(path: str) -> None:
    agg = collections.OrderedDict()
    with open(path) as f:
        for row in csv.DictReader(f):
            wgs = int(row["Grid_Size_X"] if "Grid_Size_X" in row else row["Grid_Size"]) // \
                max(1, int(row["Workgroup_Size_X"] if "Workgroup_Size_X" in row else row["Workgroup_Size"]))
            dur = int(row["End_Timestamp"]) - int(row["Start_Timestamp"])
            a = agg.setdefault((_short(row["Kernel_Name"]), wgs), [0, 0, 1 << 62, 0])
            a[0] += 1
            a[1] += dur
            a[2] = min(a[2], dur)
            a[3] = max(a[3], dur)
    total = sum(a[1] for a in agg.values()) or 1
    print(f"{'kernel':66s} {'wgs':>6s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'share%':>7s}")
    for (name, wgs), a in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        if a[1] * 1000 < total:
            continue
        print(f"{name:66s} {wgs:6d} {a[0]:6d} {a[1] / a[0] / 1e3:9.2f} {a[2] / 1e3:9.2f} {a[3] / 1e3:9.2f} {100.0 * a[1] / total:7.1f}")


def pmc(paths) -> None:
    agg = collections.OrderedDict()
    for path in paths:
        with open(path) as f:
            for row in csv.DictReader(f):
                wgs = int(row["Grid_Size"]) // max(1, int(row["Workgroup_Size"]))
                agg.setdefault((_short(row["Kernel_Name"]), wgs), collections.OrderedDict()) \
                   .setdefault(row["Counter_Name"], []).append(float(row["Counter_Value"]))
    for (name, wgs), counters in agg.items():
        if not any(max(v) > 0 for v in counters.values()):
            continue
        print(f"{name}  wgs={wgs}")
        for cname, v in counters.items():
            print(f"    {cname:28s} dispatches={len(v):5d}  avg={sum(v) / len(v):16.1f}")


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("trace", "pmc"):
        print(__doc__)
        sys.exit(2)
    if sys.argv[1] == "trace":
        trace(sys.argv[2])
    else:
        pmc(sys.argv[2:])
