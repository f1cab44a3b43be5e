"""Turn the CSV output of `rocprofv3 --kernel-trace --stats --output-format csv` (and of
`rocprofv3 --pmc ... --output-format csv`) into the short text summaries kept under profiles/.

    python -m paper_2310_00837_amd.prof trace  <dir> <prefix>     # per-kernel durations
    python -m paper_2310_00837_amd.prof trace  <dir> <prefix> --by-grid   # ... one line per kernel and grid size
    python -m paper_2310_00837_amd.prof pmc    <dir> <prefix> <COUNTER>   # per-kernel counter sums

Kernels of this library are listed one line per kernel name.  The row-copy kernel's last template
argument names its source (gather_rows_kernel<L, CPL, R, SRC>: SRC 0 = HBM tier or another device
table, 1 = host tier, 2 = storage stand-in); its grid follows the length of the list, so the
workgroup column gives the range seen.  With --by-grid a kernel gets one line per grid size it was
launched with (a recorded batch keeps its grids, so the launches of one mini-batch, of a gang of
several and of the separately launched copies come apart); grid sizes seen fewer than five times go
into one line per kernel.
"""
import collections
import csv
import os
import sys


def _short(name: str) -> str:
    return name.replace("helios::(anonymous namespace)::", "").replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0]


def _ours(name: str) -> bool:
    return "helios" in name or "missq_" in name


def trace(d: str, prefix: str, by_grid: bool = False) -> str:
    rows = list(csv.DictReader(open(os.path.join(d, f"{prefix}_kernel_trace.csv"))))
    agg = collections.OrderedDict()

    def add(key, dur, wg):
        a = agg.setdefault(key, [0, 0, 1 << 62, 0, 1 << 62, 0])
        a[0] += 1
        a[1] += dur
        a[2] = min(a[2], dur)
        a[3] = max(a[3], dur)
        a[4] = min(a[4], wg)
        a[5] = max(a[5], wg)

    seen = collections.Counter()
    if by_grid:
        for r in rows:
            if _ours(r["Kernel_Name"]):
                seen[(_short(r["Kernel_Name"]), int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1))] += 1
    for r in rows:
        if not _ours(r["Kernel_Name"]):
            continue
        key = _short(r["Kernel_Name"])
        wg = int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1)
        dur = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
        if by_grid:
            key = (key, wg if seen[(key, wg)] >= 5 else -1)
        add(key, dur, wg)
    lines = list(agg.items())
    if by_grid:
        lines = [(nm if wg >= 0 else nm + " (other grids)", a)
                 for (nm, wg), a in sorted(agg.items(), key=lambda kv: (kv[0][0], kv[0][1] < 0, kv[0][1]))]
    total = sum(a[1] for a in agg.values()) or 1
    out = [f"{'kernel':44s} {'workgroups':>13s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'share':>6s}"]
    for nm, a in lines:
        wgs = f"{a[4]}" if a[4] == a[5] else f"{a[4]}-{a[5]}"
        out.append(f"{nm:44s} {wgs:>13s} {a[0]:6d} {a[1] / a[0] / 1e3:9.2f} {a[2] / 1e3:9.2f} {a[3] / 1e3:9.2f} "
                   f"{100.0 * a[1] / total:5.1f}%")
    return "\n".join(out)


def pmc(d: str, prefix: str, counter: str) -> str:
    rows = list(csv.DictReader(open(os.path.join(d, f"{prefix}_counter_collection.csv"))))
    agg = collections.OrderedDict()
    for r in rows:
        if r.get("Counter_Name") != counter:
            continue
        name = r["Kernel_Name"]
        if not _ours(name):
            continue
        key = _short(name)
        wg = int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1)
        a = agg.setdefault(key, [0, 0.0, 1 << 62, 0])
        a[0] += 1
        a[1] += float(r["Counter_Value"])
        a[2] = min(a[2], wg)
        a[3] = max(a[3], wg)
    out = [f"{'kernel':44s} {'workgroups':>13s} {'dispatches':>10s} {counter + ' avg/dispatch':>26s}"]
    for nm, a in agg.items():
        wgs = f"{a[2]}" if a[2] == a[3] else f"{a[2]}-{a[3]}"
        out.append(f"{nm:44s} {wgs:>13s} {a[0]:10d} {a[1] / a[0]:26.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "trace":
        print(trace(sys.argv[2], sys.argv[3], by_grid="--by-grid" in sys.argv[4:]))
    elif len(sys.argv) >= 5 and sys.argv[1] == "pmc":
        print(pmc(sys.argv[2], sys.argv[3], sys.argv[4]))
    else:
        print(__doc__)
        sys.exit(2)
