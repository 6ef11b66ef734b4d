"""Text summaries of rocprofv3 CSV output for the library's kernels.

    python -m paper_2503_21261_amd.rocprof_summary trace  <..._kernel_trace.csv>
    python -m paper_2503_21261_amd.rocprof_summary counter <..._counter_collection.csv> FETCH_SIZE

Launches are grouped by (kernel, grid size): within one benchmark workload every layer shape
gives a kernel a grid of its own, so a group is one kernel role of one layer shape.  `trace`:
calls, average / min / max duration and share of the total per group, in order of first
launch; kernels that run on a capped grid give every layer shape the same grid, so a group
whose durations (or counter values) spread by more than 2.5x is split in two at the geometric
mean of its extremes ("small" and "large" inputs).  `counter`: the average of one hardware
counter per group, plus the runtime's
device-to-device copy kernel when the profiled command ran one (bench.py --calibrate-copy
copies 154 927 104 bytes), which calibrates the counter's unit.
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def _short(name: str):
    m = re.search(r"hot::(\w+)(<.*>)?", name.replace("(anonymous namespace)::", ""))
    if m:
        args = m.group(2) or ""
        args = re.sub(r"\(hot::\w+\)", "", args)
        return m.group(1) + args
    if "copyBuffer" in name or "direct_copy" in name or "vectorized_elementwise_kernel" in name and "copy" in name.lower():
        return "device_copy"
    return None


def _grid(r) -> str:
    if "Grid_Size_X" in r:
        return f"{r.get('Grid_Size_X', '?')}/{r.get('Workgroup_Size_X', '?')}"
    return f"{r.get('Grid_Size', '?')}/{r.get('Workgroup_Size', '?')}"


def _split(groups):
    """Groups whose values spread widely hold two layer shapes on one (capped) grid: split them."""
    out = collections.OrderedDict()
    for (name, grid), vs in groups.items():
        lo, hi = min(vs), max(vs)
        if lo > 0 and hi / lo > 2.5:
            cut = (lo * hi) ** 0.5
            out[(name, grid + " small")] = [v for v in vs if v < cut]
            out[(name, grid + " large")] = [v for v in vs if v >= cut]
        else:
            out[(name, grid)] = vs
    return out


def trace(path: str) -> str:
    rows = [r for r in csv.DictReader(open(path)) if "hot::" in r["Kernel_Name"]]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    stats = collections.OrderedDict()
    for r in rows:
        stats.setdefault((_short(r["Kernel_Name"]), _grid(r)), []).append(
            int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    stats = _split(stats)
    total = sum(sum(ds) for ds in stats.values())
    out = [f"# {len(rows)} library launches in the trace, {total / 1e6:.3f} ms of kernel time",
           f"{'kernel':72} {'grid/wg':>20} {'calls':>6} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'share':>6}"]
    for (name, grid), ds in stats.items():
        out.append(f"{name[:72]:72} {grid:>20} {len(ds):>6} {sum(ds) / len(ds) / 1e3:10.2f} {min(ds) / 1e3:10.2f} "
                   f"{max(ds) / 1e3:10.2f} {100.0 * sum(ds) / total:5.1f}%")
    return "\n".join(out)


def counter(path: str, which: str) -> str:
    rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == which]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    agg = collections.OrderedDict()
    for r in rows:
        name = _short(r["Kernel_Name"])
        if name:
            key = (name, "" if name == "device_copy" else _grid(r))
            agg.setdefault(key, []).append(float(r["Counter_Value"]))
    out = [f"# {which}: average per launch",
           f"{'kernel':72} {'grid/wg':>20} {'calls':>6} {'avg':>16}"]
    copies = {k: v for k, v in agg.items() if k[0] == "device_copy"}
    agg = _split(collections.OrderedDict((k, v) for k, v in agg.items() if k[0] != "device_copy"))
    agg.update(copies)
    for (name, grid), vs in agg.items():
        # the runtime also copies small buffers: the calibration copy is the largest
        avg = max(vs) if name == "device_copy" else sum(vs) / len(vs)
        out.append(f"{name[:72]:72} {grid:>20} {len(vs):>6} {avg:16.1f}" + (" (largest)" if name == "device_copy" else ""))
    return "\n".join(out)


def main(argv) -> int:
    if len(argv) >= 3 and argv[1] == "trace":
        print(trace(argv[2]))
        return 0
    if len(argv) >= 4 and argv[1] == "counter":
        print(counter(argv[2], argv[3]))
        return 0
    sys.stderr.write(__doc__)
    return 2


if __name__ == "__main__":
    sys.exit(main(sys.argv))
