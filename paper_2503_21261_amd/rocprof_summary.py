"""Text summaries of rocprofv3 CSV output for the library's kernels.

    python -m paper_2503_21261_amd.rocprof_summary trace   <..._kernel_trace.csv> [bench.json]
    python -m paper_2503_21261_amd.rocprof_summary counter <..._counter_collection.csv> FETCH_SIZE [bench.json]

With the JSON line that bench.py printed in the profiled run, every launch is labelled
"<layer>.<role>": bench.py records the order of the library's launches within one step
("launch_sequence"), every step of a run repeats it, so a launch's position in the periodic
part of the trace names it.  Without the JSON, launches are grouped by (kernel, grid size).
`trace`: calls, average / min / max duration and share of the total per group.  `counter`: the
average of one hardware counter per group, plus the runtime's device-to-device copy kernel when
the profiled command ran one (bench.py --calibrate-copy copies 154 927 104 bytes; the largest
copy in the run is reported), which calibrates the counter's unit.
"""
from __future__ import annotations

import collections
import csv
import json
import re
import sys


def _short(name: str):
    m = re.search(r"hot::(\w+)(<.*>)?", name.replace("(anonymous namespace)::", ""))
    if m:
        args = m.group(2) or ""
        args = re.sub(r"\(hot::\w+\)", "", args)
        return m.group(1) + args
    if "copyBuffer" in name or "direct_copy" in name:
        return "device_copy"
    return None


def _grid(r) -> str:
    if "Grid_Size_X" in r:
        return f"{r.get('Grid_Size_X', '?')}/{r.get('Workgroup_Size_X', '?')}"
    return f"{r.get('Grid_Size', '?')}/{r.get('Workgroup_Size', '?')}"


def _labels(names, bench_json):
    """Label of every launch (None before the periodic part of the run starts)."""
    if not bench_json:
        return None
    seq = json.load(open(bench_json))["launch_sequence"]
    P = len(seq)
    if P == 0 or len(names) < 2 * P:
        return None
    # the periodic tail: the longest suffix with names[i] == names[i + P], cut to whole steps
    start = len(names) - P
    while start > 0 and names[start - 1] == names[start - 1 + P]:
        start -= 1
    start += (len(names) - start) % P
    return [None if i < start else seq[(i - start) % P] for i in range(len(names))]


def _group(rows, names, value, bench_json):
    labels = _labels(names, bench_json)
    groups = collections.OrderedDict()
    skipped = 0
    for i, r in enumerate(rows):
        if labels is not None and labels[i] is None:
            skipped += 1
            continue
        key = (labels[i] if labels is not None else "", names[i], _grid(r))
        groups.setdefault(key, []).append(value(r))
    return groups, skipped


def trace(path: str, bench_json=None) -> str:
    rows = [r for r in csv.DictReader(open(path)) if "hot::" in r["Kernel_Name"]]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    names = [_short(r["Kernel_Name"]) for r in rows]
    stats, skipped = _group(rows, names, lambda r: int(r["End_Timestamp"]) - int(r["Start_Timestamp"]), bench_json)
    total = sum(sum(ds) for ds in stats.values())
    out = [f"# {len(rows)} library launches in the trace ({skipped} before the repeating steps, not listed), "
           f"{total / 1e6:.3f} ms of kernel time listed",
           f"{'layer.role':28} {'kernel':64} {'grid/wg':>14} {'calls':>6} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'share':>6}"]
    for (label, name, grid), ds in stats.items():
        out.append(f"{label:28} {name[:64]:64} {grid:>14} {len(ds):>6} {sum(ds) / len(ds) / 1e3:10.2f} "
                   f"{min(ds) / 1e3:10.2f} {max(ds) / 1e3:10.2f} {100.0 * sum(ds) / total:5.1f}%")
    return "\n".join(out)


def counter(path: str, which: str, bench_json=None) -> str:
    rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == which]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    lib = [r for r in rows if "hot::" in r["Kernel_Name"]]
    names = [_short(r["Kernel_Name"]) for r in lib]
    agg, skipped = _group(lib, names, lambda r: float(r["Counter_Value"]), bench_json)
    out = [f"# {which}: average per launch ({skipped} launches before the repeating steps not listed)",
           f"{'layer.role':28} {'kernel':64} {'grid/wg':>14} {'calls':>6} {'avg':>16}"]
    for (label, name, grid), vs in agg.items():
        out.append(f"{label:28} {name[:64]:64} {grid:>14} {len(vs):>6} {sum(vs) / len(vs):16.1f}")
    copies = [float(r["Counter_Value"]) for r in rows if _short(r["Kernel_Name"]) == "device_copy"]
    if copies:
        out.append(f"{'':28} {'device_copy (largest of the run)':64} {'':>14} {len(copies):>6} {max(copies):16.1f}")
    return "\n".join(out)


def main(argv) -> int:
    if len(argv) >= 3 and argv[1] == "trace":
        print(trace(argv[2], argv[3] if len(argv) > 3 else None))
        return 0
    if len(argv) >= 4 and argv[1] == "counter":
        print(counter(argv[2], argv[3], argv[4] if len(argv) > 4 else None))
        return 0
    sys.stderr.write(__doc__)
    return 2


if __name__ == "__main__":
    sys.exit(main(sys.argv))
