"""Text summaries of rocprofv3 CSV output for the library's kernels.

    python -m paper_2503_21261_amd.rocprof_summary trace  <..._kernel_trace.csv>
    python -m paper_2503_21261_amd.rocprof_summary counter <..._counter_collection.csv> FETCH_SIZE

`trace`: average / min / max duration per kernel role, a role being the kernel's position
within one benchmark step (the launch sequence repeats every step).  `counter`: the same
grouping for one hardware counter, plus the runtime's device-to-device copy kernel when the
profiled command ran one (bench.py --calibrate-copy), which calibrates the counter's unit.
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def _short(name: str):
    m = re.search(r"hot::(\w+)(<[^>]*>)?", name.replace("(anonymous namespace)::", ""))
    if m:
        return m.group(1) + (m.group(2) or "")
    if "copyBuffer" in name or "direct_copy" in name:
        return "device_copy"
    return None


def _period(names):
    for p in range(2, 40):
        if len(names) >= 3 * p and names[:p] == names[p:2 * p] == names[2 * p:3 * p]:
            return p
    return None


def trace(path: str) -> str:
    rows = [r for r in csv.DictReader(open(path)) if "hot::" in r["Kernel_Name"]]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    names = [_short(r["Kernel_Name"]) for r in rows]
    period = _period(names)
    stats = collections.OrderedDict()
    for i, r in enumerate(rows):
        key = (i % period if period else 0, names[i])
        stats.setdefault(key, []).append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    out = [f"# launches per step = {period}; {len(rows)} library launches in the trace",
           f"{'pos':>3} {'kernel':50} {'calls':>5} {'avg_us':>9} {'min_us':>9} {'max_us':>9}  grid/wg"]
    total = 0.0
    for (pos, name), ds in sorted(stats.items()):
        r0 = rows[pos]
        grid = (f"{r0.get('Grid_Size_X', '?')}x{r0.get('Grid_Size_Y', '?')}x{r0.get('Grid_Size_Z', '?')}"
                f"/{r0.get('Workgroup_Size_X', '?')}")
        avg = sum(ds) / len(ds) / 1e3
        total += avg
        out.append(f"{pos:>3} {name:50} {len(ds):>5} {avg:9.2f} {min(ds) / 1e3:9.2f} {max(ds) / 1e3:9.2f}  {grid}")
    out.append(f"sum of averages per step: {total:.1f} us")
    return "\n".join(out)


def counter(path: str, which: str) -> str:
    rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == which]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    seq = [(_short(r["Kernel_Name"]), float(r["Counter_Value"])) for r in rows]
    seq = [x for x in seq if x[0]]
    lib = [x for x in seq if x[0] != "device_copy"]
    period = _period([x[0] for x in lib])
    agg = collections.OrderedDict()
    for i, (n, v) in enumerate(lib):
        agg.setdefault((i % period if period else 0, n), []).append(v)
    out = [f"# {which}: launches per step = {period}"]
    for (pos, n), vs in sorted(agg.items()):
        out.append(f"{pos:>3} {n:50} n={len(vs):3d} avg={sum(vs) / len(vs):14.1f}")
    cp = [v for n, v in seq if n == "device_copy"]
    if cp:
        out.append(f"    device_copy (calibration) n={len(cp)} avg={sum(cp) / len(cp):14.1f}")
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
