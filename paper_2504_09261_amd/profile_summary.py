"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python3 -m paper_2504_09261_amd.profile_summary stats    <..._kernel_stats.csv>
    python3 -m paper_2504_09261_amd.profile_summary counters <..._counter_collection.csv>
            [--calib <copy run's ..._counter_collection.csv> --calib-bytes N --calib-kernel SUBSTR]
            [--trace <the same run's ..._kernel_trace.csv>]

`stats` lists calls / average / min / max duration per kernel.  `counters` lists,
per kernel, the mean of every collected counter per dispatch; with --calib the
same counter's mean over the dispatches of a plain copy kernel that is known to
read and write N bytes gives the bytes-per-count factor that is applied to the
FETCH_SIZE / WRITE_SIZE rows.  With --trace the mean duration of every kernel's
dispatches in the same run is listed too (a counter that ticks once per clock,
divided by that duration, gives the clock the kernel ran at).
"""
from __future__ import annotations

import argparse
import collections
import csv
import re
import sys

csv.field_size_limit(1 << 30)


def _own_mangled(name: str) -> str:
    """The profiler leaves very long names mangled: kernel<int/bool template arguments> of this library's own kernels."""
    m = re.match(r"_ZN4hack\d+_GLOBAL__N_1(\d+)", name)
    if not m:
        return name
    n = int(m.group(1))
    base, rest = name[m.end():m.end() + n], name[m.end() + n:]
    args = []
    if rest.startswith("I"):
        for a in re.finditer(r"L([ib])(\d+)E", rest[1:rest.index("EEE") + 1] if "EEE" in rest else rest):
            args.append(a.group(2) if a.group(1) == "i" else ("true" if a.group(2) == "1" else "false"))
    return base + ("<" + ",".join(args) + ">" if args else "")


def short(name: str) -> str:
    name = _own_mangled(name)
    name = re.sub(r"\(anonymous namespace\)::|hack::|void ", "", name)
    name = re.sub(r"\(.*$", "", name)
    return name[:72]


def stats(path: str) -> None:
    rows = list(csv.DictReader(open(path)))
    print(f"{'kernel':72s} {'calls':>7s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'total_ms':>10s} {'pct':>6s}")
    for r in rows:
        print(f"{short(r['Name']):72s} {int(r['Calls']):7d} {float(r['AverageNs']) / 1e3:10.2f} "
              f"{float(r['MinNs']) / 1e3:10.2f} {float(r['MaxNs']) / 1e3:10.2f} "
              f"{float(r['TotalDurationNs']) / 1e6:10.3f} {float(r['Percentage']):6.2f}")


def counter_means(path: str):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        acc[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return acc


def durations(path: str) -> None:
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        acc[short(r["Kernel_Name"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    print(f"{'kernel':72s} {'dispatches':>10s} {'mean_duration_us':>18s}")
    for kern, v in sorted(acc.items()):
        print(f"{kern:72s} {len(v):10d} {sum(v) / len(v) / 1e3:18.2f}")


def counters(path: str, calib: str | None, calib_bytes: int, calib_kernel: str) -> None:
    factor = {}
    if calib:
        for kern, cs in counter_means(calib).items():
            if calib_kernel in kern:
                for c, v in cs.items():
                    mean = sum(v) / len(v)
                    factor[c] = calib_bytes / mean
                    print(f"calibration: {kern}: {c} mean {mean:.1f} per dispatch for {calib_bytes} bytes"
                          f" -> {factor[c]:.2f} bytes per count")
    print(f"{'kernel':72s} {'counter':24s} {'dispatches':>10s} {'mean/dispatch':>16s} {'bytes/dispatch':>16s}")
    for kern, cs in sorted(counter_means(path).items()):
        for c, v in sorted(cs.items()):
            mean = sum(v) / len(v)
            b = f"{mean * factor[c]:16.0f}" if c in factor else f"{'-':>16s}"
            print(f"{kern:72s} {c:24s} {len(v):10d} {mean:16.1f} {b}")


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["stats", "counters"])
    ap.add_argument("csv")
    ap.add_argument("--calib")
    ap.add_argument("--calib-bytes", type=int, default=0)
    ap.add_argument("--calib-kernel", default="UnaryFunctor")
    ap.add_argument("--trace")
    a = ap.parse_args()
    if a.what == "stats":
        stats(a.csv)
    else:
        counters(a.csv, a.calib, a.calib_bytes, a.calib_kernel)
        if a.trace:
            durations(a.trace)


if __name__ == "__main__":
    sys.exit(main())
