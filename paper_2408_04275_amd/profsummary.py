"""Turns rocprofv3 CSV output into the short text tables kept under profiles/.

    python -m paper_2408_04275_amd.profsummary trace    <..._kernel_stats.csv>
    python -m paper_2408_04275_amd.profsummary counters <..._counter_collection.csv> [more csv files ...]

`trace` prints one line per kernel of a `rocprofv3 --kernel-trace --stats` run (calls, total ms, average us, share).
`counters` prints, per kernel, the mean value per dispatch of every counter found in the given `rocprofv3 --pmc` runs
(one run per counter group; FETCH_SIZE and WRITE_SIZE are in KiB) and the number of dispatches; bench.py reads the
FETCH_SIZE / WRITE_SIZE table of workload 3 back from profiles/layer_config3_hbm_traffic.txt.
Kernel names are shortened to the function name and its template arguments.
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def short_name(name: str) -> str:
    name = re.sub(r"^void\s+", "", name.strip())
    name = name.replace("(anonymous namespace)::", "").replace("mmt::", "")
    name = re.sub(r"\(.*$", "", name)                       # drop the parameter list
    return name.strip()


def trace(path: str) -> None:
    rows = list(csv.DictReader(open(path)))
    print("%-64s %6s %12s %12s %7s" % ("kernel", "calls", "total_ms", "avg_us", "pct"))
    for r in rows:
        print("%-64s %6d %12.3f %12.1f %7.2f" % (short_name(r["Name"])[:64], int(r["Calls"]), float(r["TotalDurationNs"]) / 1e6,
                                                 float(r["AverageNs"]) / 1e3, float(r["Percentage"])))


def counters(paths) -> None:
    total = collections.defaultdict(lambda: collections.defaultdict(float))
    count = collections.defaultdict(collections.Counter)
    for path in paths:
        for r in csv.DictReader(open(path)):
            k = short_name(r["Kernel_Name"])
            total[k][r["Counter_Name"]] += float(r["Counter_Value"])
            count[k][r["Counter_Name"]] += 1
    names = sorted({c for v in total.values() for c in v})
    print("%-56s" % "kernel" + "".join("%16s" % c for c in names) + "   dispatches")
    order = sorted(total, key=lambda k: -sum(total[k].values()))
    for k in order:
        d = max(count[k].values())
        print("%-56s" % k[:56] + "".join("%16.1f" % (total[k][c] / count[k][c] if count[k][c] else 0.0) for c in names)
              + "   %d" % d)


def main(argv) -> int:
    if len(argv) >= 2 and argv[0] == "trace":
        trace(argv[1])
    elif len(argv) >= 2 and argv[0] == "counters":
        counters(argv[1:])
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
