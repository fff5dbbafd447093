"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2602_02108_amd.profile_summary stats <..._kernel_stats.csv>
  python -m paper_2602_02108_amd.profile_summary pmc <..._counter_collection.csv> <COUNTER> [<COUNTER> ...]

`stats` prints calls / average / total per kernel of this library (and the largest other kernels).
`pmc` prints, per kernel, the per-dispatch mean of each counter over the dispatches recorded.
"""
from __future__ import annotations

import collections
import csv
import sys


def _short(name: str) -> str:
    name = name.split("(")[0]
    return name if len(name) <= 70 else "..." + name[-67:]


def stats(path: str) -> None:
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    print(f"{'kernel':72s} {'calls':>7s} {'avg_us':>10s} {'total_ms':>10s} {'pct':>6s}")
    shown = 0
    for r in rows:
        ours = "oomb::" in r["Name"]
        if not ours and shown >= 6:
            continue
        shown += 0 if ours else 1
        print(f"{_short(r['Name']):72s} {int(r['Calls']):7d} {float(r['AverageNs']) / 1e3:10.1f} "
              f"{float(r['TotalDurationNs']) / 1e6:10.3f} {float(r['Percentage']):6.2f}")


def pmc(path: str, counters: list) -> None:
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] in counters:
            agg[_short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    print(f"{'kernel':72s} " + " ".join(f"{c + ' (mean/dispatch)':>28s}" for c in counters) + f" {'dispatches':>10s}")
    for k, d in sorted(agg.items(), key=lambda kv: -sum(sum(v) for v in kv[1].values())):
        if "oomb::" not in k and "copy" not in k.lower() and "elementwise" not in k.lower():
            continue
        n = max(len(v) for v in d.values())
        print(f"{k:72s} " + " ".join(f"{(sum(d[c]) / len(d[c]) if d[c] else float('nan')):28.1f}" for c in counters) +
              f" {n:10d}")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 4 and sys.argv[1] == "pmc":
        pmc(sys.argv[2], sys.argv[3:])
    else:
        print(__doc__)
        sys.exit(2)
