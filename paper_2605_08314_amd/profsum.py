"""Print a per-kernel summary (count, average / min / max duration, total) of a rocprofv3 run.

rocprofv3 on ROCm 7.2 writes its kernel trace as a rocpd SQLite database; this reads its `kernels`
view.  Usage: python -m paper_2605_08314_amd.profsum <dir-or-db> [name-filter]
With --pmc it sums the counters of a `--pmc ... --output-format csv` run per kernel name instead:
       python -m paper_2605_08314_amd.profsum --pmc <dir> [name-filter]
"""
from __future__ import annotations

import glob
import os
import sqlite3
import sys


def summarize(path: str, name_filter: str = "") -> str:
    dbs = [path] if path.endswith(".db") else sorted(glob.glob(os.path.join(path, "**", "*_results.db"), recursive=True))
    lines = []
    for dbp in dbs:
        cur = sqlite3.connect(dbp).cursor()
        rows = list(cur.execute(
            "select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
            "from kernels group by name order by sum(end-start) desc"))
        total = sum(r[5] for r in rows) or 1
        lines.append(f"# {os.path.basename(dbp)}: {sum(r[1] for r in rows)} dispatches, {total / 1e6:.3f} ms of kernel time")
        lines.append(f"{'calls':>7} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'total_ms':>10} {'pct':>6}  kernel")
        for name, n, avg, mn, mx, tot in rows:
            if name_filter and name_filter not in name:
                continue
            lines.append(f"{n:7d} {avg / 1e3:10.2f} {mn / 1e3:10.2f} {mx / 1e3:10.2f} {tot / 1e6:10.3f} {100 * tot / total:6.2f}  {name[:140]}")
    return "\n".join(lines)


def summarize_pmc(path: str, name_filter: str = "") -> str:
    """Per kernel name: dispatches and, for every counter, its mean per dispatch (counter values of one dispatch
    are the sums over the whole device that rocprofv3 reports)."""
    import collections
    import csv
    files = sorted(glob.glob(os.path.join(path, "**", "*counter_collection.csv"), recursive=True))
    lines = []
    for f in files:
        agg = collections.defaultdict(lambda: collections.defaultdict(float))
        disp = collections.defaultdict(set)
        for r in csv.DictReader(open(f)):
            k = r["Kernel_Name"]
            if name_filter and name_filter not in k:
                continue
            agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
            disp[k].add(r["Dispatch_Id"])
        lines.append(f"# {os.path.relpath(f, path)}")
        for k in sorted(agg):
            n = max(len(disp[k]), 1)
            lines.append(f"{k[:120]}  ({n} dispatches; mean per dispatch)")
            for c, x in sorted(agg[k].items()):
                lines.append(f"    {c:32s} {x / n:16.6g}")
    return "\n".join(lines)


if __name__ == "__main__":
    if sys.argv[1] == "--pmc":
        print(summarize_pmc(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else ""))
    else:
        print(summarize(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else ""))
