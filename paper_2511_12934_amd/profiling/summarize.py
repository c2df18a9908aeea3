"""Turn a rocprofv3 result database (``*_results.db``, the default rocpd output
of ``rocprofv3 --kernel-trace --stats``) into a short text table of per-kernel
durations, and a ``--pmc`` database into per-kernel counter averages.

    python -m paper_2511_12934_amd.profiling.summarize prof/c3_results.db [--pmc]
"""
from __future__ import annotations

import sqlite3
import sys


def kernel_table(path: str) -> str:
    db = sqlite3.connect(path)
    rows = list(db.execute(
        "select name, count(*), avg(end - start), min(end - start), max(end - start), sum(end - start) "
        "from kernels group by name order by 6 desc"))
    total = sum(r[5] for r in rows) or 1
    out = [f"{'kernel':72s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'share':>7s}"]
    for name, n, avg, mn, mx, tot in rows:
        out.append(f"{name[:72]:72s} {n:6d} {avg / 1e3:10.1f} {mn / 1e3:10.1f} {mx / 1e3:10.1f} {100 * tot / total:6.1f}%")
    return "\n".join(out)


def pmc_table(path: str) -> str:
    db = sqlite3.connect(path)
    tabs = [r[0] for r in db.execute("select name from sqlite_master where type in ('table','view')")]
    view = "counters_collection" if "counters_collection" in tabs else None
    if view is None:
        return "no counters_collection view in " + path
    cols = [d[1] for d in db.execute(f"pragma table_info({view})")]
    name_col = "kernel_name" if "kernel_name" in cols else "name"
    rows = list(db.execute(
        f"select {name_col}, counter_name, count(*), avg(value) from {view} group by 1, 2 order by 1, 2"))
    out = [f"{'kernel':72s} {'counter':>16s} {'dispatches':>10s} {'avg':>16s}"]
    for k, c, n, v in rows:
        out.append(f"{k[:72]:72s} {c:>16s} {n:10d} {v:16.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    p = sys.argv[1]
    print(pmc_table(p) if "--pmc" in sys.argv else kernel_table(p))
