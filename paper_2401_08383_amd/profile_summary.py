"""Prints a short text summary (per-kernel calls / total / average duration, and counter sums if
any were collected) of a rocprofv3 results database.

Usage: python -m paper_2401_08383_amd.profile_summary <results.db> [more.db ...]
"""
from __future__ import annotations

import sqlite3
import sys


def summarize(path: str) -> str:
    db = sqlite3.connect(path)
    cur = db.cursor()
    lines = [f"# {path}"]
    try:
        rows = list(cur.execute("select name, total_calls, total_duration, average, percentage from top_kernels"))
    except sqlite3.Error:
        rows = []
    if rows:
        lines.append(f"{'calls':>7} {'total_us':>12} {'avg_us':>10} {'pct':>6}  kernel")
        for name, calls, total, avg, pct in rows:
            lines.append(f"{calls:>7} {total:>12.1f} {avg:>10.3f} {pct:>6.2f}  {name}")
    try:
        q = ("select k.kernel_name, p.counter_name, count(*), avg(p.value), sum(p.value) "
             "from counters_collection p join kernel_symbols k on p.kernel_id = k.id "
             "group by k.kernel_name, p.counter_name")
        rows = list(cur.execute(q))
    except sqlite3.Error:
        rows = []
        try:
            cols = [d[0] for d in cur.execute("select * from counters_collection limit 1").description]
            lines.append("counters_collection columns: " + ", ".join(cols))
        except sqlite3.Error:
            pass
    if rows:
        lines.append(f"{'dispatches':>10} {'avg':>16} {'sum':>18}  counter  kernel")
        for kname, cname, n, avg, total in rows:
            lines.append(f"{n:>10} {avg:>16.1f} {total:>18.1f}  {cname}  {kname}")
    return "\n".join(lines)


if __name__ == "__main__":
    for p in sys.argv[1:]:
        print(summarize(p))
