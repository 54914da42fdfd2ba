#!/usr/bin/env python3
"""Tabulates a rocprofv3 output database (rocpd, `*_results.db`) as the text kept under profiles/.

    python -m paper_2102_08124_amd.profile_summary kernels <results.db> [name-filter]
        per kernel: calls, average / minimum / maximum duration in microseconds, share of the traced time
    python -m paper_2102_08124_amd.profile_summary pmc <results.db> [name-filter]
        per kernel and counter: dispatches, average / minimum / maximum counter value

Reads the database with sqlite3 only (views `kernels` and `counters_collection` that rocprofv3 creates); runs on any
machine, no GPU needed.  A measuring aid: nothing in the library or the tests depends on it.
"""
from __future__ import annotations

import re
import sqlite3
import sys


def short(name: str, width: int) -> str:
    return re.sub(r"\(.*", "", name)[:width]


def kernels(db_path: str, flt: str = "") -> str:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                       "from kernels group by name order by sum(end-start) desc").fetchall()
    total = sum(r[5] for r in rows) or 1
    out = ["%-92s %7s %10s %10s %10s %6s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "%")]
    for n, c, a, mn, mx, s in rows:
        if flt and flt not in n:
            continue
        out.append("%-92s %7d %10.2f %10.2f %10.2f %6.1f" % (short(n, 92), c, a / 1e3, mn / 1e3, mx / 1e3, 100.0 * s / total))
    return "\n".join(out)


def pmc(db_path: str, flt: str = "") -> str:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select kernel_name, counter_name, count(*), avg(value), min(value), max(value) "
                       "from counters_collection group by kernel_name, counter_name order by kernel_name, counter_name").fetchall()
    out = ["%-80s %-18s %6s %16s %16s %16s" % ("kernel", "counter", "n", "avg", "min", "max")]
    for n, c, k, a, mn, mx in rows:
        if flt and flt not in n:
            continue
        out.append("%-80s %-18s %6d %16.1f %16.1f %16.1f" % (short(n, 80), c, k, a, mn, mx))
    return "\n".join(out)


def main():
    if len(sys.argv) < 3 or sys.argv[1] not in ("kernels", "pmc"):
        print(__doc__)
        sys.exit(2)
    flt = sys.argv[3] if len(sys.argv) > 3 else ""
    print(kernels(sys.argv[2], flt) if sys.argv[1] == "kernels" else pmc(sys.argv[2], flt))


if __name__ == "__main__":
    main()
