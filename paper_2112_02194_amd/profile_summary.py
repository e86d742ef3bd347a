"""Short text summary of a rocprofv3 results database (kernel trace and/or PMC counters).

    python -m paper_2112_02194_amd.profile_summary <results.db> [--all]

Prints, for every kernel of this library (every kernel with --all), the number of dispatches and the
total / average / min / max duration, and, when the run collected counters (--pmc), the average and
total of each counter per kernel.  Only sqlite3 from the standard library is used.
"""
from __future__ import annotations

import re
import sqlite3
import sys


def _short(name: str) -> str:
    return re.sub(r"\(.*", "", name).replace("void ", "")[:96]


def summarize(db: str, only_lib: bool = True) -> str:
    con = sqlite3.connect(db)
    tables = {r[0] for r in con.execute("select name from sqlite_master where type in ('table','view')")}
    keep = (lambda n: "als::" in n) if only_lib else (lambda n: True)
    out = []
    if "kernels" in tables:
        rows = con.execute("select name, count(*), sum(end-start)/1e6, avg(end-start)/1e3, min(end-start)/1e3, "
                           "max(end-start)/1e3 from kernels group by name order by 3 desc").fetchall()
        rows = [r for r in rows if keep(r[0])]
        total = sum(r[2] for r in rows) or 1.0
        out.append(f"{'kernel':96s} {'calls':>6} {'total_ms':>10} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'%':>6}")
        for r in rows:
            out.append(f"{_short(r[0]):96s} {r[1]:6d} {r[2]:10.3f} {r[3]:10.1f} {r[4]:10.1f} {r[5]:10.1f} {100 * r[2] / total:6.2f}")
    if "pmc_events" in tables:
        rows = con.execute("select name, counter_name, count(*), avg(counter_value), sum(counter_value), avg(duration)/1e3 "
                           "from pmc_events group by name, counter_name order by 5 desc").fetchall()
        rows = [r for r in rows if keep(r[0])]
        if rows:
            out.append("")
            out.append(f"{'kernel':96s} {'counter':>12} {'calls':>6} {'avg/dispatch':>14} {'total':>16} {'avg_us':>10}")
            for r in rows:
                out.append(f"{_short(r[0]):96s} {r[1]:>12} {r[2]:6d} {r[3]:14.1f} {r[4]:16.1f} {r[5]:10.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) < 2:
        sys.exit(__doc__)
    print(summarize(sys.argv[1], only_lib="--all" not in sys.argv[2:]))
