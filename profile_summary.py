#!/usr/bin/env python3
"""Short text summaries of rocprofv3 results databases for this library's kernels.

    python profile_summary.py trace <results.db> [--all]
        per kernel: dispatches, total / average / min / max duration
    python profile_summary.py counters <results.db> [--all]
        per kernel and counter of a --pmc run: dispatches, average per dispatch, total
    python profile_summary.py mfma <results.db>
        matrix-core busy share per kernel from a run with --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA
        GRBM_GUI_ACTIVE (...): busy cycles summed over the chip / (GRBM_GUI_ACTIVE summed over the 8 XCDs x 128
        SIMDs per XCD), i.e. the share of all SIMD cycles in which a matrix instruction executes
    python profile_summary.py traffic <workload> <fetch.db> <write.db> [--json FILE]
        HBM bytes per launch of every kernel from a FETCH_SIZE run and a WRITE_SIZE run, each counter scaled
        by what it reads for the library's plain copy kernel (als::copy_probe_kernel, which both runs must
        contain: bench.py --copy-probe-mib N moves N MiB in and N MiB out); with --json the figures are
        merged into FILE under the workload's key (bench.py reads profiles/hbm_traffic.json)

Only sqlite3 from the standard library is used.
"""
from __future__ import annotations

import json
import os
import re
import sqlite3
import sys


def short_name(name: str) -> str:
    """'void als::k<1, 2>(args)' -> 'k<1,2>'"""
    name = re.sub(r"\(.*", "", name).replace("void ", "").replace("als::", "")
    return name.replace(" ", "")


def _tables(con):
    return {r[0] for r in con.execute("select name from sqlite_master where type in ('table','view')")}


def trace(db: str, only_lib: bool = True) -> str:
    con = sqlite3.connect(db)
    if "kernels" not in _tables(con):
        return "no kernel trace in " + db
    rows = con.execute("select name, count(*), sum(end-start)/1e6, avg(end-start)/1e3, min(end-start)/1e3, "
                       "max(end-start)/1e3 from kernels group by name order by 3 desc").fetchall()
    rows = [r for r in rows if not only_lib or "als::" in r[0]]
    total = sum(r[2] for r in rows) or 1.0
    out = [f"{'kernel':64s} {'calls':>6} {'total_ms':>10} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'%':>6}"]
    for r in rows:
        out.append(f"{short_name(r[0])[:64]:64s} {r[1]:6d} {r[2]:10.3f} {r[3]:10.1f} {r[4]:10.1f} {r[5]:10.1f} {100 * r[2] / total:6.2f}")
    return "\n".join(out)


def _counter_rows(db: str, only_lib: bool = True):
    con = sqlite3.connect(db)
    if "pmc_events" not in _tables(con):
        return []
    rows = con.execute("select name, counter_name, count(*), avg(counter_value), sum(counter_value), avg(duration)/1e3 "
                       "from pmc_events group by name, counter_name order by 5 desc").fetchall()
    return [r for r in rows if not only_lib or "als::" in r[0]]


def counters(db: str, only_lib: bool = True) -> str:
    out = [f"{'kernel':64s} {'counter':>28} {'calls':>6} {'avg/dispatch':>16} {'total':>18} {'avg_us':>10}"]
    for r in _counter_rows(db, only_lib):
        out.append(f"{short_name(r[0])[:64]:64s} {r[1]:>28} {r[2]:6d} {r[3]:16.1f} {r[4]:18.1f} {r[5]:10.1f}")
    return "\n".join(out)


def mfma(db: str) -> str:
    rows = {}
    for name, counter, calls, _avg, total, us in _counter_rows(db):
        rows.setdefault(short_name(name), {})[counter] = (calls, total, us)
    out = [f"{'kernel':64s} {'dispatches':>10} {'avg_us':>10} {'MFMA instr/disp':>16} {'MFMA busy % of SIMD cycles':>28}"]
    order = sorted(rows, key=lambda n: -rows[n].get("SQ_VALU_MFMA_BUSY_CYCLES", (0, 0, 0))[1])
    for name in order:
        c = rows[name]
        if "GRBM_GUI_ACTIVE" not in c or "SQ_VALU_MFMA_BUSY_CYCLES" not in c:
            continue
        disp = max(1, c["GRBM_GUI_ACTIVE"][0] // 8)  # one GRBM sample per XCD and dispatch
        busy = 100.0 * c["SQ_VALU_MFMA_BUSY_CYCLES"][1] / (c["GRBM_GUI_ACTIVE"][1] * 128.0)
        insts = c.get("SQ_INSTS_MFMA", (0, 0.0, 0))[1] / disp
        out.append(f"{name[:64]:64s} {disp:10d} {c['GRBM_GUI_ACTIVE'][2]:10.1f} {insts:16.3e} {busy:28.1f}")
    return "\n".join(out)


def traffic(workload: str, fetch_db: str, write_db: str, json_path: str | None = None) -> str:
    fetch = {short_name(r[0]): r for r in _counter_rows(fetch_db) if r[1] == "FETCH_SIZE"}
    write = {short_name(r[0]): r for r in _counter_rows(write_db) if r[1] == "WRITE_SIZE"}
    probe = "copy_probe_kernel"
    if probe not in fetch or probe not in write:
        return "both runs must contain als::copy_probe_kernel (bench.py --copy-probe-mib N)"
    # the probe's size in KiB per direction is not stored in the database: both counters are in KiB, and the
    # write counter reads the true size on every machine seen so far, so it calibrates itself and the fetch side
    probe_kib = write[probe][3]
    scale_f, scale_w = probe_kib / fetch[probe][3], 1.0
    out = [f"copy probe: WRITE_SIZE {write[probe][3]:.0f} KiB, FETCH_SIZE {fetch[probe][3]:.0f} KiB per dispatch "
           f"-> fetched bytes = {scale_f:.3f} x FETCH_SIZE KiB, written bytes = {scale_w:.3f} x WRITE_SIZE KiB",
           f"{'kernel':64s} {'calls':>6} {'fetch_GB':>10} {'write_GB':>10} {'total_GB':>10} {'avg_us':>10} {'TB/s':>7}"]
    entries = []
    for name in sorted(set(fetch) | set(write), key=lambda n: -(fetch.get(n, (0,) * 6)[4] + write.get(n, (0,) * 6)[4])):
        f, w = fetch.get(name), write.get(name)
        fb = (f[3] * scale_f * 1024) if f else 0.0
        wb = (w[3] * scale_w * 1024) if w else 0.0
        calls = (f or w)[2]
        us = (f or w)[5]
        out.append(f"{name[:64]:64s} {calls:6d} {fb / 1e9:10.3f} {wb / 1e9:10.3f} {(fb + wb) / 1e9:10.3f} {us:10.1f} "
                   f"{(fb + wb) / (us * 1e-6) / 1e12 if us else 0:7.2f}")
        entries.append({"kernel": name, "calls": calls, "fetch_bytes_per_launch": fb, "write_bytes_per_launch": wb,
                        "bytes_per_launch": fb + wb})
    if json_path:
        table = {}
        if os.path.exists(json_path):
            with open(json_path) as fh:
                table = json.load(fh)
        table[workload] = entries
        with open(json_path, "w") as fh:
            json.dump(table, fh, indent=1, sort_keys=True)
    return "\n".join(out)


if __name__ == "__main__":
    a = sys.argv[1:]
    only_lib = "--all" not in a
    a = [x for x in a if x != "--all"]
    if len(a) >= 2 and a[0] == "trace":
        print(trace(a[1], only_lib))
    elif len(a) >= 2 and a[0] == "counters":
        print(counters(a[1], only_lib))
    elif len(a) >= 2 and a[0] == "mfma":
        print(mfma(a[1]))
    elif len(a) >= 4 and a[0] == "traffic":
        jp = a[a.index("--json") + 1] if "--json" in a else None
        print(traffic(a[1], a[2], a[3], jp))
    else:
        sys.exit(__doc__)
