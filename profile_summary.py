#!/usr/bin/env python3
"""Condenses rocprofv3 output (the results database of one run) into the short text summaries kept under profiles/.

    python profile_summary.py trace <results.db> <out.txt> "<the rocprofv3 command that made it>"
        per kernel name, and per (kernel, launch shape): calls, total / average / minimum / maximum duration
    python profile_summary.py pmc <results.db> [<results.db> ...]
        per kernel name and counter: dispatches and the average counter value per dispatch (prints to stdout)

Both read the tables rocprofv3 writes (kernel dispatches with start / end time stamps, counter samples per
dispatch); table names carry a per-run suffix, so they are looked up by prefix.
"""
import re
import sqlite3
import sys


def _table(c, prefix):
    names = [r[0] for r in c.execute("select name from sqlite_master where type in ('table', 'view')")]
    exact = [n for n in names if n == prefix]
    if exact:
        return exact[0]
    cand = [n for n in names if n.startswith(prefix)]
    if not cand:
        raise SystemExit("no table %s* in the database (have: %s)" % (prefix, ", ".join(sorted(names))))
    return cand[0]


def _short(n):
    n = re.sub(r"\(.*", "", n).replace("lpm::", "").replace("void ", "")
    return n[:64]


def trace(db, out, cmd):
    c = sqlite3.connect(db)
    k = _table(c, "kernels")
    rows = c.execute("select name, grid_x, grid_y, grid_z, count(*), sum(duration), avg(duration), min(duration), max(duration) "
                     "from %s group by name, grid_x, grid_y, grid_z order by sum(duration) desc" % k).fetchall()
    tot = sum(r[5] for r in rows)
    byname = {}
    for r in rows:
        e = byname.setdefault(_short(r[0]), [0, 0])
        e[0] += r[4]
        e[1] += r[5]
    with open(out, "w") as f:
        f.write("rocprofv3 kernel trace summary\ncommand: %s\n" % cmd)
        f.write("durations in microseconds; grid = threads per dimension; one line per (kernel, launch shape)\n\n")
        f.write("by kernel name\n%-66s %8s %12s %9s %6s\n" % ("kernel", "calls", "total_us", "avg_us", "%"))
        for name, (n, t) in sorted(byname.items(), key=lambda kv: -kv[1][1]):
            f.write("%-66s %8d %12.1f %9.2f %6.2f\n" % (name, n, t / 1e3, t / 1e3 / n, 100 * t / tot))
        f.write("total kernel time %.1f us\n\nby kernel and launch shape (top 40)\n" % (tot / 1e3))
        f.write("%-66s %-18s %7s %11s %9s %9s %9s\n" % ("kernel", "grid", "calls", "total_us", "avg_us", "min_us", "max_us"))
        for r in rows[:40]:
            f.write("%-66s %-18s %7d %11.1f %9.2f %9.2f %9.2f\n" % (_short(r[0]), "%dx%dx%d" % (r[1], r[2], r[3]), r[4], r[5] / 1e3,
                                                                 r[6] / 1e3, r[7] / 1e3, r[8] / 1e3))


def pmc(dbs):
    """Per kernel name, launch size (work-items) and counter: dispatches and the average value per dispatch."""
    for db in dbs:
        c = sqlite3.connect(db)
        view = _table(c, "counters_collection")
        cols = [r[1] for r in c.execute("pragma table_info(%s)" % view)]
        size = "grid_size" if "grid_size" in cols else "0"
        rows = c.execute("select kernel_name, %s, counter_name, count(*), avg(value) from %s group by kernel_name, %s, counter_name"
                         % (size, view, size)).fetchall()
        for name, threads, counter, n, v in rows:
            s = _short(name)
            if "at::" in s:
                continue
            print("%-56s work-items=%-10d %-30s n=%5d avg=%.1f" % (s, threads or 0, counter, n, v))


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "trace":
        trace(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) >= 3 and sys.argv[1] == "pmc":
        pmc(sys.argv[2:])
    else:
        raise SystemExit(__doc__)
