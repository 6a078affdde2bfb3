"""Text summary of a rocprofv3 run (its rocpd SQLite database): per-kernel durations and PMC counters.

    rocprofv3 --kernel-trace --stats -d OUT -o run -- python3 bench.py --workload 2 --no-extras --no-cpu
    python -m paper_1811_05213_amd.profile_summary OUT/run_results.db [kernel-name-substring ...]

With --pmc runs the counter table is printed as well (FETCH_SIZE / WRITE_SIZE are KiB per dispatch
as the tool reports them; calibrate against fs_copy_probe_kernel, whose traffic is known).
"""
from __future__ import annotations

import sqlite3
import sys


def summarize(path: str, filters=()) -> str:
    c = sqlite3.connect(path)
    out = []
    where = ""
    args = []
    if filters:
        where = "where " + " or ".join("name like ?" for _ in filters)
        args = [f"%{f}%" for f in filters]
    rows = list(c.execute(
        "select name, count(*), avg(duration)/1000.0, min(duration)/1000.0, max(duration)/1000.0, sum(duration)/1000.0, "
        f"avg(grid_x), avg(workgroup_x), max(static_lds_size), max(scratch_size) from kernels {where} group by name order by 6 desc limit 400", args))
    out.append("%-56s %6s %9s %9s %9s %12s %9s %5s %6s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "total_us", "grid_thr", "wg", "lds", "scratch"))
    for r in rows:
        out.append("%-56s %6d %9.2f %9.2f %9.2f %12.1f %9d %5d %6d %7d" % (r[0][:56], *r[1:]))
    try:
        cw = where.replace("name like", "kernel_name like")
        rows = list(c.execute("select kernel_name, counter_name, count(*), avg(value), min(value), max(value) from counters_collection "
                              f"{cw} group by kernel_name, counter_name order by 1, 2 limit 600", args))
    except sqlite3.Error:
        rows = []
    if rows:
        out.append("")
        out.append("%-56s %-14s %6s %14s %14s %14s" % ("kernel", "counter", "calls", "avg", "min", "max"))
        for r in rows:
            out.append("%-56s %-14s %6d %14.2f %14.2f %14.2f" % (r[0][:56], *r[1:]))
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) < 2:
        print(__doc__)
        sys.exit(1)
    print(summarize(sys.argv[1], sys.argv[2:]))
