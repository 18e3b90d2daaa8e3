"""Summarise a rocprofv3 result database (rocpd sqlite) as a few lines of text.

    python -m paper_2506_06295_amd.prof_summary kernels <results.db>   # --kernel-trace runs
    python -m paper_2506_06295_amd.prof_summary pmc <results.db>       # --pmc runs

`kernels` prints calls / total / average / min / max duration per kernel name and launch grid,
the totals per kernel over all grids, then the idle time between consecutive dispatches (end of one kernel to start of the next);
`pmc` prints the number of dispatches and the average counter value per kernel name and grid.
"""
from __future__ import annotations

import sqlite3
import sys


def short(name: str) -> str:
    for s in ("void ", "dllmc::", "(anonymous namespace)::"):
        name = name.replace(s, "")
    return name[:64]


def kernels(db: str) -> None:
    c = sqlite3.connect(db)
    rows = c.execute(
        "select name, grid_x / workgroup_x, grid_y, grid_z, count(*), sum(end - start), "
        "avg(end - start), min(end - start), max(end - start) from kernels "
        "group by name, grid_x, grid_y, grid_z order by 6 desc").fetchall()
    total = sum(r[5] for r in rows) or 1
    print(f"{'kernel':64s} {'grid (workgroups)':>20s} {'calls':>7s} {'total_ms':>10s} {'avg_us':>9s} "
          f"{'min_us':>9s} {'max_us':>9s} {'%':>6s}")
    for r in rows:
        grid = f"({r[1]},{r[2]},{r[3]})"
        print(f"{short(r[0]):64s} {grid:>20s} {r[4]:7d} {r[5] / 1e6:10.2f} {r[6] / 1e3:9.2f} "
              f"{r[7] / 1e3:9.2f} {r[8] / 1e3:9.2f} {100 * r[5] / total:6.2f}")
    print(f"total kernel time {total / 1e6:.2f} ms over {sum(r[4] for r in rows)} dispatches")
    # the same per kernel, all template arguments and grids together
    fam = {}
    for r in rows:
        base = short(r[0]).split("<")[0].split("(")[0]
        n, t = fam.get(base, (0, 0))
        fam[base] = (n + r[4], t + r[5])
    print()
    for base, (n, t) in sorted(fam.items(), key=lambda kv: -kv[1][1])[:8]:
        print(f"{base} over all grids: {n} launches, {t / 1e6:.2f} ms, average {t / n / 1e3:.2f} us per launch")
    # idle time between back-to-back kernels of this library (gaps above 50 us are host pauses
    # between steps or phases of the benchmark, not launch gaps, and are left out)
    ev = c.execute("select start, end, name from kernels order by start").fetchall()
    gaps = sorted((b[0] - a[1]) / 1e3 for a, b in zip(ev, ev[1:])
                  if "dllmc" in a[2] and "dllmc" in b[2] and 0 <= b[0] - a[1] < 50_000)
    if gaps:
        n = len(gaps)
        print(f"gap between consecutive kernels: n {n}, median {gaps[n // 2]:.2f} us, "
              f"mean {sum(gaps) / n:.2f} us, p90 {gaps[(9 * n) // 10]:.2f} us, "
              f"sum {sum(gaps) / 1e3:.2f} ms")


def pmc(db: str) -> None:
    c = sqlite3.connect(db)
    rows = c.execute(
        "select kernel_name, grid_size_x / workgroup_size_x, grid_size_y, grid_size_z, counter_name, "
        "count(*), avg(value), sum(value) from counters_collection "
        "group by kernel_name, grid_size_x, grid_size_y, grid_size_z, counter_name "
        "order by 8 desc").fetchall()
    print(f"{'kernel':64s} {'grid (workgroups)':>20s} {'counter':>12s} {'dispatches':>10s} "
          f"{'avg value':>14s} {'sum':>16s}")
    for r in rows:
        grid = f"({r[1]},{r[2]},{r[3]})"
        print(f"{short(r[0]):64s} {grid:>20s} {r[4]:>12s} {r[5]:10d} {r[6]:14.1f} {r[7]:16.1f}")


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("kernels", "pmc"):
        sys.exit(__doc__)
    {"kernels": kernels, "pmc": pmc}[sys.argv[1]](sys.argv[2])
