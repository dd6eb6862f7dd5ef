"""Text summaries of rocprofv3 output databases (rocpd SQLite): per-kernel durations from a
--kernel-trace run, per-kernel counter averages from a --pmc run.

    python -m paper_2511_13587_amd.profsum kernels <results.db>
    python -m paper_2511_13587_amd.profsum counters <results.db>
"""
import re
import sqlite3
import sys


def short(name: str) -> str:
    return re.sub(r"\(.*", "", name).replace("void ", "")


def kernels(db: str, top: int = 30) -> str:
    cur = sqlite3.connect(db).cursor()
    rows = cur.execute("select name, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start) "
                       "from kernels group by name order by 3 desc").fetchall()
    total = sum(r[2] for r in rows) or 1
    out = [f"{'kernel':64s} {'calls':>7s} {'total_ms':>10s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}"]
    for n, c, s, a, mn, mx in rows[:top]:
        out.append(f"{short(n)[:64]:64s} {c:7d} {s / 1e6:10.3f} {a / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {100 * s / total:6.2f}")
    out.append("")
    out.append("per launch shape (grid in workgroups) of the hot kernels:")
    rows = cur.execute("select name, grid_x / workgroup_x, grid_y / workgroup_y, grid_z / workgroup_z, count(*), avg(end-start), min(end-start) "
                       "from kernels where name like '%gemm%' or name like '%attn%' or name like '%accept%' or name like '%rmsnorm%' "
                       "or name like '%commit_kv%' group by 1, 2, 3, 4 order by 1, 2, 3, 4").fetchall()
    for n, gx, gy, gz, c, a, mn in rows:
        out.append(f"{short(n)[:48]:48s} grid ({gx:5d},{gy:3d},{gz:2d}) calls {c:6d} avg {a / 1e3:8.2f} us min {mn / 1e3:8.2f} us")
    return "\n".join(out)


def counters(db: str) -> str:
    cur = sqlite3.connect(db).cursor()
    rows = cur.execute("select kernel_name, grid_size_x / workgroup_size_x, grid_size_y / workgroup_size_y, grid_size_z / workgroup_size_z, "
                       "counter_name, count(*), avg(value) from counters_collection group by 1, 2, 3, 4, 5 order by 1, 2, 3, 4, 5").fetchall()
    out = [f"{'kernel':48s} {'grid (workgroups)':20s} {'counter':18s} {'dispatches':>10s} {'avg per dispatch':>18s}"]
    for n, gx, gy, gz, cn, c, v in rows:
        out.append(f"{short(n)[:48]:48s} ({gx:6d},{gy:3d},{gz:2d})      {cn:18s} {c:10d} {v:18.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("kernels", "counters"):
        sys.exit(__doc__)
    print(kernels(sys.argv[2]) if sys.argv[1] == "kernels" else counters(sys.argv[2]))
