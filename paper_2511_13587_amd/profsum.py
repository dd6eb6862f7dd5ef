"""Text summaries of rocprofv3 output databases (rocpd SQLite): per-kernel durations from a
--kernel-trace run, per-kernel counter averages from a --pmc run.

    python -m paper_2511_13587_amd.profsum kernels <results.db>
    python -m paper_2511_13587_amd.profsum counters <results.db>
    python -m paper_2511_13587_amd.profsum pivot <results.db> [<results.db> ...]
    python -m paper_2511_13587_amd.profsum ratios <results.db> [<results.db> ...]
    python -m paper_2511_13587_amd.profsum window <results.db> <first kernel substring> <last kernel substring>
    python -m paper_2511_13587_amd.profsum traffic <fetch.db> <write.db> <kernel substring> <grid_x list, workgroups> [out.json]

`window`: the dispatches between the first launch of one kernel and the last launch of another (e.g. the
drafting calls of a bench run: from the first k_draft_state to the last k_draft_select), per kernel and per
call of the first kernel.

`pivot`: one line per (hot kernel, grid) with every counter of the given --pmc runs as a column (average per
dispatch, summed over the chip's instances as rocprofv3 reports them), for reading ratios such as MFMA-busy
cycles per CU-busy cycle.

`ratios`: the same dispatches as `pivot`, reduced to the ratios that say what a kernel waits for: MFMA-busy cycles per
SIMD cycle of the busy CUs (SQ_VALU_MFMA_BUSY_CYCLES counts per SIMD, SQ_BUSY_CU_CYCLES per CU), the share of wave
cycles spent waiting for any instruction / for LDS, VALU-active share, L2 hit rate, mean L1-to-L2 read latency in
cycles, LDS bank-conflict cycles per LDS-active cycle.

`traffic`: HBM bytes per launch of one kernel from a FETCH_SIZE run and a WRITE_SIZE run (KiB per
dispatch), each scaled by what the same counter reads for the 256 MiB k_copy_bytes launches of the
same run (bench.py --calibrate-copy).
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


def window(db: str, first: str, last: str) -> str:
    cur = sqlite3.connect(db).cursor()
    t0 = cur.execute("select min(start) from kernels where name like ?", (f"%{first}%",)).fetchone()[0]
    t1 = cur.execute("select max(end) from kernels where name like ?", (f"%{last}%",)).fetchone()[0]
    calls = cur.execute("select count(*) from kernels where name like ?", (f"%{first}%",)).fetchone()[0]
    rows = cur.execute("select name, count(*), sum(end-start), avg(end-start) from kernels where start >= ? and end <= ? "
                       "group by name order by 3 desc", (t0, t1)).fetchall()
    busy = sum(r[2] for r in rows)
    n = sum(r[1] for r in rows)
    out = [f"window: first {first} .. last {last}: {calls} calls, {n} launches ({n / calls:.1f} per call), "
           f"kernel time {busy / calls / 1e3:.1f} us per call, span {(t1 - t0) / calls / 1e3:.1f} us per call",
           f"{'kernel':64s} {'per call':>9s} {'avg_us':>9s} {'us/call':>9s} {'pct':>6s}"]
    for name, c, sm, a in rows:
        out.append(f"{short(name)[:64]:64s} {c / calls:9.2f} {a / 1e3:9.2f} {sm / calls / 1e3:9.2f} {100 * sm / busy:6.2f}")
    return "\n".join(out)


def counters(db: str) -> str:
    cur = sqlite3.connect(db).cursor()
    rows = cur.execute("select kernel_name, grid_size_x / workgroup_size_x, grid_size_y / workgroup_size_y, grid_size_z / workgroup_size_z, "
                       "counter_name, count(*), avg(value) from counters_collection group by 1, 2, 3, 4, 5 order by 1, 2, 3, 4, 5").fetchall()
    out = [f"{'kernel':48s} {'grid (workgroups)':20s} {'counter':18s} {'dispatches':>10s} {'avg per dispatch':>18s}"]
    for n, gx, gy, gz, cn, c, v in rows:
        out.append(f"{short(n)[:48]:48s} ({gx:6d},{gy:3d},{gz:2d})      {cn:18s} {c:10d} {v:18.1f}")
    return "\n".join(out)


def pivot(dbs) -> str:
    table, names = {}, []
    for db in dbs:
        cur = sqlite3.connect(db).cursor()
        rows = cur.execute("select kernel_name, grid_size_x / workgroup_size_x, grid_size_y / workgroup_size_y, grid_size_z / workgroup_size_z, "
                           "counter_name, count(*), avg(value) from counters_collection where kernel_name like '%gemm%' or kernel_name like "
                           "'%attn%' or kernel_name like '%accept_node%' or kernel_name like '%commit_kv%' or kernel_name like '%rmsnorm%' "
                           "group by 1, 2, 3, 4, 5").fetchall()
        for n, gx, gy, gz, cn, c, v in rows:
            table.setdefault((short(n)[:44], gx, gy, gz), {"dispatches": c})[cn] = v
            if cn not in names:
                names.append(cn)
    out = [f"{'kernel':44s} {'grid':>14s} {'disp':>6s} " + " ".join(f"{n[-22:]:>22s}" for n in names)]
    for (n, gx, gy, gz), row in sorted(table.items()):
        out.append(f"{n:44s} {f'({gx},{gy},{gz})':>14s} {row['dispatches']:6d} " + " ".join(f"{row.get(k, float('nan')):22.1f}" for k in names))
    return "\n".join(out)


def ratios(dbs) -> str:
    table = {}
    for db in dbs:
        cur = sqlite3.connect(db).cursor()
        rows = cur.execute("select kernel_name, grid_size_x / workgroup_size_x, grid_size_y / workgroup_size_y, grid_size_z / workgroup_size_z, "
                           "counter_name, count(*), avg(value) from counters_collection where kernel_name like '%gemm%' or kernel_name like "
                           "'%attn%' or kernel_name like '%accept_node%' or kernel_name like '%rmsnorm%' group by 1, 2, 3, 4, 5").fetchall()
        for n, gx, gy, gz, cn, c, v in rows:
            table.setdefault((short(n)[:44], gx, gy, gz), {"dispatches": c})[cn] = v
    nan = float("nan")

    def div(r, a, b, k=1.0):
        return r[a] / (k * r[b]) if a in r and b in r and r[b] else nan

    out = [f"{'kernel':44s} {'grid':>14s} {'disp':>6s} {'mfma_util':>9s} {'wait_any':>8s} {'wait_lds':>8s} {'valu':>6s} {'l2_hit':>6s} {'l1_l2_lat':>9s} {'bank_conf':>9s}"]
    for (n, gx, gy, gz), r in sorted(table.items()):
        out.append(f"{n:44s} {f'({gx},{gy},{gz})':>14s} {r['dispatches']:6d} {div(r, 'SQ_VALU_MFMA_BUSY_CYCLES', 'SQ_BUSY_CU_CYCLES', 4.0):9.2f} "
                   f"{div(r, 'SQ_WAIT_INST_ANY', 'SQ_WAVE_CYCLES'):8.2f} {div(r, 'SQ_WAIT_INST_LDS', 'SQ_WAVE_CYCLES'):8.3f} "
                   f"{div(r, 'SQ_ACTIVE_INST_VALU', 'SQ_WAVE_CYCLES'):6.2f} {div(r, 'TCC_HIT_sum', 'TCC_REQ_sum'):6.2f} "
                   f"{div(r, 'TCP_TCC_READ_REQ_LATENCY_sum', 'TCP_TCC_READ_REQ_sum'):9.0f} {div(r, 'SQ_LDS_BANK_CONFLICT', 'SQ_LDS_IDX_ACTIVE'):9.2f}")
    return "\n".join(out)


def traffic(fetch_db: str, write_db: str, kernel: str, grids, out_json=None) -> str:
    import json
    res = {"kernel": kernel, "grids_x_workgroups": grids, "copy_bytes": 256 << 20}
    total = 0.0
    lines = []
    for name, db in (("FETCH_SIZE", fetch_db), ("WRITE_SIZE", write_db)):
        cur = sqlite3.connect(db).cursor()
        cal = cur.execute("select avg(value) from counters_collection where kernel_name like '%k_copy_bytes%' and counter_name = ?",
                          (name,)).fetchone()[0]
        factor = (256 << 10) / cal            # the copy reads and writes 262144 KiB
        names = [k for k in kernel.split(",") if k]      # several kernel-name substrings, comma-separated
        q = ("select count(*), avg(value) from counters_collection where (%s) and counter_name = ? "
             "and grid_size_x / workgroup_size_x in (%s)" % (" or ".join("kernel_name like ?" for _ in names),
                                                            ",".join(str(int(g)) for g in grids)))
        n, avg = cur.execute(q, tuple(f"%{k}%" for k in names) + (name,)).fetchone()
        res[name] = {"copy_kernel_reads_KiB": cal, "scale_factor": factor, "dispatches": n, "avg_KiB_per_dispatch": avg,
                     "scaled_bytes_per_launch": avg * 1024 * factor}
        total += avg * 1024 * factor
        lines.append(f"{name}: copy kernel reads {cal:.1f} KiB for 262144 KiB moved -> factor {factor:.3f}; {kernel}: {n} dispatches, "
                     f"avg {avg:.1f} KiB -> {avg * 1024 * factor / 1e6:.2f} MB per launch")
    res["hbm_bytes_per_launch"] = total
    lines.append(f"HBM traffic per launch (fetch + write): {total / 1e6:.2f} MB")
    if out_json:
        json.dump(res, open(out_json, "w"), indent=1)
    return "\n".join(lines)


if __name__ == "__main__":
    if len(sys.argv) >= 6 and sys.argv[1] == "traffic":
        print(traffic(sys.argv[2], sys.argv[3], sys.argv[4], [int(g) for g in sys.argv[5].split(",")],
                      sys.argv[6] if len(sys.argv) > 6 else None))
    elif len(sys.argv) >= 3 and sys.argv[1] in ("pivot", "ratios"):
        print(pivot(sys.argv[2:]) if sys.argv[1] == "pivot" else ratios(sys.argv[2:]))
    elif len(sys.argv) == 5 and sys.argv[1] == "window":
        print(window(sys.argv[2], sys.argv[3], sys.argv[4]))
    elif len(sys.argv) == 3 and sys.argv[1] in ("kernels", "counters"):
        print(kernels(sys.argv[2]) if sys.argv[1] == "kernels" else counters(sys.argv[2]))
    else:
        sys.exit(__doc__)
