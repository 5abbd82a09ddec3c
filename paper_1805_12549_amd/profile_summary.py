"""Turn a rocprofv3 ``*_results.db`` (rocpd SQLite output of ``--kernel-trace --stats``) into
the short per-kernel text table kept under ``profiles/``.

    python -m paper_1805_12549_amd.profile_summary gpurun_out/prof/run_results.db "command line" > profiles/x.txt
"""
import sqlite3
import sys


def summarize(db_path: str, command: str = "") -> str:
    db = sqlite3.connect(db_path)
    cur = db.cursor()
    rows = list(cur.execute(
        "select name, count(*), sum(duration), avg(duration), min(duration), max(duration) "
        "from kernels group by name order by sum(duration) desc"))
    total = sum(r[2] for r in rows) or 1
    out = []
    if command:
        out.append("command: " + command)
    out.append("source: rocprofv3 --kernel-trace --stats (durations in microseconds)")
    out.append("%-9s %-12s %-10s %-10s %-10s %-6s %s" % ("calls", "total_us", "avg_us", "min_us", "max_us", "pct", "kernel"))
    for name, calls, tot, avg, mn, mx in rows[:12]:
        short = name if len(name) < 110 else name[:107] + "..."
        out.append("%-9d %-12.1f %-10.2f %-10.2f %-10.2f %-6.2f %s" % (
            calls, tot / 1e3, avg / 1e3, mn / 1e3, mx / 1e3, 100.0 * tot / total, short))
    # per-grid breakdown of the dominant kernel (one line per layer shape)
    if rows:
        dom = rows[0][0]
        out.append("")
        out.append("dominant kernel by launch grid (one grid size per layer shape):")
        out.append("%-10s %-8s %-10s %-8s %-8s" % ("grid_x", "calls", "avg_us", "lds", "vgpr"))
        for g, calls, avg, lds, vg, av in cur.execute(
                "select grid_x, count(*), avg(duration), max(lds_size), max(vgpr_count), max(accum_vgpr_count) "
                "from kernels where name = ? group by grid_x order by grid_x desc", (dom,)):
            out.append("%-10d %-8d %-10.2f %-8d %d+%d" % (g, calls, avg / 1e3, lds, vg, av))
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    sys.stdout.write(summarize(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else ""))
