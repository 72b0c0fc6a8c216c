"""Turns a rocprofv3 rocpd database (--kernel-trace) into the short per-kernel text summary kept under
profiles/.  Usage: python -m paper_2605_00789_amd.prof_summary <results.db> "<command that made it>" """
import sqlite3
import sys


def summarize(db_path: str, command: str) -> str:
    con = sqlite3.connect(db_path)
    rows = list(con.execute(
        "select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
        "from kernels group by name order by 6 desc"))
    total = sum(r[5] for r in rows) or 1
    lines = ["command: " + command, "source : rocprofv3 --kernel-trace (rocpd database), durations in microseconds", "",
             "%-78s %7s %10s %10s %10s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "share")]
    for name, n, avg, mn, mx, tot in rows:
        lines.append("%-78s %7d %10.2f %10.2f %10.2f %6.1f%%" % (name[:78], n, avg / 1e3, mn / 1e3, mx / 1e3, 100.0 * tot / total))
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    sys.stdout.write(summarize(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else ""))
