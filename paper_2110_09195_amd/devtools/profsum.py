"""Summarise a rocprofv3 kernel trace (the rocpd SQLite file it writes) as text.

    python -m paper_2110_09195_amd.devtools.profsum gpurun_out/prof/x_results.db > profiles/<name>.txt

Prints, per kernel name: launches, average / min / max duration in microseconds and the
share of total kernel time.  Used to produce the summaries under profiles/.
"""
import sqlite3
import sys


def summarise(path, out=sys.stdout):
    db = sqlite3.connect(path)
    rows = db.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                      "from kernels group by name order by 6 desc").fetchall()
    total = sum(r[5] for r in rows) or 1
    out.write("%-72s %7s %10s %10s %10s %7s\n" % ("kernel", "calls", "avg us", "min us", "max us", "share"))
    for name, n, avg, mn, mx, tot in rows:
        short = name.replace("snn::(anonymous namespace)::", "").replace("void ", "")
        short = short.split("(")[0]
        out.write("%-72s %7d %10.2f %10.2f %10.2f %6.1f%%\n" % (short[:72], n, avg / 1e3, mn / 1e3, mx / 1e3, 100.0 * tot / total))


if __name__ == "__main__":
    summarise(sys.argv[1])
