"""Prints the per-kernel summary of a `rocprofv3 --kernel-trace --stats` run (its SQLite output).

    cd /tmp && export TMPDIR=/tmp
    rocprofv3 --kernel-trace --stats -d <out>/kt -o kt -- python3 bench.py --steps 50 --warmup 5 --no-cpu-baseline
    python -m paper_1709_04057_amd.kernel_stats <out>/kt/kt_results.db > profiles/<name>.txt
"""
import sqlite3
import sys


def main():
    cur = sqlite3.connect(sys.argv[1]).cursor()
    print("%-100s %6s %12s %12s %12s %12s %6s" % ("kernel", "calls", "total_us", "avg_us", "min_us", "max_us", "%"))
    rows = cur.execute("select name, count(*), sum(duration), avg(duration), min(duration), max(duration) from kernels "
                       "group by name order by sum(duration) desc").fetchall()
    total = sum(r[2] for r in rows) or 1
    for name, n, tot, avg, mn, mx in rows:
        print("%-100s %6d %12.1f %12.1f %12.1f %12.1f %6.2f" % (name[:100], n, tot / 1e3, avg / 1e3, mn / 1e3, mx / 1e3,
                                                                 100.0 * tot / total))


if __name__ == "__main__":
    main()
