"""Summarise a rocprofv3 result database (rocpd sqlite, the default output of ROCm 7) as text.

  python -m paper_2511_21699_amd.profile_summary kernels  <results.db>    per-kernel call count and durations
  python -m paper_2511_21699_amd.profile_summary counters <results.db>    per-kernel mean of each collected counter

Used to produce the short summaries kept under profiles/.
"""
import sqlite3
import sys


def kernels(db: str) -> str:
    c = sqlite3.connect(db)
    out = [f"{'kernel':72s} {'calls':>7s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_ms':>9s}"]
    q = ("select name, count(*), avg(duration), min(duration), max(duration), sum(duration) from kernels "
         "group by name order by sum(duration) desc limit 20")
    for name, n, avg, mn, mx, tot in c.execute(q):
        out.append(f"{name[:72]:72s} {n:7d} {avg / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {tot / 1e6:9.3f}")
    return "\n".join(out)


def counters(db: str) -> str:
    c = sqlite3.connect(db)
    rows = c.execute("select kernel_name, counter_name, count(*), avg(value), max(value) from counters_collection "
                     "group by kernel_name, counter_name order by kernel_name, counter_name")
    out = [f"{'kernel':60s} {'counter':24s} {'dispatches':>10s} {'mean value':>14s} {'max value':>14s}"]
    for k, cn, n, v, mx in rows:
        out.append(f"{k[:60]:60s} {cn:24s} {n:10d} {v:14.1f} {mx:14.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("kernels", "counters"):
        print(__doc__)
        sys.exit(2)
    print(kernels(sys.argv[2]) if sys.argv[1] == "kernels" else counters(sys.argv[2]))
