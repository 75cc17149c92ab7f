"""Summarise a rocprofv3 rocpd database (the *_results.db a `rocprofv3 --kernel-trace [--stats|--pmc ...]`
run writes) as a short text table: per kernel calls, average and total duration, and, when the run
collected counters, the per-dispatch average of each.

    python -m paper_2511_13841_amd.rocprof_summary <output dir>/run_results.db [--top 16]
"""
import argparse
import sqlite3


def short(name):
    return name.split("(")[0].replace("void ", "")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--top", type=int, default=16)
    a = ap.parse_args()
    c = sqlite3.connect(a.db)
    print(f"{'calls':>7} {'avg us':>10} {'total ms':>10} {'%':>6}  kernel")
    for name, calls, total, avg, pct in c.execute(
            "select name, total_calls, total_duration, average, percentage from top_kernels limit ?", (a.top,)):
        print(f"{calls:7d} {avg:10.2f} {total / 1e3:10.2f} {pct:6.2f}  {short(name)}")
    rows = list(c.execute("select kernel_name, counter_name, count(*), avg(value), avg(duration) from counters_collection "
                          "group by kernel_name, counter_name order by sum(duration) desc"))
    if rows:
        print(f"\n{'counter':28} {'dispatches':>10} {'avg/dispatch':>16} {'avg us':>9}  kernel")
        seen = []
        for kname, cname, n, avg, dur in rows:
            if kname not in seen:
                if len(seen) >= a.top:
                    continue
                seen.append(kname)
            print(f"{cname:28} {n:10d} {avg:16.1f} {dur / 1e3:9.1f}  {short(kname)}")


if __name__ == "__main__":
    main()
