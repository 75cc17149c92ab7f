"""Summarise a rocprofv3 rocpd database (the *_results.db a `rocprofv3 --kernel-trace [--stats|--pmc ...]`
run writes) as a short text table: per kernel calls, average and total duration, and, when the run
collected a counter, its per-dispatch average.

    python -m paper_2511_13841_amd.rocprof_summary gpurun_out/prof/run_results.db [--counter FETCH_SIZE]
"""
import argparse
import sqlite3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--counter", default=None)
    ap.add_argument("--top", type=int, default=16)
    a = ap.parse_args()
    c = sqlite3.connect(a.db)
    print(f"{'calls':>7} {'avg us':>10} {'total ms':>10} {'%':>6}  kernel")
    for name, calls, total, avg, pct in c.execute(
            "select name, total_calls, total_duration, average, percentage from top_kernels limit ?", (a.top,)):
        print(f"{calls:7d} {avg:10.2f} {total / 1e3:10.2f} {pct:6.2f}  {name.split(chr(40))[0]}")
    if a.counter:
        cols = [r[1] for r in c.execute("pragma table_info(counters_collection)")]
        namecol = "kernel_name" if "kernel_name" in cols else "name"
        q = (f"select {namecol}, count(*), avg(value), sum(value) from counters_collection "
             f"where counter_name = ? group by {namecol} order by sum(value) desc limit ?")
        print(f"\n{a.counter}: {'dispatches':>10} {'avg/dispatch':>14} {'sum':>14}  kernel")
        for name, n, avg, tot in c.execute(q, (a.counter, a.top)):
            print(f"{'':11} {n:10d} {avg:14.1f} {tot:14.1f}  {name.split(chr(40))[0]}")


if __name__ == "__main__":
    main()
