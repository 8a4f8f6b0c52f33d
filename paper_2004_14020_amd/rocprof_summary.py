"""Text summaries of a rocprofv3 results database (the `*_results.db` that
`rocprofv3 --kernel-trace` or `rocprofv3 --pmc ...` writes), as kept under profiles/.

  python -m paper_2004_14020_amd.rocprof_summary kernels  <results.db> [--per-step N]
  python -m paper_2004_14020_amd.rocprof_summary counters <results.db>

`kernels` reads the view `kernels(name, start, end, queue_id, grid_x, workgroup_x)`:
per kernel name the number of dispatches and the average / minimum / maximum / total duration
(end - start, nanoseconds), and -- with --per-step N, the number of this library's launches in
one step -- for the last half of the steps the span from the first launch's start to the last
launch's end, the sum of the launch durations (their ratio = launches in flight), the gaps
between consecutive launches of a queue, and the period from one step's start to the next's.

`counters` reads the view `counters_collection(kernel_name, counter_name, value, dispatch_id)`:
per kernel name and counter the number of dispatches and the mean value per dispatch.
"""
from __future__ import annotations

import argparse
import re
import sqlite3
import statistics
import sys


def short(name: str) -> str:
    name = name.replace("void caramel::(anonymous namespace)::", "").replace("void (anonymous namespace)::", "")
    name = re.sub(r"\(.*", "", name)
    return name if len(name) <= 64 else name[:61] + "..."


def kernels(path: str, per_step: int) -> None:
    cur = sqlite3.connect(path).cursor()
    rows = list(cur.execute("select name, start, end, queue_id, grid_x, workgroup_x from kernels order by start"))
    by = {}
    for name, start, end, *_ in rows:
        by.setdefault(short(name), []).append(end - start)
    total = sum(sum(v) for v in by.values())
    print(f"{'kernel':66s} {'calls':>6s} {'avg_ns':>11s} {'min_ns':>10s} {'max_ns':>10s} {'total_ns':>13s} {'share':>7s}")
    for name, d in sorted(by.items(), key=lambda kv: -sum(kv[1])):
        print(f"{name:66s} {len(d):6d} {sum(d) / len(d):11.1f} {min(d):10d} {max(d):10d} {sum(d):13d} {100 * sum(d) / total:6.2f}%")
    if not per_step:
        return
    mine = [r for r in rows if "caramel" in r[0]]
    steps = [mine[i * per_step:(i + 1) * per_step] for i in range(len(mine) // per_step)]
    use = steps[len(steps) // 2:]
    print(f"\n{len(mine)} launches of this library = {len(steps)} steps of {per_step}; the last of them:")
    t0 = use[-1][0][1]
    for name, start, end, queue, grid, wg in use[-1]:
        print(f"  queue {queue}  {(start - t0) / 1e3:9.1f} .. {(end - t0) / 1e3:9.1f} us  ({(end - start) / 1e3:8.1f} us)  "
              f"{grid // wg:6d} workgroups of {wg:4d}  {short(name)}")
    spans, busy, gaps, period = [], [], [], []
    for i, s in enumerate(use):
        a, b = min(r[1] for r in s), max(r[2] for r in s)
        spans.append((b - a) / 1e3)
        busy.append(sum(r[2] - r[1] for r in s) / 1e3)
        g, per_queue = 0, {}
        for r in s:
            per_queue.setdefault(r[3], []).append(r)
        for rs in per_queue.values():
            for x, y in zip(rs, rs[1:]):
                g += max(0, y[1] - x[2])
        gaps.append(g / 1e3)
        if i + 1 < len(use):
            period.append((min(r[1] for r in use[i + 1]) - a) / 1e3)
    m = statistics.mean
    print(f"over the last {len(use)} steps: span first start .. last end {m(spans):.1f} us, sum of launch durations "
          f"{m(busy):.1f} us (launches in flight {m(busy) / m(spans):.2f}), gaps between launches of a queue "
          f"{m(gaps):.1f} us, start-to-start period {m(period) if period else float('nan'):.1f} us")


def counters(path: str) -> None:
    cur = sqlite3.connect(path).cursor()
    q = ("select kernel_name, counter_name, count(*), avg(value) from counters_collection "
         "group by kernel_name, counter_name order by kernel_name, counter_name")
    print(f"{'kernel':66s} {'counter':28s} {'dispatches':>10s} {'mean per dispatch':>20s}")
    for name, counter, n, mean in cur.execute(q):
        print(f"{short(name):66s} {counter:28s} {n:10d} {mean:20.1f}")


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["kernels", "counters"])
    ap.add_argument("db")
    ap.add_argument("--per-step", type=int, default=0)
    args = ap.parse_args()
    if args.what == "kernels":
        kernels(args.db, args.per_step)
    else:
        counters(args.db)
    return 0


if __name__ == "__main__":
    sys.exit(main())
