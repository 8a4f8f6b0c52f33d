#!/usr/bin/env python3
"""Batching threshold from measurements, the way section 4.2 describes it: time sequential
aggregations of two sizes (the paper takes 64 B and 4 MB), fit the line  time = a + b * bytes
through the two points, and take the smallest size x with f(2x) / (2 f(x)) > 0.8.  Here the
"network" is this library's own all-reduce of W replicas on one GPU, so `a` is the fixed cost
of a call (launch and stream signalling) and 1/b the streaming rate.

  python -m paper_2004_14020_amd.threshold_fit [--world 8] [--small 64] [--large 134217728]
"""
from __future__ import annotations

import argparse
import time

import torch

from . import Plan, caramel_net_model_fit, caramel_threshold_estimate
from .device import Replicas


def seconds_per_call(world: int, nbytes: int, calls: int) -> float:
    """Mean time of one all-reduce of a single fp32 tensor of `nbytes` per replica, each call
    finished before the next starts (sequential transfers)."""
    n = max(1, nbytes // 4)
    plan = Plan(world, [n], num_streams=2)
    dev = Replicas(plan, [n], with_workspace=False)
    dev.fill_random(0)
    s = torch.cuda.current_stream().cuda_stream
    for _ in range(20):
        plan.allreduce(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        plan.allreduce(s)
        torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / calls
    plan.close()
    return dt


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--world", type=int, default=8)
    ap.add_argument("--small", type=int, default=64, help="bytes per replica of the small probe")
    ap.add_argument("--large", type=int, default=128 << 20,
                    help="bytes per replica of the large probe; the paper's 4 MB would sit in this GPU's "
                         "256 MB last-level cache when the call is repeated, so the default is 128 MiB")
    ap.add_argument("--calls", type=int, default=300)
    args = ap.parse_args()
    t1 = seconds_per_call(args.world, args.small, args.calls) * 1e6
    t2 = seconds_per_call(args.world, args.large, args.calls) * 1e6
    a, b = caramel_net_model_fit(args.small, t1, args.large, t2)
    print(f"W = {args.world}: {args.small} B per replica in {t1:.2f} us, {args.large} B in {t2:.2f} us")
    print(f"model: time = {a:.3f} us + {b:.3e} us/B * bytes   (streaming rate {1e-3 / b:.1f} GB/s per replica, "
          f"{2 * args.world * 1e-3 / b:.0f} GB/s of algorithmic traffic)")
    thr = caramel_threshold_estimate(a, b)
    print(f"threshold: smallest x with f(2x) / (2 f(x)) > 0.8  ->  {thr} bytes ({thr / (1 << 20):.2f} MiB) per replica")
    for x in (thr // 4, thr, 4 * thr):
        f1, f2 = a + b * x, a + b * 2 * x
        print(f"  check x = {x:>10d}: f(2x) / (2 f(x)) = {f2 / (2 * f1):.3f}")


if __name__ == "__main__":
    main()
