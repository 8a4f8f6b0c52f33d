#!/usr/bin/env python3
"""Depth sweep: time of one all-reduce of a single tensor versus its size, for fixed depths
1, 2, 4, 8 and for the adaptive rule -- the single-GPU counterpart of the paper's depth
experiment (section 6.3: small transfers get slower with depth, large ones faster, and the
adaptive choice follows the better curve).  Here the per-chunk overhead is a kernel launch and
the overlap is between the launches of the two streams.

  python -m paper_2004_14020_amd.depth_sweep [--world 8] [--threshold-bytes 4194304]
"""
from __future__ import annotations

import argparse
import time

import torch

from . import (LAUNCH_PER_UNIT, OPT_LAUNCH_MIN_BYTES, OPT_LAUNCH_MODE, OPT_LONG_LAUNCH_MIN_BYTES, SPLIT_ADAPTIVE, SPLIT_FIXED, SPLIT_NONE, Plan)
from .device import Replicas


def time_plan(plan: Plan, elems, steps: int) -> float:
    dev = Replicas(plan, elems, with_workspace=False)
    dev.fill_random(0)
    s = torch.cuda.current_stream().cuda_stream
    for _ in range(5):
        plan.allreduce(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        plan.allreduce(s)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / steps
    plan.close()
    return us


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--world", type=int, default=8)
    ap.add_argument("--threshold-bytes", type=int, default=4 << 20,
                    help="S of the adaptive rule: depth = clamp(floor(bytes / S), 1, 8)")
    ap.add_argument("--steps", type=int, default=50)
    args = ap.parse_args()
    W = args.world
    print(f"# one fp32 tensor per replica, W = {W}, two streams, one launch per chunk; microseconds per all-reduce")
    print(f"# adaptive: depth = clamp(floor(bytes / {args.threshold_bytes}), 1, 8)")
    print(f"{'bytes':>12} {'d=1':>9} {'d=2':>9} {'d=4':>9} {'d=8':>9} {'adaptive':>9} {'(depth)':>8} {'GB/s best':>10}")
    size = 16 << 10
    while size <= (512 << 20):
        n = size // 4
        row = []
        for depth in (1, 2, 4, 8):
            piece = max(16, (size // depth + 15) // 16 * 16)
            mode = SPLIT_NONE if depth == 1 else SPLIT_FIXED
            plan = Plan(W, [n], split_mode=mode, split_bytes=piece if depth > 1 else 0, num_streams=2)
            plan.set_option(OPT_LAUNCH_MODE, LAUNCH_PER_UNIT)
            plan.set_option(OPT_LAUNCH_MIN_BYTES, 0)
            plan.set_option(OPT_LONG_LAUNCH_MIN_BYTES, 0)
            row.append(time_plan(plan, [n], args.steps))
        plan = Plan(W, [n], split_mode=SPLIT_ADAPTIVE, split_bytes=args.threshold_bytes, max_depth=8, num_streams=2)
        plan.set_option(OPT_LAUNCH_MODE, LAUNCH_PER_UNIT)
        plan.set_option(OPT_LAUNCH_MIN_BYTES, 0)
        plan.set_option(OPT_LONG_LAUNCH_MIN_BYTES, 0)
        adaptive_depth = plan.counts()[0]
        row.append(time_plan(plan, [n], args.steps))
        best = min(row)
        print(f"{size:>12} " + " ".join(f"{x:>9.1f}" for x in row) + f" {adaptive_depth:>8} {2 * W * size / best / 1e3:>10.0f}",
              flush=True)
        size *= 4


if __name__ == "__main__":
    main()
