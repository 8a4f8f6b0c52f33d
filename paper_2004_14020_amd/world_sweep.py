#!/usr/bin/env python3
"""World-size sweep: one all-reduce of a single fp32 (or bf16) tensor, split into 4 MiB chunks,
with the replicas together holding a fixed number of bytes, for a range of world sizes and the
three aggregation patterns (paper sections 2 and 6.3: ring, halving-doubling, shuffle).
World sizes 2, 4, 8 and 16 run kernels specialised for them, every other size the generic
kernel; halving-doubling needs a power of two.  Prints algorithmic GB/s (2 * W * N * s bytes per
call) and the fraction of the 8 TB/s HBM peak.

  python -m paper_2004_14020_amd.world_sweep [--total-mib 1024] [--bf16]
"""
from __future__ import annotations

import argparse
import time

import torch

from . import BF16, F32, PATTERN_HALVING_DOUBLING, PATTERN_RING, PATTERN_SHUFFLE, SPLIT_FIXED, Plan
from .device import Replicas


def time_plan(plan: Plan, elems, steps: int) -> float:
    dev = Replicas(plan, elems, with_workspace=False, large_align=256)
    dev.fill_random(0)
    s = torch.cuda.current_stream().cuda_stream
    best = None
    for _ in range(3):
        for _ in range(3):
            plan.allreduce(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            plan.allreduce(s)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        best = dt if best is None else min(best, dt)
    plan.close()
    return best


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--total-mib", type=int, default=1024, help="bytes held by all replicas together")
    ap.add_argument("--bf16", action="store_true")
    ap.add_argument("--steps", type=int, default=30)
    args = ap.parse_args()
    es = 2 if args.bf16 else 4
    print(f"# one {'bf16' if args.bf16 else 'fp32'} tensor per replica, 4 MiB chunks, replicas together {args.total_mib} MiB, "
          f"default launch options; best of 3 x {args.steps} calls")
    print(f"{'W':>3} {'MiB/replica':>12} {'ring ms':>9} {'%peak':>6} {'halving-doubling ms':>20} {'%peak':>6} {'shuffle ms':>11} {'%peak':>6}")
    for W in (2, 3, 4, 5, 6, 7, 8, 12, 16, 24, 32, 48, 64):
        n = (args.total_mib << 20) // W // es // 64 * 64 + 4     # not a multiple of the tile size
        row = f"{W:>3} {n * es / 2 ** 20:>12.1f}"
        for pattern, width in ((PATTERN_RING, 9), (PATTERN_HALVING_DOUBLING, 20), (PATTERN_SHUFFLE, 11)):
            if pattern == PATTERN_HALVING_DOUBLING and W & (W - 1):
                row += f" {'-':>{width}} {'-':>6}"
                continue
            plan = Plan(W, [n], dtype=BF16 if args.bf16 else F32, split_mode=SPLIT_FIXED, split_bytes=4 << 20,
                        num_streams=2, pattern=pattern)
            t = time_plan(plan, [n], args.steps)
            row += f" {t * 1e3:>{width}.4f} {100 * 2 * W * n * es / t / 8e12:>6.1f}"
        print(row, flush=True)


if __name__ == "__main__":
    main()
