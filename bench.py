#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

A step is one caramel_allreduce (pack + ring reduce + unpack of all transfer units) over the
W resident gradient replicas of one synthetic workload.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E peak, GB/s


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vgg16")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--streams", type=int, default=None, help="override the workload's stream count")
    ap.add_argument("--launch-mode", choices=["unit", "stream", "auto"], default=None)
    ap.add_argument("--batch-path", choices=["staged", "direct"], default=None)
    ap.add_argument("--tile-vecs", type=int, default=None)
    ap.add_argument("--max-grid", type=int, default=None)
    ap.add_argument("--nontemporal", type=int, default=None)
    ap.add_argument("--unroll", type=int, default=None)
    ap.add_argument("--block", type=int, default=None)
    ap.add_argument("--pattern", choices=["ring", "hd", "shuffle"], default="ring")
    ap.add_argument("--launch-min-bytes", type=int, default=None)
    ap.add_argument("--align-tiles", type=int, default=None, help="0..3, see CARAMEL_OPT_ALIGN_TILES")
    ap.add_argument("--device-fill", action="store_true",
                    help="fill the replicas on the device instead of uploading Philox samples")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain in-place copy of known size (a W=1 reduction of one 1 GiB "
                         "tensor, kernel k_ring_reduce_any) so that a counter run can scale "
                         "FETCH_SIZE / WRITE_SIZE by what they read for it")
    ap.add_argument("--cpu-repeats", type=int, default=21)
    return ap.parse_args()


def read_traffic(name: str):
    """HBM bytes per reduce-kernel launch from the committed counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"ring_reduce_{name}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main() -> int:
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the W replicas are resident on it); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2004_14020_amd as cm
    from paper_2004_14020_amd.device import Replicas
    from workloads import gradients
    from workloads.shapes import workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    cm.lib()

    wl = workload(args.workload)
    elems = wl.elems()
    streams = args.streams or wl.num_streams
    plan = cm.Plan(wl.world, elems, dtype=wl.dtype, batch_threshold_bytes=wl.batch_threshold_bytes,
                   split_mode=wl.split_mode, split_bytes=wl.split_bytes, max_depth=wl.max_depth,
                   align_bytes=wl.align_bytes, num_streams=streams,
                   pattern={"ring": cm.PATTERN_RING, "hd": cm.PATTERN_HALVING_DOUBLING,
                            "shuffle": cm.PATTERN_SHUFFLE}[args.pattern])
    staged = args.batch_path == "staged"
    if args.launch_mode:
        plan.set_option(cm.OPT_LAUNCH_MODE, {"unit": cm.LAUNCH_PER_UNIT, "stream": cm.LAUNCH_PER_STREAM,
                                             "auto": cm.LAUNCH_AUTO}[args.launch_mode])
    if args.batch_path:
        plan.set_option(cm.OPT_BATCH_PATH, cm.BATCH_STAGED if staged else cm.BATCH_DIRECT)
    for opt, val in ((cm.OPT_TILE_VECS, args.tile_vecs), (cm.OPT_MAX_GRID, args.max_grid),
                     (cm.OPT_NONTEMPORAL, args.nontemporal), (cm.OPT_UNROLL, args.unroll),
                     (cm.OPT_BLOCK, args.block), (cm.OPT_LAUNCH_MIN_BYTES, args.launch_min_bytes),
                     (cm.OPT_ALIGN_TILES, args.align_tiles)):
        if val is not None:
            plan.set_option(opt, val)

    dev = Replicas(plan, elems, device="cuda:0", with_workspace=staged)
    grads = None
    if args.device_fill:
        dev.fill_random(args.seed)
    else:
        grads = gradients.replica_set(args.seed, wl.world, elems, bf16=(wl.dtype == cm.BF16), threads=16)
        dev.upload(grads)

    stream = torch.cuda.current_stream().cuda_stream
    if args.calibrate:
        n_cal = (1 << 30) // 4
        cal = cm.Plan(1, [n_cal], num_streams=1)
        buf = torch.zeros(n_cal, dtype=torch.float32, device="cuda:0")
        cal.bind([[buf.data_ptr()]], None)
        for _ in range(3):
            cal.allreduce(stream)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        cal.close()
        del buf
    for _ in range(args.warmup):
        plan.allreduce(stream)
    torch.cuda.synchronize()
    plan.profile(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plan.allreduce(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    stats = plan.profile_read()
    plan.profile(0)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    alg_bytes = wl.algorithmic_bytes()
    gbs = alg_bytes / (ms_per_step * 1e-3) / 1e9

    # Dominant kernels: the two variants of the ring-reduce kernel (stream-major for long launches
    # over large units, all-at-once for the rest); in the default direct mode nothing else runs.  The
    # library brackets everything each internal stream does in a call with one pair of HIP events
    # recorded on that stream; launches of one stream run back to back, so a launch's average
    # duration is the stream's busy time divided by its launches.  The two streams overlap in
    # time (that is the pipeline), i.e. a launch shares the memory system with a launch of the
    # other stream while it runs:
    #   per_launch_achieved = algorithmic bytes of a launch / its average duration
    #   achieved            = algorithmic bytes of a step / time from the first launch's start to
    #                         the last launch's end (= per-launch figure x launches in flight)
    red, seq = stats[cm.K_REDUCE], stats[cm.K_SEQUENCE]
    launches_per_step = red["launches"] / args.steps
    avg_ms = seq["total_ms"] / max(1, red["launches"])
    span_ms = seq["span_ms"] / max(1, seq["calls"])
    bytes_per_launch = alg_bytes / launches_per_step       # 2*W*s per element the launch reduces
    per_launch = bytes_per_launch / (avg_ms * 1e-3) / 1e9
    achieved = alg_bytes / (span_ms * 1e-3) / 1e9
    traffic = read_traffic(wl.name)
    roofline = {
        "bound": "hbm", "kernel": "k_ring_reduce_sm (large units) + k_ring_reduce (others)", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
        "launches_per_step": launches_per_step, "avg_launch_ms": round(avg_ms, 6),
        "bytes_per_launch": round(bytes_per_launch), "per_launch_achieved": round(per_launch, 1),
        "launches_in_flight": round(seq["total_ms"] / max(seq["span_ms"], 1e-9), 3),
        "step_span_ms": round(span_ms, 5),
    }

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ocfg = oracle.Config(wl.world, wl.dtype, wl.batch_threshold_bytes, wl.split_mode, wl.max_depth,
                             wl.split_bytes, wl.align_bytes, wl.num_streams,
                             {"ring": 0, "hd": 1, "shuffle": 2}[args.pattern])
        oplan = oracle.build_plan(ocfg, elems)
        if grads is None:
            grads = gradients.replica_set(args.seed, wl.world, elems, bf16=(wl.dtype == cm.BF16), threads=16)
        fused = oracle.new_fused(oplan)
        times = []
        for _ in range(args.cpu_repeats):
            c0 = time.perf_counter()
            oracle.allreduce(oplan, grads, fused)       # in place; speed does not depend on values
            times.append(time.perf_counter() - c0)
        med = sorted(times)[len(times) // 2]
        cpu = {"value": round(alg_bytes / med / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"the whole {wl.name} workload (W={wl.world}), pack+ring_reduce+unpack, "
                         f"median of {args.cpu_repeats} passes, {med * 1e3:.0f} ms per pass"}
        # the same oracle functions with the (independent) units dealt out to the host's cores
        from concurrent.futures import ThreadPoolExecutor
        n_thr = max(1, min(16, os.cpu_count() or 1))

        def reduce_one(u):
            oracle.reduce_unit(oracle.unit_views(oplan, u, grads, fused), u.seg_start, ocfg.dtype, ocfg.pattern)

        par = []
        with ThreadPoolExecutor(n_thr) as pool:
            for _ in range(5):
                c0 = time.perf_counter()
                oracle.pack(oplan, grads, fused)
                list(pool.map(reduce_one, oplan.units))
                oracle.unpack(oplan, grads, fused)
                par.append(time.perf_counter() - c0)
        pmed = sorted(par)[len(par) // 2]
        cpu["all_cores"] = {"value": round(alg_bytes / pmed / 1e9, 3), "unit": "GB/s", "cores": n_thr,
                            "sample": f"same workload and functions, units dealt to {n_thr} threads, median of 5 passes, "
                                      f"{pmed * 1e3:.0f} ms per pass"}

    out = {
        "metric": "fused pack+ring-reduce+unpack HBM GB/s and % of peak, VGG-16 shape, W=8",
        "value": round(gbs, 1), "unit": "GB/s", "pct_of_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == cm.F32 else "bf16 in/out, f32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "world": wl.world, "tensors": len(elems), "elems_per_replica": wl.total_elems,
                   "algorithmic_bytes": alg_bytes, "batch_threshold_bytes": wl.batch_threshold_bytes,
                   "split_mode": ["none", "fixed", "adaptive"][wl.split_mode], "split_bytes": wl.split_bytes,
                   "units": plan.counts()[0], "num_streams": streams,
                   "pattern": args.pattern, "launch_mode": args.launch_mode or "auto", "batch_path": args.batch_path or "direct"},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    plan.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
