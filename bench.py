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
    ap.add_argument("--long-run-bytes", type=int, default=None, help="see CARAMEL_OPT_LONG_RUN_BYTES")
    ap.add_argument("--large-align", type=int, default=256,
                    help="start of every tensor of >= 1 MiB inside a replica's arena (a multiple of 256)")
    ap.add_argument("--device-fill", action="store_true",
                    help="fill the replicas on the device instead of uploading Philox samples")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-repeats", type=int, default=21)
    ap.add_argument("--probe", action="store_true",
                    help="instead of the benchmark: time plain streaming kernels of known traffic "
                         "(caramel_stream_probe) in the access shapes of the reduce kernels, and a 1 GiB "
                         "torch copy; prints one line per case")
    ap.add_argument("--probe-mib", type=int, default=512, help="--probe: MiB per buffer")
    ap.add_argument("--profile-level", type=int, default=2,
                    help="HIP-event timing of the steps that follow the timed region: 2 = a pair per kernel "
                         "launch (needed for the roofline line), 1 = a pair per stream and call")
    ap.add_argument("--profile-steps", type=int, default=50, help="steps timed launch by launch after the timed region")
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


def probe(args, cm, torch) -> int:
    """Ceilings for the reduce kernels: W buffers read, written, and updated in place (every value
    read once and written once, like the ring reduction) by plain kernels without descriptor
    tables, in 4 KiB, 16 KiB and 64 KiB runs per workgroup; and copies of known size, one of them
    not this library's (torch), to check a profiler's counters against."""
    nbytes = args.probe_mib << 20
    stream = torch.cuda.current_stream().cuda_stream

    def timed(fn, moved):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / 10
            best = dt if best is None else min(best, dt)
        return best * 1e3, moved / best / 1e9

    for W in (1, 8, 16):
        bufs = [torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda:0") for _ in range(W)]
        ptrs = [b.data_ptr() for b in bufs]
        for mode, name, factor in ((cm.PROBE_READ, "read", 1), (cm.PROBE_WRITE, "write", 1), (cm.PROBE_UPDATE, "update", 2)):
            for run, block in ((4096, 256), (16384, 1024), (65536, 1024)):
                if mode != cm.PROBE_UPDATE and run != 16384:
                    continue
                ms, gbs = timed(lambda: cm.stream_probe(mode, ptrs, nbytes, run, block, stream), factor * W * nbytes)
                print(json.dumps({"probe": name, "buffers": W, "mib_per_buffer": args.probe_mib, "run_bytes": run,
                                  "block": block, "ms": round(ms, 4), "GB/s": round(gbs, 1),
                                  "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}), flush=True)
        del bufs
    gib = 1 << 30
    a = torch.zeros(gib // 4, dtype=torch.float32, device="cuda:0")
    b = torch.zeros(gib // 4, dtype=torch.float32, device="cuda:0")
    ms, gbs = timed(lambda: cm.stream_probe(cm.PROBE_COPY, [a.data_ptr(), b.data_ptr()], gib, 16384, 1024, stream), 2 * gib)
    print(json.dumps({"probe": "copy 1 GiB (k_probe)", "ms": round(ms, 4), "GB/s": round(gbs, 1),
                      "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}), flush=True)
    ms, gbs = timed(lambda: b.copy_(a), 2 * gib)
    print(json.dumps({"probe": "copy 1 GiB (torch copy_)", "ms": round(ms, 4), "GB/s": round(gbs, 1),
                      "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}), flush=True)
    return 0


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

    if args.probe:
        return probe(args, cm, torch)

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
                     (cm.OPT_ALIGN_TILES, args.align_tiles), (cm.OPT_LONG_RUN_BYTES, args.long_run_bytes)):
        if val is not None:
            plan.set_option(opt, val)

    dev = Replicas(plan, elems, device="cuda:0", with_workspace=staged, large_align=args.large_align)
    grads = None
    if args.device_fill:
        dev.fill_random(args.seed)
    else:
        grads = gradients.replica_set(args.seed, wl.world, elems, bf16=(wl.dtype == cm.BF16), threads=16)
        dev.upload(grads)

    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(args.warmup):
        plan.allreduce(stream)
    torch.cuda.synchronize()
    # The timed region: K steps between two synchronisations, with no timing events inside (a
    # pair of events per launch costs about 20 us per step, a tenth of a short step), bracketed
    # by one pair of events on the stream the kernels are launched on.
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        plan.allreduce(stream)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    region_ms = ev0.elapsed_time(ev1)
    # Right after it, the same steps again with one pair of HIP events around every kernel launch
    # (recorded by the library on the launch stream): each kernel's own average duration.
    plan.profile(args.profile_level)
    for _ in range(args.profile_steps):
        plan.allreduce(stream)
    stats = plan.profile_read()
    plan.profile(0)
    prof_steps = args.profile_steps

    # the same calls issued from inside the library: what a call costs the host, and what it
    # costs on the stream, without the interpreter in between
    host_us, stream_us = plan.allreduce_loop(max(args.steps, 100), stream)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    alg_bytes = wl.algorithmic_bytes()
    gbs = alg_bytes / (ms_per_step * 1e-3) / 1e9

    # Dominant kernel: k_ring_reduce_sm, the stream-major ring reduction over long tiles (in the
    # default in-place mode the only other kernel is k_ring_reduce over the few short runs).
    #   achieved = algorithmic bytes of its launches (2*W*s per element they cover)
    #              / the sum of their durations, both counted by the library over the timed region
    es = 4 if wl.dtype == cm.F32 else 2
    lng, sml, seq = stats[cm.K_REDUCE], stats[cm.K_REDUCE_SMALL], stats[cm.K_SEQUENCE]
    per_elem = 2 * wl.world * es

    def kernel_line(st):
        if not st["launches"]:
            return None
        out = {"launches_per_step": st["launches"] / max(1, prof_steps),
               "bytes_per_launch": round(per_elem * st["elements"] / st["launches"])}
        if st["total_ms"] > 0:
            out["avg_launch_ms"] = round(st["total_ms"] / st["launches"], 6)
            out["achieved"] = round(per_elem * st["elements"] / (st["total_ms"] * 1e-3) / 1e9, 1)
        return out

    dom_name, dom = ("k_ring_reduce_sm", lng) if lng["elements"] >= sml["elements"] else ("k_ring_reduce", sml)
    dom_line = kernel_line(dom) or {}
    span_ms = seq["span_ms"] / max(1, seq["calls"])
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": dom_line.get("achieved"), "peak": HBM_PEAK_GBS,
                "unit": "GB/s",
                "frac": round(dom_line["achieved"] / HBM_PEAK_GBS, 4) if dom_line.get("achieved") else None,
                "traffic": read_traffic(wl.name),
                "launches_per_step": dom_line.get("launches_per_step"),
                "avg_launch_ms": dom_line.get("avg_launch_ms"), "bytes_per_launch": dom_line.get("bytes_per_launch"),
                "share_of_step_bytes": round(dom["elements"] / max(1, lng["elements"] + sml["elements"]), 4),
                "other_kernel": kernel_line(sml if dom is lng else lng),
                "step_span_ms": round(span_ms, 5) if seq["calls"] else None,
                "step_frac": round(gbs / HBM_PEAK_GBS, 4),
                "timed_region_event_ms_per_step": round(region_ms / args.steps, 5),
                "per_launch_event_steps": prof_steps}
    c_loop = {"host_us_per_call": round(host_us, 2), "stream_us_per_call": round(stream_us, 2),
              "GB/s_on_stream": round(alg_bytes / stream_us / 1e3, 1)}

    # staged route only: the pack and unpack kernels (k_copy) timed on their own; each moves the
    # batched parameters of every replica once: 2 * s bytes per small element and replica
    copy = None
    if args.batch_path == "staged":
        units = plan.units()
        small = sum(e.elems for e in plan.entries() if units[e.unit].kind == cm.KIND_BATCH)
        moved = 2 * small * es * wl.world
        copy = {"kernel": "k_copy", "bytes_per_call": moved}
        for label, fn in (("pack", plan.pack), ("unpack", plan.unpack)):
            best = None
            for _ in range(3):
                for _ in range(3):
                    fn(stream)
                torch.cuda.synchronize()
                c0 = time.perf_counter()
                for _ in range(30):
                    fn(stream)
                torch.cuda.synchronize()
                dt = (time.perf_counter() - c0) / 30
                best = dt if best is None else min(best, dt)
            copy[label] = {"ms": round(best * 1e3, 5), "GB/s": round(moved / best / 1e9, 1),
                           "frac": round(moved / best / 1e9 / HBM_PEAK_GBS, 4)}

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
        # one core: numpy's elementwise arithmetic is single-threaded, and the process is pinned
        allowed = os.sched_getaffinity(0)
        os.sched_setaffinity(0, {min(allowed)})
        try:
            for _ in range(args.cpu_repeats):
                c0 = time.perf_counter()
                oracle.allreduce(oplan, grads, fused)       # in place; speed does not depend on values
                times.append(time.perf_counter() - c0)
        finally:
            os.sched_setaffinity(0, allowed)
        med = sorted(times)[len(times) // 2]
        cpu = {"value": round(alg_bytes / med / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"the whole {wl.name} workload (W={wl.world}), pack+ring_reduce+unpack, "
                         f"pinned to one core, median of {args.cpu_repeats} passes, {med * 1e3:.0f} ms per pass"}
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
        "calls_issued_from_c": c_loop,
        "pack_unpack": copy,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    plan.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
