"""MI355X-native implementation of the hot path of Caramel's AllReduce aggregation.

The work is done by hand-written HIP kernels behind the C ABI declared in
include/caramel.h; this package only marshals arguments (binding.py) and, in
device.py, uses PyTorch to hold device memory and streams.
"""
from .binding import (BIN_BACKWARD, BIN_FORWARD, BATCH_DIRECT, BATCH_STAGED, BF16, F32, K_COUNT, K_PACK, K_REDUCE, K_REDUCE_SMALL, K_SEQUENCE, K_UNPACK,
                      KIND_BATCH, KIND_CHUNK, LAUNCH_AUTO, LAUNCH_PER_STREAM, LAUNCH_PER_UNIT, OPT_BATCH_PATH,
                      PATTERN_HALVING_DOUBLING, PATTERN_RING, PATTERN_SHUFFLE, OPT_BLOCK, OPT_LAUNCH_MIN_BYTES, OPT_LAUNCH_MODE, OPT_PIPELINE_MIN_BYTES, OPT_SMALL_TILE_VECS, OPT_SMALL_BLOCK, OPT_LONG_RUN_BYTES, OPT_STREAM_MAJOR, OPT_LONG_LAUNCH_MIN_BYTES, OPT_ALIGN_TILES, OPT_MERGE_SMALL_BYTES, OPT_TAIL_TILES, OPT_SPLIT_TILES, OPT_MAX_GRID, OPT_NONTEMPORAL, OPT_TILE_VECS, OPT_UNROLL,
                      SPLIT_ADAPTIVE, SPLIT_FIXED, SPLIT_NONE, STATIC_TABLE_BYTES, CaramelError, Config, Entry, Plan, ScheduleSummary, Slot,
                      Unit, lib, net_model_fit, schedule_transfers, stream_probe, threshold_estimate,
                      PROBE_COPY, PROBE_READ, PROBE_UPDATE, PROBE_WRITE)


# Functional spellings with the names of the C entry points.
def caramel_plan_create(world, elems, **kw) -> Plan:
    return Plan(world, elems, **kw)


def caramel_plan_create_timed(world, elems, ready_time, net_a, net_b, **kw) -> Plan:
    return Plan(world, elems, ready_time=ready_time, net_a=net_a, net_b=net_b, **kw)


def caramel_plan_times(plan: Plan):
    return plan.times()


def caramel_net_model_fit(bytes1, time1, bytes2, time2):
    return net_model_fit(bytes1, time1, bytes2, time2)


def caramel_threshold_estimate(a, b) -> int:
    return threshold_estimate(a, b)


def caramel_schedule_transfers(group_bytes, ready, need, bp_len, fp_len, net_a, net_b):
    return schedule_transfers(group_bytes, ready, need, bp_len, fp_len, net_a, net_b)


def caramel_plan_windows(plan: Plan, ready_time, read_time):
    return plan.windows(ready_time, read_time)


def caramel_plan_destroy(plan: Plan) -> None:
    plan.close()


def caramel_plan_counts(plan: Plan):
    return plan.counts()


def caramel_plan_units(plan: Plan):
    return plan.units()


def caramel_plan_entries(plan: Plan):
    return plan.entries()


def caramel_plan_segments(plan: Plan, unit: int):
    return plan.segments(unit)


def caramel_plan_serialize(plan: Plan) -> bytes:
    return plan.serialize()


def caramel_plan_set_option(plan: Plan, option: int, value: int) -> None:
    plan.set_option(option, value)


def caramel_bind(plan: Plan, grad_ptrs, fused_ws) -> None:
    plan.bind(grad_ptrs, fused_ws)


def caramel_pack(plan: Plan, stream: int = 0) -> None:
    plan.pack(stream)


def caramel_ring_reduce(plan: Plan, stream: int = 0) -> None:
    plan.ring_reduce(stream)


def caramel_unpack(plan: Plan, stream: int = 0) -> None:
    plan.unpack(stream)


def caramel_allreduce(plan: Plan, stream: int = 0) -> None:
    plan.allreduce(stream)


def caramel_allreduce_static(plan: Plan, grad_ptrs, stream: int = 0) -> None:
    plan.allreduce_static(grad_ptrs, stream)


def caramel_allreduce_loop(plan: Plan, n_calls: int, stream: int = 0):
    return plan.allreduce_loop(n_calls, stream)


def caramel_profile(plan: Plan, level: int) -> None:
    plan.profile(level)


def caramel_profile_read(plan: Plan):
    return plan.profile_read()


def caramel_stream_probe(mode, buffers, nbytes, run_bytes=4096, block=256, stream: int = 0) -> None:
    stream_probe(mode, buffers, nbytes, run_bytes, block, stream)


def caramel_version() -> int:
    return lib().caramel_version()
