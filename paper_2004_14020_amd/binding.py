"""ctypes binding of libcaramel.so: argument marshalling only.

Every step of the path (plan, pack, ring reduce, unpack, pipeline) runs inside the
library.  There is no fallback: if the shared library is missing or a call fails,
an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcaramel.so")

OK, EINVAL, ENOMEM, EHIP, ESTATE = 0, 1, 2, 3, 4
BIN_BACKWARD, BIN_FORWARD = 0, 1
F32, BF16 = 0, 1
SPLIT_NONE, SPLIT_FIXED, SPLIT_ADAPTIVE = 0, 1, 2
KIND_BATCH, KIND_CHUNK = 0, 1
PATTERN_RING, PATTERN_HALVING_DOUBLING, PATTERN_SHUFFLE = 0, 1, 2
(OPT_LAUNCH_MODE, OPT_BATCH_PATH, OPT_TILE_VECS, OPT_MAX_GRID, OPT_NONTEMPORAL, OPT_UNROLL, OPT_BLOCK,
 OPT_LAUNCH_MIN_BYTES, OPT_PIPELINE_MIN_BYTES, OPT_SMALL_TILE_VECS, OPT_SMALL_BLOCK, OPT_LONG_RUN_BYTES,
 OPT_STREAM_MAJOR, OPT_LONG_LAUNCH_MIN_BYTES, OPT_ALIGN_TILES, OPT_MERGE_SMALL_BYTES, OPT_TAIL_TILES, OPT_SPLIT_TILES) = range(18)
STATIC_TABLE_BYTES = 4 << 20
LAUNCH_PER_UNIT, LAUNCH_PER_STREAM, LAUNCH_AUTO = 0, 1, 2
BATCH_STAGED, BATCH_DIRECT = 0, 1
K_PACK, K_REDUCE, K_UNPACK, K_SEQUENCE, K_REDUCE_SMALL, K_COUNT = 0, 1, 2, 3, 4, 5

EXPORTS = (
    "caramel_plan_create", "caramel_plan_create_timed", "caramel_plan_times", "caramel_net_model_fit",
    "caramel_threshold_estimate", "caramel_schedule_transfers", "caramel_plan_windows", "caramel_plan_destroy", "caramel_plan_counts", "caramel_plan_units",
    "caramel_plan_entries", "caramel_plan_segments", "caramel_plan_serialize", "caramel_bind",
    "caramel_pack", "caramel_ring_reduce", "caramel_unpack", "caramel_allreduce", "caramel_allreduce_static",
    "caramel_plan_set_option", "caramel_profile", "caramel_profile_read", "caramel_last_error",
    "caramel_version", "caramel_stream_probe", "caramel_allreduce_loop",
)


class Config(C.Structure):
    _fields_ = [("world", C.c_uint32), ("dtype", C.c_uint32), ("batch_threshold_bytes", C.c_uint64),
                ("split_mode", C.c_uint32), ("max_depth", C.c_uint32), ("split_bytes", C.c_uint64),
                ("align_bytes", C.c_uint32), ("num_streams", C.c_uint32), ("pattern", C.c_uint32),
                ("reserved", C.c_uint32)]


class Unit(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("stream", C.c_uint32), ("first_entry", C.c_uint32),
                ("n_entries", C.c_uint32), ("elems", C.c_uint64), ("fused_off", C.c_uint64)]


class Entry(C.Structure):
    _fields_ = [("tensor", C.c_uint32), ("unit", C.c_uint32), ("tensor_off", C.c_uint64),
                ("unit_off", C.c_uint64), ("elems", C.c_uint64)]


class Slot(C.Structure):
    _fields_ = [("bin", C.c_uint32), ("stage", C.c_uint32), ("start", C.c_double), ("end", C.c_double)]


class ScheduleSummary(C.Structure):
    _fields_ = [("comm_time", C.c_double), ("compute_time", C.c_double), ("bp_overrun", C.c_double),
                ("fp_overrun", C.c_double), ("iteration_time", C.c_double), ("overlap", C.c_double),
                ("utilization", C.c_double)]


class KernelStat(C.Structure):
    _fields_ = [("launches", C.c_uint64), ("total_ms", C.c_double), ("span_ms", C.c_double),
                ("calls", C.c_uint64), ("elements", C.c_uint64)]


class CaramelError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"caramel status {status}: {message}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2004_14020_amd.build`")
    # PyTorch ships its own HIP runtime, and a process can only initialise one.  Importing torch
    # first makes the library's dependency on libamdhip64 resolve to the copy torch has loaded,
    # so device pointers and streams made by torch are valid inside the library.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    P = C.c_void_p
    L.caramel_plan_create.argtypes = [C.POINTER(Config), C.POINTER(C.c_uint64), C.c_uint32, C.POINTER(P)]
    L.caramel_plan_create_timed.argtypes = [C.POINTER(Config), C.POINTER(C.c_uint64), C.c_uint32,
                                            C.POINTER(C.c_double), C.c_double, C.c_double, C.POINTER(P)]
    L.caramel_plan_times.argtypes = [P, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_uint32]
    L.caramel_net_model_fit.argtypes = [C.c_uint64, C.c_double, C.c_uint64, C.c_double,
                                        C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.caramel_threshold_estimate.argtypes = [C.c_double, C.c_double, C.POINTER(C.c_uint64)]
    D = C.POINTER(C.c_double)
    L.caramel_schedule_transfers.argtypes = [C.POINTER(C.c_uint64), D, D, C.c_uint32, C.c_double, C.c_double,
                                             C.c_double, C.c_double, C.POINTER(Slot), C.POINTER(ScheduleSummary)]
    L.caramel_plan_windows.argtypes = [P, D, D, C.POINTER(C.c_uint64), D, D, C.c_uint32]
    L.caramel_plan_destroy.argtypes = [P]
    L.caramel_plan_destroy.restype = None
    L.caramel_plan_counts.argtypes = [P, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)]
    L.caramel_plan_units.argtypes = [P, C.POINTER(Unit), C.c_uint32]
    L.caramel_plan_entries.argtypes = [P, C.POINTER(Entry), C.c_uint32]
    L.caramel_plan_segments.argtypes = [P, C.c_uint32, C.POINTER(C.c_uint64)]
    L.caramel_plan_serialize.argtypes = [P, P, C.POINTER(C.c_size_t)]
    L.caramel_bind.argtypes = [P, C.POINTER(P), P]
    for name in ("caramel_pack", "caramel_ring_reduce", "caramel_unpack", "caramel_allreduce"):
        getattr(L, name).argtypes = [P, P]
    L.caramel_allreduce_static.argtypes = [P, C.POINTER(P), P]
    L.caramel_plan_set_option.argtypes = [P, C.c_uint32, C.c_uint64]
    L.caramel_profile.argtypes = [P, C.c_int]
    L.caramel_profile_read.argtypes = [P, C.POINTER(KernelStat)]
    L.caramel_last_error.restype = C.c_char_p
    L.caramel_last_error.argtypes = []
    L.caramel_version.argtypes = []
    L.caramel_allreduce_loop.argtypes = [P, P, C.c_uint32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.caramel_stream_probe.argtypes = [C.c_uint32, C.POINTER(P), C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, P]
    _lib = L
    return L


def _check(status: int) -> None:
    if status != OK:
        raise CaramelError(status, lib().caramel_last_error().decode())


class Plan:
    """Owner of one caramel_plan handle."""

    def __init__(self, world: int, elems: Sequence[int], dtype: int = F32, batch_threshold_bytes: int = 0,
                 split_mode: int = SPLIT_NONE, split_bytes: int = 0, max_depth: int = 8,
                 align_bytes: int = 16, num_streams: int = 2, ready_time: Optional[Sequence[float]] = None,
                 net_a: float = 0.0, net_b: float = 0.0, pattern: int = PATTERN_RING):
        self._h = C.c_void_p()
        self.cfg = Config(world, dtype, batch_threshold_bytes, split_mode, max_depth, split_bytes,
                          align_bytes, num_streams, pattern, 0)
        self.n_tensors = len(elems)
        arr = (C.c_uint64 * max(1, len(elems)))(*[int(e) for e in elems])
        if ready_time is None:
            _check(lib().caramel_plan_create(C.byref(self.cfg), arr, len(elems), C.byref(self._h)))
        else:
            if len(ready_time) != len(elems):
                raise ValueError("ready_time must have one entry per tensor")
            rt = (C.c_double * max(1, len(elems)))(*[float(t) for t in ready_time])
            _check(lib().caramel_plan_create_timed(C.byref(self.cfg), arr, len(elems), rt, float(net_a),
                                                   float(net_b), C.byref(self._h)))

    # -- lifetime
    def close(self) -> None:
        if self._h:
            lib().caramel_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- introspection
    def counts(self):
        nu, ne, fe = C.c_uint32(), C.c_uint32(), C.c_uint64()
        _check(lib().caramel_plan_counts(self._h, C.byref(nu), C.byref(ne), C.byref(fe)))
        return nu.value, ne.value, fe.value

    @property
    def fused_elems(self) -> int:
        return self.counts()[2]

    def units(self) -> List[Unit]:
        n = self.counts()[0]
        buf = (Unit * max(1, n))()
        _check(lib().caramel_plan_units(self._h, buf, n))
        return list(buf[:n])

    def entries(self) -> List[Entry]:
        n = self.counts()[1]
        buf = (Entry * max(1, n))()
        _check(lib().caramel_plan_entries(self._h, buf, n))
        return list(buf[:n])

    def segments(self, unit: int) -> List[int]:
        buf = (C.c_uint64 * (self.cfg.world + 1))()
        _check(lib().caramel_plan_segments(self._h, unit, buf))
        return list(buf)

    def times(self):
        """(enqueue, start, finish) lists of a timing-aware plan."""
        n = self.counts()[0]
        bufs = [(C.c_double * max(1, n))() for _ in range(3)]
        _check(lib().caramel_plan_times(self._h, bufs[0], bufs[1], bufs[2], n))
        return tuple(list(b[:n]) for b in bufs)

    def windows(self, ready_time: Sequence[float], read_time: Sequence[float]):
        """(bytes, ready, need) lists, one entry per unit: the units' transfer boundaries."""
        if len(ready_time) != self.n_tensors or len(read_time) != self.n_tensors:
            raise ValueError("one update time and one read time per tensor")
        n = self.counts()[0]
        rt = (C.c_double * max(1, self.n_tensors))(*[float(t) for t in ready_time])
        rd = (C.c_double * max(1, self.n_tensors))(*[float(t) for t in read_time])
        b = (C.c_uint64 * max(1, n))()
        r, d = (C.c_double * max(1, n))(), (C.c_double * max(1, n))()
        _check(lib().caramel_plan_windows(self._h, rt, rd, b, r, d, n))
        return list(b[:n]), list(r[:n]), list(d[:n])

    def serialize(self) -> bytes:
        n = C.c_size_t(0)
        _check(lib().caramel_plan_serialize(self._h, None, C.byref(n)))
        buf = C.create_string_buffer(n.value)
        _check(lib().caramel_plan_serialize(self._h, buf, C.byref(n)))
        return buf.raw[:n.value]

    # -- device
    def set_option(self, option: int, value: int) -> None:
        _check(lib().caramel_plan_set_option(self._h, option, value))

    def bind(self, grad_ptrs: Sequence[Sequence[int]], fused_ws: Optional[int]) -> None:
        """grad_ptrs[w][t]: device address of worker w's tensor t; fused_ws: device address or None."""
        W, n = self.cfg.world, self.n_tensors
        if len(grad_ptrs) != W or any(len(r) != n for r in grad_ptrs):
            raise ValueError("grad_ptrs must be world x n_tensors")
        flat = (C.c_void_p * (W * n))(*[int(grad_ptrs[w][t]) for w in range(W) for t in range(n)])
        _check(lib().caramel_bind(self._h, flat, C.c_void_p(fused_ws or 0)))

    def pack(self, stream: int = 0) -> None:
        _check(lib().caramel_pack(self._h, C.c_void_p(stream)))

    def ring_reduce(self, stream: int = 0) -> None:
        _check(lib().caramel_ring_reduce(self._h, C.c_void_p(stream)))

    def unpack(self, stream: int = 0) -> None:
        _check(lib().caramel_unpack(self._h, C.c_void_p(stream)))

    def allreduce(self, stream: int = 0) -> None:
        _check(lib().caramel_allreduce(self._h, C.c_void_p(stream)))

    def allreduce_static(self, grad_ptrs: Sequence[Sequence[int]], stream: int = 0) -> None:
        """caramel_allreduce_static: grad_ptrs as for bind; no device allocation inside the call."""
        W, n = self.cfg.world, self.n_tensors
        if len(grad_ptrs) != W or any(len(r) != n for r in grad_ptrs):
            raise ValueError("grad_ptrs must be world x n_tensors")
        flat = (C.c_void_p * (W * n))(*[int(grad_ptrs[w][t]) for w in range(W) for t in range(n)])
        _check(lib().caramel_allreduce_static(self._h, flat, C.c_void_p(stream)))

    def allreduce_loop(self, n_calls: int, stream: int = 0):
        """(host microseconds to issue one call, microseconds one call takes on the stream)."""
        host, dev = C.c_double(), C.c_double()
        _check(lib().caramel_allreduce_loop(self._h, C.c_void_p(stream), n_calls, C.byref(host), C.byref(dev)))
        return host.value, dev.value

    def profile(self, level: int) -> None:
        _check(lib().caramel_profile(self._h, int(level)))

    def profile_read(self):
        buf = (KernelStat * K_COUNT)()
        _check(lib().caramel_profile_read(self._h, buf))
        return [dict(launches=s.launches, total_ms=s.total_ms, span_ms=s.span_ms, calls=s.calls, elements=s.elements)
                for s in buf]


PROBE_READ, PROBE_WRITE, PROBE_UPDATE, PROBE_COPY = 0, 1, 2, 3


def stream_probe(mode: int, buffers: Sequence[int], nbytes: int, run_bytes: int = 4096, block: int = 256,
                 stream: int = 0) -> None:
    """caramel_stream_probe: a plain streaming kernel over the given device buffers."""
    arr = (C.c_void_p * len(buffers))(*[int(b) for b in buffers])
    st = lib().caramel_stream_probe(mode, arr, len(buffers), nbytes, run_bytes, block, C.c_void_p(stream))
    if st != OK:
        raise CaramelError(st, "caramel_stream_probe: bad arguments" if st == EINVAL else "caramel_stream_probe: launch failed")


def net_model_fit(bytes1: int, time1: float, bytes2: int, time2: float):
    a, b = C.c_double(), C.c_double()
    _check(lib().caramel_net_model_fit(bytes1, time1, bytes2, time2, C.byref(a), C.byref(b)))
    return a.value, b.value


def schedule_transfers(group_bytes: Sequence[int], ready: Sequence[float], need: Sequence[float], bp_len: float,
                       fp_len: float, net_a: float, net_b: float):
    """(slots, summary): one Slot per group in the caller's order, and the schedule's totals."""
    n = len(group_bytes)
    if len(ready) != n or len(need) != n:
        raise ValueError("one boundary pair per group")
    b = (C.c_uint64 * max(1, n))(*[int(x) for x in group_bytes])
    r = (C.c_double * max(1, n))(*[float(x) for x in ready])
    d = (C.c_double * max(1, n))(*[float(x) for x in need])
    slots = (Slot * max(1, n))()
    summary = ScheduleSummary()
    _check(lib().caramel_schedule_transfers(b, r, d, n, float(bp_len), float(fp_len), float(net_a), float(net_b),
                                            slots, C.byref(summary)))
    return list(slots[:n]), summary


def threshold_estimate(a: float, b: float) -> int:
    out = C.c_uint64()
    _check(lib().caramel_threshold_estimate(a, b, C.byref(out)))
    return out.value
