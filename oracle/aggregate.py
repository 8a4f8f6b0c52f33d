"""CPU oracle, part 2: pack, ring aggregation, unpack, and reference sums.

TEST INFRASTRUCTURE (see plan.py).  numpy, single thread, nothing blocked or
fused: each function is the definition written out.

Data model (paper section 2): W workers each hold an update of the same byte
length for every parameter, aggregation is addition, and after the barrier every
worker holds the aggregate.  `grads[w][t]` is worker w's 1-D array for tensor t
(float32, or uint16 holding bf16 bit patterns); everything is done in place.

Ring order.  In the ring (bucket) pattern the unit is cut into W segments; the
partial sum of segment c starts at worker c+1 and travels c+2, ..., wrapping
round, each worker adding its own contribution on arrival, until it reaches
worker c, which owns the result (reduce-scatter).  The owner scales by 1/W and
the finished segment travels round once more (all-gather).  Hence for every
element of segment c

    acc = x[c+1];  acc = fl32(acc + x[c+2]);  ...  acc = fl32(acc + x[c]);
    y   = fl32(acc * fl32(1/W))

with worker indices mod W.  bf16 inputs are widened exactly, all partial sums
stay in fp32, and y is rounded once, to nearest-even, on the way out.

Other patterns (paper sections 2 and 6.3 name them; only the order of the
additions differs, the segments, scaling and all-gather are the same):

* halving-doubling (recursive vector halving with distance doubling): in step k
  worker r exchanges one half of its current range with worker r XOR 2^k and adds
  what it receives to what it kept.  Every element therefore ends up as the
  balanced pairwise tree  ((x0+x1)+(x2+x3)) + ((x4+x5)+(x6+x7)) ...  whatever
  segment it lies in (fp addition is commutative, so who adds to whom is immaterial).
* shuffle: the owner of a slice receives that slice from every worker and sums the
  W pieces in worker order, x0 + x1 + ... + x(W-1), again the same for every slice.
"""
from __future__ import annotations

from typing import List

import numpy as np

from .plan import (BF16, F32, KIND_BATCH, PATTERN_HALVING_DOUBLING, PATTERN_RING, PATTERN_SHUFFLE, Plan)


# ---------------------------------------------------------------- bf16 <-> fp32
def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening: the bf16 pattern becomes the high half of the fp32 word."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16, ties to the even mantissa; NaN stays NaN (quiet)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (b >> np.uint64(16)) & np.uint64(1)
    r = ((b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, ((b >> np.uint64(16)) | np.uint64(0x0040)).astype(np.uint16), r)
    return r


def _np_dtype(plan: Plan):
    return np.float32 if plan.cfg.dtype == F32 else np.uint16


def new_fused(plan: Plan) -> np.ndarray:
    """A [W, fused_elems] workspace filled with a recognisable non-zero pattern."""
    buf = np.empty((plan.cfg.world, plan.fused_elems), dtype=_np_dtype(plan))
    buf.view(np.uint8)[...] = 0xA5
    return buf


# ---------------------------------------------------------------- pack / unpack
def pack(plan: Plan, grads: List[List[np.ndarray]], fused: np.ndarray) -> None:
    """Section 4.2: members of each batch are combined into one contiguous transfer.
    Alignment padding inside a batch is written as +0.0."""
    for u in plan.units:
        if u.kind != KIND_BATCH:
            continue
        for w in range(plan.cfg.world):
            region = fused[w, u.fused_off:u.fused_off + u.elems]
            region[...] = 0
            for e in plan.entries[u.first_entry:u.first_entry + u.n_entries]:
                region[e.unit_off:e.unit_off + e.elems] = \
                    grads[w][e.tensor][e.tensor_off:e.tensor_off + e.elems]


def unpack(plan: Plan, grads: List[List[np.ndarray]], fused: np.ndarray) -> None:
    """Inverse of pack; padding is never read."""
    for u in plan.units:
        if u.kind != KIND_BATCH:
            continue
        for w in range(plan.cfg.world):
            region = fused[w, u.fused_off:u.fused_off + u.elems]
            for e in plan.entries[u.first_entry:u.first_entry + u.n_entries]:
                grads[w][e.tensor][e.tensor_off:e.tensor_off + e.elems] = \
                    region[e.unit_off:e.unit_off + e.elems]


# ---------------------------------------------------------------- ring aggregation
def reduce_unit(xs: List[np.ndarray], seg_start: List[int], dtype: int, pattern: int = PATTERN_RING) -> None:
    """Reduce-scatter + scale + all-gather of one unit, in place.
    xs[w] is worker w's view of the unit; seg_start has W+1 element offsets."""
    W = len(xs)
    inv_w = np.float32(1.0) / np.float32(W)
    for c in range(W):
        a, b = seg_start[c], seg_start[c + 1]
        if a == b:
            continue

        def val(w):
            v = xs[w % W][a:b]
            return bf16_to_f32(v) if dtype == BF16 else v

        if pattern == PATTERN_RING:
            acc = val(c + 1).copy()
            for k in range(2, W + 1):
                acc = acc + val(c + k)          # fp32 + fp32 -> fp32, one rounding
        elif pattern == PATTERN_SHUFFLE:
            acc = val(0).copy()
            for w in range(1, W):
                acc = acc + val(w)
        elif pattern == PATTERN_HALVING_DOUBLING:
            part = [val(w) for w in range(W)]
            while len(part) > 1:                # neighbours first, then pairs of pairs, ...
                part = [part[i] + part[i + 1] for i in range(0, len(part), 2)]
            acc = part[0]
        else:
            raise ValueError("pattern")
        y = acc * inv_w
        out = f32_to_bf16_rne(y) if dtype == BF16 else y
        for w in range(W):
            xs[w][a:b] = out


def unit_views(plan: Plan, u, grads, fused) -> List[np.ndarray]:
    if u.kind == KIND_BATCH:
        return [fused[w, u.fused_off:u.fused_off + u.elems] for w in range(plan.cfg.world)]
    e = plan.entries[u.first_entry]
    return [grads[w][e.tensor][e.tensor_off:e.tensor_off + e.elems] for w in range(plan.cfg.world)]


def ring_reduce(plan: Plan, grads: List[List[np.ndarray]], fused: np.ndarray) -> None:
    """All units: batch units on the fused buffers, chunk units on tensor memory."""
    for u in plan.units:
        reduce_unit(unit_views(plan, u, grads, fused), u.seg_start, plan.cfg.dtype, plan.cfg.pattern)


def allreduce(plan: Plan, grads: List[List[np.ndarray]], fused: np.ndarray = None) -> None:
    """pack -> ring_reduce -> unpack; afterwards every replica holds the average."""
    if fused is None:
        fused = new_fused(plan)
    pack(plan, grads, fused)
    ring_reduce(plan, grads, fused)
    unpack(plan, grads, fused)


# ---------------------------------------------------------------- references
def mean_f64(plan: Plan, grads: List[List[np.ndarray]], t: int) -> np.ndarray:
    """Double-precision mean over workers of tensor t, summed in worker order."""
    acc = np.zeros(grads[0][t].shape, dtype=np.float64)
    for w in range(plan.cfg.world):
        v = grads[w][t]
        acc += (bf16_to_f32(v) if plan.cfg.dtype == BF16 else v).astype(np.float64)
    return acc / plan.cfg.world


def abs_sum_f64(plan: Plan, grads: List[List[np.ndarray]], t: int) -> np.ndarray:
    acc = np.zeros(grads[0][t].shape, dtype=np.float64)
    for w in range(plan.cfg.world):
        v = grads[w][t]
        acc += np.abs((bf16_to_f32(v) if plan.cfg.dtype == BF16 else v).astype(np.float64))
    return acc
