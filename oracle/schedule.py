"""CPU oracle, part 4: the network transfer scheduler (paper section 4.3).

TEST INFRASTRUCTURE (see plan.py).  Plain Python, quadratic, tiny inputs and plan-sized
inputs only.

What is computed.  One training iteration offers the network two windows that run
in parallel with computation: the backward pass, of length `bp_len`, and the next
iteration's forward pass, of length `fp_len`.  A group of parameters (a transfer
unit made by the batcher) may not start before its transfer boundary in the
backward pass -- the moment the LAST of its members has been updated -- and must be
finished by its boundary in the forward pass -- the moment the FIRST of its members
is read.  The network carries one transfer at a time; a group of d bytes occupies it
for f(d) = a + b*d.

The scheduler is a greedy packing of these transfers into the two windows:

  1. Groups are taken in descending order of size (equal sizes: in queue order).
  2. Each group is tried in the backward pass first -- anywhere from its boundary to
     the end of the pass -- and, failing that, in the forward pass -- anywhere from
     the start of the pass to its boundary.  Groups that fit nowhere stay unassigned.
  3. The unassigned groups are taken again in the same order.  Now a transfer may run
     past the end of the backward pass, or before the start of the forward pass; both
     lengthen the iteration.  For either side the time it would add is computed and
     the side that adds less is taken.

Times of backward-pass slots count from the start of the backward pass, times of
forward-pass slots from the start of the forward pass (negative = before it).

Readings of what the section leaves open:
  * "anywhere" is resolved towards the group's own boundary: in the backward pass the
    earliest free start at or after the boundary, in the forward pass the latest free
    end at or before the boundary.  The two windows are then mirror images of each
    other, and stage 3's overrun grows away from the computation on both sides.
  * Transfers may touch but not overlap.
  * Added time: how far the slot pushes the end of the (already extended) backward
    window out, or the start of the (already extended) forward window back; a slot
    that fits a hole of the extended window adds nothing.  Equal cost: backward pass.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

from .plan import Plan

BIN_BACKWARD, BIN_FORWARD = 0, 1


@dataclass
class Slot:
    bin: int          # BIN_BACKWARD or BIN_FORWARD
    start: float
    end: float
    stage: int        # 2: placed beside computation; 3: placed with overrun allowed


@dataclass
class Schedule:
    slots: List[Slot]         # one per group, in the caller's group order
    comm_time: float          # N: sum of all transfer times
    compute_time: float       # C: bp_len + fp_len
    bp_overrun: float         # how far transfers run past the end of the backward pass
    fp_overrun: float         # how far before the start of the forward pass they begin
    iteration_time: float     # T = C + both overruns
    overlap: float            # alpha = (N + C - T) / min(N, C)   (section 3)
    utilization: float        # U = C / T


def group_windows(plan: Plan, ready_time: Sequence[float], read_time: Sequence[float]):
    """Bytes and transfer boundaries of every unit of a plan: a batch is bounded by its
    member that is updated last and by its member that is read first (section 4.3)."""
    es = plan.cfg.elem_size
    nbytes, ready, need = [], [], []
    for u in plan.units:
        members = [e.tensor for e in plan.entries[u.first_entry:u.first_entry + u.n_entries]]
        nbytes.append(u.elems * es)
        ready.append(max(ready_time[t] for t in members))
        need.append(min(read_time[t] for t in members))
    return nbytes, ready, need


def _free(placed: List[Slot], which: int, start: float, end: float) -> bool:
    return all(not (s.start < end and start < s.end) for s in placed if s is not None and s.bin == which)


def _earliest_start(placed, ready: float, dur: float, limit: float):
    """Backward pass: the smallest feasible start >= ready with end <= limit, else None.
    A feasible earliest start is either the boundary itself or the end of a placed slot."""
    cands = [float(ready)] + [s.end for s in placed if s is not None and s.bin == BIN_BACKWARD and s.end >= ready]
    good = [c for c in cands if c + dur <= limit and _free(placed, BIN_BACKWARD, c, c + dur)]
    return min(good) if good else None


def _latest_end(placed, need: float, dur: float, limit: float):
    """Forward pass: the largest feasible end <= need with start >= limit, else None."""
    cands = [float(need)] + [s.start for s in placed if s is not None and s.bin == BIN_FORWARD and s.start <= need]
    good = [c for c in cands if c - dur >= limit and _free(placed, BIN_FORWARD, c - dur, c)]
    return max(good) if good else None


def schedule_transfers(nbytes: Sequence[int], ready: Sequence[float], need: Sequence[float],
                       bp_len: float, fp_len: float, net_a: float, net_b: float) -> Schedule:
    n = len(nbytes)
    if not (len(ready) == n and len(need) == n):
        raise ValueError("one boundary pair per group")
    if not (bp_len >= 0.0 and fp_len >= 0.0 and net_a >= 0.0 and net_b >= 0.0):
        raise ValueError("lengths and model coefficients must be non-negative")
    for g in range(n):
        if not (0.0 <= ready[g] <= bp_len and 0.0 <= need[g] <= fp_len):
            raise ValueError("a boundary lies outside its pass")
    dur = [net_a + net_b * float(b) for b in nbytes]
    if any(not d > 0.0 for d in dur):
        raise ValueError("a transfer takes no time")
    inf = float("inf")

    order = sorted(range(n), key=lambda g: (-nbytes[g], g))
    slots: List[Slot] = [None] * n
    # stage 2: beside the computation
    for g in order:
        s = _earliest_start(slots, ready[g], dur[g], bp_len)
        if s is not None:
            slots[g] = Slot(BIN_BACKWARD, s, s + dur[g], 2)
            continue
        e = _latest_end(slots, need[g], dur[g], 0.0)
        if e is not None:
            slots[g] = Slot(BIN_FORWARD, e - dur[g], e, 2)
    # stage 3: what is left, overrun allowed
    for g in order:
        if slots[g] is not None:
            continue
        bp_end = max([bp_len] + [s.end for s in slots if s is not None and s.bin == BIN_BACKWARD])
        fp_begin = min([0.0] + [s.start for s in slots if s is not None and s.bin == BIN_FORWARD])
        s = _earliest_start(slots, ready[g], dur[g], inf)
        e = _latest_end(slots, need[g], dur[g], -inf)
        cost_bp = max(0.0, (s + dur[g]) - bp_end)
        cost_fp = max(0.0, fp_begin - (e - dur[g]))
        if cost_bp <= cost_fp:
            slots[g] = Slot(BIN_BACKWARD, s, s + dur[g], 3)
        else:
            slots[g] = Slot(BIN_FORWARD, e - dur[g], e, 3)

    comm = 0.0
    for d in dur:
        comm += d
    compute = bp_len + fp_len
    bp_over = max([bp_len] + [s.end for s in slots if s.bin == BIN_BACKWARD]) - bp_len
    fp_over = 0.0 - min([0.0] + [s.start for s in slots if s.bin == BIN_FORWARD])
    total = compute + bp_over + fp_over
    lesser = min(comm, compute)
    overlap = (comm + compute - total) / lesser if lesser > 0.0 else 0.0
    util = compute / total if total > 0.0 else 0.0
    return Schedule(slots, comm, compute, bp_over, fp_over, total, overlap, util)
