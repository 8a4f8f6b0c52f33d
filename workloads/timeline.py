"""Synthetic compute timeline of one training iteration, for the transfer scheduler.

The scheduler (paper section 4.3) needs, per parameter, the time in the backward pass at which
its gradient has been produced and the time in the next forward pass at which it is first read.
The paper takes both from traces of the real models; here they follow from a cost model in
which a layer's compute time grows with its parameter count: cost = elems + 1 % of the mean
tensor size (so that biases and norms take some time too), the forward pass visits tensors in
forward order, the backward pass in the reverse order at `bp_ratio` times the forward cost.

No arithmetic of the aggregation method lives here: the module only makes inputs, shared by the
CPU oracle's tests and the library's tests.
"""
from __future__ import annotations

from typing import List, Tuple

from .shapes import Workload


def compute_timeline(wl: Workload, fp_len: float = 100.0, bp_ratio: float = 2.0) -> Tuple[List[float], List[float], float, float]:
    """Returns (ready_time, read_time, bp_len, fp_len); both lists in UPDATE order (the order of
    `wl.elems()`), ready_time non-decreasing."""
    upd = wl.elems()                       # update order = reversed forward order
    fwd = list(reversed(upd))
    n = len(fwd)
    floor = 0.01 * sum(fwd) / n
    cost = [e + floor for e in fwd]
    scale = fp_len / sum(cost)
    read_fwd, acc = [], 0.0
    for c in cost:
        read_fwd.append(scale * acc)       # read when the layers before it are done
        acc += c
    ready_upd, acc = [], 0.0
    for f in range(n - 1, -1, -1):         # backward pass: last layer first
        acc += cost[f]
        ready_upd.append(bp_ratio * scale * acc)
    read_upd = [read_fwd[n - 1 - i] for i in range(n)]
    return ready_upd, read_upd, ready_upd[-1], fp_len
