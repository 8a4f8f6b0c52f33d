"""CPU oracle, part 3: the ring pattern simulated message by message.

TEST INFRASTRUCTURE (see plan.py).  Tiny inputs only: pure-Python loops over
workers, steps and elements.

This follows the ring (bucket) algorithm as a protocol rather than as a formula
(paper section 2 names the pattern; section 4.4 describes its stages: data is
sent over the network, reduced by the receiving application, and the result is
sent on).  W workers hold private copies of a unit cut into W segments.

Reduce-scatter, steps t = 0 .. W-2, all workers at once:
    worker r sends its current copy of segment (r - 1 - t) mod W to worker r+1,
    which replaces its own copy of that segment by  received + own.
After W-1 steps worker c holds the complete sum of segment c; it multiplies by
1/W.  All-gather, steps t = 0 .. W-2:
    worker r sends segment (r - t) mod W to worker r+1, which overwrites its copy.

The direct formula in aggregate.py must give the same bits; a test checks that.
"""
from __future__ import annotations

from typing import List

import numpy as np


def ring_allreduce_sim(xs: List[np.ndarray], seg_start: List[int]) -> List[np.ndarray]:
    """xs[w]: float32 copy of the unit at worker w.  Returns the W final buffers."""
    W = len(xs)
    buf = [np.array(x, dtype=np.float32, copy=True) for x in xs]
    inv_w = np.float32(1.0) / np.float32(W)

    def seg(c):
        c %= W
        return slice(seg_start[c], seg_start[c + 1])

    for t in range(W - 1):
        # every worker posts its message before anyone applies what it received
        msgs = [(r, (r - 1 - t) % W, buf[r][seg(r - 1 - t)].copy()) for r in range(W)]
        for r, c, payload in msgs:
            dst = (r + 1) % W
            own = buf[dst][seg(c)]
            res = np.empty_like(own)
            for i in range(len(own)):
                res[i] = np.float32(payload[i]) + np.float32(own[i])
            buf[dst][seg(c)] = res
    for c in range(W):
        s = seg(c)
        for i in range(s.start, s.stop):
            buf[c][i] = np.float32(buf[c][i]) * inv_w
    for t in range(W - 1):
        msgs = [(r, (r - t) % W, buf[r][seg(r - t)].copy()) for r in range(W)]
        for r, c, payload in msgs:
            buf[(r + 1) % W][seg(c)] = payload
    return buf
