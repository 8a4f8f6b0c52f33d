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


def halving_doubling_sim(xs: List[np.ndarray], granule: int = 4) -> List[np.ndarray]:
    """Recursive vector halving / distance doubling reduce-scatter followed by the mirrored
    all-gather, message by message, for a power-of-two number of workers.

    Step k = 0, 1, ...: partner = r XOR 2^k.  Each worker cuts its current range in two (on a
    granule boundary); the worker whose bit k is clear keeps the lower half and sends the upper
    one, its partner does the opposite; each adds what it receives to what it kept.  After
    log2(W) steps every worker holds the finished sum of its own final range, scales it by
    1/W, and the steps are replayed backwards with plain copies."""
    W = len(xs)
    assert W & (W - 1) == 0
    n = len(xs[0])
    buf = [np.array(x, dtype=np.float32, copy=True) for x in xs]
    inv_w = np.float32(1.0) / np.float32(W)
    rng = [(0, n) for _ in range(W)]
    history = []
    k = 1
    while k < W:
        new_rng = list(rng)
        msgs = []
        for r in range(W):
            lo, hi = rng[r]
            mid = lo + ((hi - lo) // 2 + granule - 1) // granule * granule
            mid = min(mid, hi)
            keep, send = ((lo, mid), (mid, hi)) if r & k == 0 else ((mid, hi), (lo, mid))
            msgs.append((r ^ k, send, buf[r][send[0]:send[1]].copy()))
            new_rng[r] = keep
        for dst, (a, b), payload in msgs:
            for i in range(a, b):
                buf[dst][i] = np.float32(buf[dst][i]) + np.float32(payload[i - a])
        history.append((k, rng))
        rng = new_rng
        k *= 2
    for r in range(W):
        a, b = rng[r]
        for i in range(a, b):
            buf[r][i] = np.float32(buf[r][i]) * inv_w
    for k, before in reversed(history):
        msgs = [(r ^ k, rng[r], buf[r][rng[r][0]:rng[r][1]].copy()) for r in range(W)]
        for dst, (a, b), payload in msgs:
            buf[dst][a:b] = payload
        rng = before
    return buf


def shuffle_sim(xs: List[np.ndarray], seg_start: List[int]) -> List[np.ndarray]:
    """Shuffle pattern: worker c receives slice c from every worker, adds the W pieces in
    worker order, scales, and sends the finished slice back to everybody."""
    W = len(xs)
    buf = [np.array(x, dtype=np.float32, copy=True) for x in xs]
    inv_w = np.float32(1.0) / np.float32(W)
    inbox = [[buf[src][seg_start[c]:seg_start[c + 1]].copy() for src in range(W)] for c in range(W)]
    done = []
    for c in range(W):
        pieces = inbox[c]
        acc = pieces[0].copy()
        for src in range(1, W):
            for i in range(len(acc)):
                acc[i] = np.float32(acc[i]) + np.float32(pieces[src][i])
        for i in range(len(acc)):
            acc[i] = np.float32(acc[i]) * inv_w
        done.append(acc)
    for c in range(W):
        for dst in range(W):
            buf[dst][seg_start[c]:seg_start[c + 1]] = done[c]
    return buf
