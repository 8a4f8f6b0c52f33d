"""Seeded synthetic gradient values for the benchmark configurations.

Element j of tensor t at worker w is drawn from N(0, sigma_t); sigma_t is
log-uniform in [1e-4, 1e-1] and shared by all workers, which mimics gradients
whose scale differs from layer to layer.  Every (seed, worker, tensor) triple
owns a counter-based Philox stream, so any tensor of any replica can be
regenerated alone and in any order.

The module draws numbers only; it contains nothing of the aggregation method.
bf16 samples are the fp32 samples with the low 16 bits dropped (a plain bit
truncation, deliberately not the rounding rule the method itself applies to its
outputs).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import List, Sequence

import numpy as np

_SIGMA_STREAM = 0xFFFFFFFF


def _key(seed: int, worker: int, tensor: int) -> np.ndarray:
    return np.array([seed, (worker << 32) | tensor], dtype=np.uint64)


def sigma(seed: int, tensor: int) -> np.float32:
    g = np.random.Generator(np.random.Philox(key=_key(seed, _SIGMA_STREAM, tensor)))
    u = g.random()
    return np.float32(10.0 ** (-4.0 + 3.0 * u))


def tensor_values(seed: int, worker: int, tensor: int, n: int, bf16: bool = False) -> np.ndarray:
    """Values of one tensor of one replica: float32[n], or uint16[n] bf16 bit patterns."""
    g = np.random.Generator(np.random.Philox(key=_key(seed, worker, tensor)))
    x = g.standard_normal(n, dtype=np.float32)
    x *= sigma(seed, tensor)
    if bf16:
        return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return x


def replica_set(seed: int, world: int, elems: Sequence[int], bf16: bool = False,
                threads: int = 8) -> List[List[np.ndarray]]:
    """grads[w][t] for all workers and tensors (tensor index = position in `elems`)."""
    jobs = [(w, t) for w in range(world) for t in range(len(elems))]

    def make(job):
        w, t = job
        return tensor_values(seed, w, t, int(elems[t]), bf16)

    if threads > 1 and sum(elems) * world > (1 << 22):
        with ThreadPoolExecutor(max_workers=threads) as ex:
            flat = list(ex.map(make, jobs))
    else:
        flat = [make(j) for j in jobs]
    n = len(elems)
    return [flat[w * n:(w + 1) * n] for w in range(world)]
