"""Shared helpers of the GPU parity tests (not collected by pytest)."""
from __future__ import annotations

import numpy as np

import oracle
import paper_2004_14020_amd as cm
from paper_2004_14020_amd.device import Replicas
from workloads import gradients


def lib_plan(cfg: oracle.Config, elems, opts: dict = None) -> cm.Plan:
    p = cm.Plan(cfg.world, elems, dtype=cfg.dtype, batch_threshold_bytes=cfg.batch_threshold_bytes,
                split_mode=cfg.split_mode, split_bytes=cfg.split_bytes, max_depth=cfg.max_depth,
                align_bytes=cfg.align_bytes, num_streams=cfg.num_streams, pattern=cfg.pattern)
    for k, v in (opts or {}).items():
        p.set_option(k, v)
    return p


def clone(grads):
    return [[a.copy() for a in row] for row in grads]


def bits(a: np.ndarray) -> np.ndarray:
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


def assert_same_bits(got, ref, what=""):
    for w, (grow, rrow) in enumerate(zip(got, ref)):
        for t, (g, r) in enumerate(zip(grow, rrow)):
            if not np.array_equal(bits(g), bits(r)):
                bad = np.flatnonzero(bits(g) != bits(r))
                raise AssertionError(f"{what}: replica {w} tensor {t}: {bad.size} of {g.size} elements differ, "
                                     f"first at {bad[0]}: got {g[bad[0]]!r} want {r[bad[0]]!r}")


def make_inputs(cfg: oracle.Config, elems, seed: int):
    return gradients.replica_set(seed, cfg.world, list(elems), bf16=(cfg.dtype == oracle.BF16))


def oracle_result(cfg: oracle.Config, elems, grads):
    plan = oracle.build_plan(cfg, list(elems))
    ref = clone(grads)
    oracle.allreduce(plan, ref)
    return ref
