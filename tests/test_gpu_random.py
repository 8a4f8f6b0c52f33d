"""Seeded random configurations on the GPU against the oracle, bit for bit: world size, dtype,
threshold, split rule, granule, streams, pattern, batch path, launch options, tensor sizes and the
placement of the replicas in memory are all drawn together, so that combinations no hand-written
case lists are met."""
import random

import numpy as np
import pytest

import oracle
import paper_2004_14020_amd as cm
from paper_2004_14020_amd.device import Replicas

from gpu_util import assert_same_bits, bits, lib_plan, make_inputs, oracle_result

pytestmark = pytest.mark.gpu

SIZES = [1, 2, 3, 5, 7, 8, 15, 16, 17, 63, 64, 100, 255, 256, 257, 1000, 1023, 1024, 1025, 4096, 5000, 16384,
         30011, 65536, 70000, 100000, 262144, 300001]


def draw(rng: random.Random):
    pattern = rng.choice([oracle.PATTERN_RING, oracle.PATTERN_RING, oracle.PATTERN_HALVING_DOUBLING,
                          oracle.PATTERN_SHUFFLE])
    if pattern == oracle.PATTERN_HALVING_DOUBLING:
        W = rng.choice([1, 2, 4, 8, 16, 32, 64])
    else:
        W = rng.choice([1, 2, 3, 4, 5, 7, 8, 8, 9, 12, 16, 16, 20, 33])
    dtype = rng.choice([oracle.F32, oracle.BF16])
    align = rng.choice([16, 16, 32, 64, 256])
    mode = rng.choice([oracle.SPLIT_NONE, oracle.SPLIT_FIXED, oracle.SPLIT_ADAPTIVE])
    S = rng.choice([1, 4, 16, 64]) * max(align, 1024)
    cfg = oracle.Config(W, dtype, rng.choice([0, 256, 4096, 65536, 1 << 20]), mode, rng.choice([1, 2, 8]), S, align,
                        rng.choice([1, 2]), pattern)
    elems = [rng.choice(SIZES) for _ in range(rng.randint(1, 16))]
    opts = {cm.OPT_BATCH_PATH: rng.choice([cm.BATCH_STAGED, cm.BATCH_DIRECT]),
            cm.OPT_LAUNCH_MODE: rng.choice([cm.LAUNCH_PER_UNIT, cm.LAUNCH_PER_STREAM, cm.LAUNCH_AUTO]),
            cm.OPT_PIPELINE_MIN_BYTES: rng.choice([0, 1 << 40]),
            cm.OPT_SMALL_TILE_VECS: rng.choice([64, 256, 1024]),
            cm.OPT_SMALL_BLOCK: rng.choice([256, 512, 1024]),
            cm.OPT_TILE_VECS: rng.choice([0, 512, 4096, 8192]),
            cm.OPT_BLOCK: rng.choice([256, 1024]),
            cm.OPT_LONG_RUN_BYTES: rng.choice([0, 1, 1024, 32768, 32768, 1 << 40]),
            cm.OPT_LONG_LAUNCH_MIN_BYTES: rng.choice([0, 200000, 64 << 20]),
            cm.OPT_STREAM_MAJOR: rng.choice([0, 2, 4, 8]),
            cm.OPT_MERGE_SMALL_BYTES: rng.choice([0, 1 << 20, 1 << 40]),
            cm.OPT_TAIL_TILES: rng.choice([0, 3, 256]),
            cm.OPT_ALIGN_TILES: rng.choice([0, 1, 2, 3]),
            cm.OPT_SPLIT_TILES: rng.choice([0, 1, 1]),
            cm.OPT_LAUNCH_MIN_BYTES: rng.choice([0, 65536, 4 << 20]),
            cm.OPT_NONTEMPORAL: rng.choice([0, 1]),
            cm.OPT_UNROLL: rng.choice([0, 1, 2, 4]),
            cm.OPT_MAX_GRID: rng.choice([0, 0, 7, 300])}
    place = dict(slot_align=rng.choice([256, 256, 4096]), large_align=rng.choice([256, 65536]),
                 large_bytes=rng.choice([65536, 1 << 20]),
                 arena_phase=rng.choice([None, 0, 256, 1536, 4096, 65536 - 256]))
    return cfg, elems, opts, place


@pytest.mark.parametrize("chunk", range(6))
def test_random_configurations(chunk):
    rng = random.Random(20041402 + chunk)
    for case in range(20):
        cfg, elems, opts, place = draw(rng)
        print(f"case: random chunk {chunk} case {case}: {cfg} elems={elems} opts={opts} place={place}", flush=True)
        grads = make_inputs(cfg, elems, seed=1000 * chunk + case)
        ref = oracle_result(cfg, elems, grads)
        plan = lib_plan(cfg, elems, opts)
        dev = Replicas(plan, elems, **place)
        dev.upload(grads)
        dev.fill_fused(0xA5)
        plan.allreduce()
        assert_same_bits(dev.download(), ref, f"chunk {chunk} case {case}")
        plan.close()
