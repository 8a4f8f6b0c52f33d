"""Pins for the halving-doubling and shuffle summation orders (paper sections 2 and 6.3), CPU only."""
import json
import os

import numpy as np
import pytest

import oracle
from oracle import (BF16, F32, PATTERN_HALVING_DOUBLING, PATTERN_RING, PATTERN_SHUFFLE, Config, build_plan)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def wide(rng, n):
    return (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 6, n)).astype(np.float32)


def test_worked_example_values():
    with open(os.path.join(GOLDEN, "ring_worked_examples.json")) as f:
        ex = json.load(f)["other_patterns"][0]
    n = 52
    for pattern, key in ((PATTERN_HALVING_DOUBLING, "halving_doubling"), (PATTERN_SHUFFLE, "shuffle")):
        grads = [[np.full(n, g, dtype=np.float32)] for g in ex["g"]]
        plan = build_plan(Config(ex["world"], F32, 0, pattern=pattern), [n])
        oracle.allreduce(plan, grads)
        for w in range(ex["world"]):
            assert (grads[w][0] == np.float32(ex[key])).all()


@pytest.mark.parametrize("W", [1, 2, 4, 8, 16, 32, 64])
def test_halving_doubling_formula_equals_protocol_simulation(W):
    rng = np.random.default_rng(W)
    for n in (4, 5, 16, 64, 67, 4 * W * 3 + 1):
        xs = [wide(rng, n) for _ in range(W)]
        sim = oracle.halving_doubling_sim(xs)
        got = [x.copy() for x in xs]
        oracle.reduce_unit(got, oracle.ring_segments(Config(W), n), F32, PATTERN_HALVING_DOUBLING)
        for w in range(W):
            assert np.array_equal(sim[w].view(np.uint32), got[w].view(np.uint32))


@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 8, 16])
def test_shuffle_formula_equals_protocol_simulation(W):
    rng = np.random.default_rng(100 + W)
    for n in (3, 16, 64, 67, 4 * W * 3 + 1):
        seg = oracle.ring_segments(Config(W), n)
        xs = [wide(rng, n) for _ in range(W)]
        sim = oracle.shuffle_sim(xs, seg)
        got = [x.copy() for x in xs]
        oracle.reduce_unit(got, seg, F32, PATTERN_SHUFFLE)
        for w in range(W):
            assert np.array_equal(sim[w].view(np.uint32), got[w].view(np.uint32))


def test_the_three_orders_differ_in_bits_but_agree_within_the_bound():
    W, n = 8, 4096
    rng = np.random.default_rng(0)
    xs = [wide(rng, n) for _ in range(W)]
    res = {}
    for p in (PATTERN_RING, PATTERN_HALVING_DOUBLING, PATTERN_SHUFFLE):
        got = [x.copy() for x in xs]
        oracle.reduce_unit(got, oracle.ring_segments(Config(W), n), F32, p)
        res[p] = got[0]
    assert (res[PATTERN_RING] != res[PATTERN_SHUFFLE]).any()
    assert (res[PATTERN_HALVING_DOUBLING] != res[PATTERN_SHUFFLE]).any()
    mean = sum(x.astype(np.float64) for x in xs) / W
    mag = sum(np.abs(x.astype(np.float64)) for x in xs)
    for p in res:
        assert (np.abs(res[p] - mean) <= 4e-7 * mag).all()


@pytest.mark.parametrize("pattern", [PATTERN_HALVING_DOUBLING, PATTERN_SHUFFLE])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_integer_inputs_are_exact_in_every_order(pattern, dtype):
    W, elems = 8, [10, 700, 33, 5000]
    rng = np.random.default_rng(3)
    ints = [[rng.integers(-7, 8, n) * W for n in elems] for _ in range(W)]
    if dtype == F32:
        grads = [[a.astype(np.float32) for a in row] for row in ints]
    else:
        grads = [[oracle.f32_to_bf16_rne(a.astype(np.float32)) for a in row] for row in ints]
    plan = build_plan(Config(W, dtype, 2048, oracle.SPLIT_FIXED, 8, 4096, pattern=pattern), elems)
    oracle.allreduce(plan, grads)
    for t in range(len(elems)):
        mean = sum(ints[w][t] for w in range(W)) / W
        got = grads[0][t] if dtype == F32 else oracle.bf16_to_f32(grads[0][t])
        assert np.array_equal(got.astype(np.float64), mean)


def test_halving_doubling_needs_a_power_of_two():
    for W in (3, 5, 24, 48):
        with pytest.raises(ValueError):
            build_plan(Config(W, F32, 0, pattern=PATTERN_HALVING_DOUBLING), [16])
    with pytest.raises(ValueError):
        build_plan(Config(4, F32, 0, pattern=7), [16])
