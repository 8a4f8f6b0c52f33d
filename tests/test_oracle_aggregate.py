"""Pins for the oracle's pack / ring aggregation / unpack (CPU only).

None of these compares the oracle with itself: the ring order is pinned by a
message-by-message simulation of the ring protocol and by hand-worked examples,
the sums by cases whose exact result is known (integers, powers of two, equal
replicas), the accuracy by a float64 sum, and the bf16 rounding by the
definition of round-to-nearest-even and by an independent library conversion.
"""
import json
import os
import random

import numpy as np
import pytest

import oracle
from oracle import BF16, F32, KIND_BATCH, SPLIT_FIXED, SPLIT_NONE, Config, build_plan
from workloads import gradients
from workloads.shapes import workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def clone(grads):
    return [[a.copy() for a in row] for row in grads]


def small_case(seed=3, W=4, dtype=F32, T=2048, mode=SPLIT_FIXED, S=4096,
               elems=(10, 700, 33, 5000, 1, 257, 3000, 64, 129)):
    cfg = Config(W, dtype, T, mode, 8, S, 16, 2)
    plan = build_plan(cfg, list(elems))
    grads = gradients.replica_set(seed, W, list(elems), bf16=(dtype == BF16))
    return cfg, plan, grads


# ------------------------------------------------------------------ pack / unpack
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_pack_then_unpack_is_identity_and_padding_is_zero(dtype):
    cfg, plan, grads = small_case(dtype=dtype)
    fused = oracle.new_fused(plan)
    before = clone(grads)
    oracle.pack(plan, grads, fused)
    # members landed where the plan says
    covered = np.zeros(plan.fused_elems, dtype=bool)
    for u in plan.units:
        if u.kind != KIND_BATCH:
            continue
        for e in plan.entries[u.first_entry:u.first_entry + u.n_entries]:
            a = u.fused_off + e.unit_off
            covered[a:a + e.elems] = True
            for w in range(cfg.world):
                assert np.array_equal(fused[w, a:a + e.elems], before[w][e.tensor])
    # every other element of the workspace is +0.0 (all bits clear)
    assert (~covered).any()
    for w in range(cfg.world):
        assert not fused[w, ~covered].view(np.uint8).any()
    # wipe the tensors, unpack, and get the originals back bit for bit
    for row in grads:
        for a in row:
            a.view(np.uint8)[...] = 0x5A
    oracle.unpack(plan, grads, fused)
    for w in range(cfg.world):
        for t, a in enumerate(grads[w]):
            is_small = any(e.tensor == t and plan.units[e.unit].kind == KIND_BATCH for e in plan.entries)
            if is_small:
                assert np.array_equal(a.view(np.uint8), before[w][t].view(np.uint8))
            else:
                assert (a.view(np.uint8) == 0x5A).all()      # large tensors untouched


def test_pack_places_position_codes():
    # each element carries (tensor, index); after pack the fused buffer reads back the plan
    elems = [5, 9, 100, 3, 41]
    cfg = Config(2, F32, 1 << 20)
    plan = build_plan(cfg, elems)
    grads = [[(t * 1000 + np.arange(n)).astype(np.float32) + w * 0.5 for t, n in enumerate(elems)]
             for w in range(2)]
    fused = oracle.new_fused(plan)
    oracle.pack(plan, grads, fused)
    at = 0
    for t, n in enumerate(elems):
        at = (at + 3) // 4 * 4
        assert np.array_equal(fused[1, at:at + n], t * 1000 + np.arange(n) + 0.5)
        at += n


# ------------------------------------------------------------------ ring order
def test_worked_examples():
    with open(os.path.join(GOLDEN, "ring_worked_examples.json")) as f:
        gold = json.load(f)
    for ex in gold["examples"]:
        W = ex["world"]
        cfg = Config(W, F32, 0)
        n = 4 * W * 3 + 4           # 13 granules: segments of 4,3,3,3
        plan = build_plan(cfg, [n])
        grads = [[np.full(n, g, dtype=np.float32)] for g in ex["g"]]
        oracle.allreduce(plan, grads)
        seg = plan.units[0].seg_start
        for w in range(W):
            for c in range(W):
                assert (grads[w][0][seg[c]:seg[c + 1]] == np.float32(ex["segment_outputs"][c])).all()


@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 8, 16])
def test_formula_equals_message_passing_simulation(W):
    rng = np.random.default_rng(W)
    cfg = Config(W, F32, 0)
    for granules in list(range(0, 3 * W + 6, max(1, W // 3))) + [3 * W + 5]:
        for tail in (0, 1, 3):
            n = granules * 4 + tail
            if n == 0:
                continue
            seg = oracle.ring_segments(cfg, n)
            # wide dynamic range so that the order of additions matters
            xs = [(rng.standard_normal(n) * 10.0 ** rng.integers(-6, 6, n)).astype(np.float32)
                  for _ in range(W)]
            sim = oracle.ring_allreduce_sim(xs, seg)
            got = [x.copy() for x in xs]
            oracle.reduce_unit(got, seg, F32)
            for w in range(W):
                assert np.array_equal(sim[w].view(np.uint32), got[w].view(np.uint32))
                assert np.array_equal(got[w], got[0])


def test_rotation_matters_in_the_random_case():
    # guards the test above: with these inputs a different start worker changes bits
    W, n = 8, 4096
    rng = np.random.default_rng(0)
    xs = [(rng.standard_normal(n) * 10.0 ** rng.integers(-6, 6, n)).astype(np.float32) for _ in range(W)]
    a = [x.copy() for x in xs]
    oracle.reduce_unit(a, oracle.ring_segments(Config(W), n), F32)
    plain = xs[0].copy()
    for w in range(1, W):
        plain = plain + xs[w]
    plain = plain * np.float32(1.0 / W)
    assert (a[0] != plain).any()


# ------------------------------------------------------------------ exact sums
@pytest.mark.parametrize("W", [2, 4, 8, 16])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_integer_inputs_give_exact_mean(W, dtype):
    elems = [10, 700, 33, 5000, 257]
    cfg = Config(W, dtype, 2048, SPLIT_FIXED, 8, 4096)
    plan = build_plan(cfg, elems)
    rng = np.random.default_rng(W)
    if dtype == F32:
        ints = [[rng.integers(-60000, 60000, n) for n in elems] for _ in range(W)]
        grads = [[a.astype(np.float32) for a in row] for row in ints]
    else:
        # multiples of W in [-128, 127]*W are exact in bf16 and so are their means
        ints = [[rng.integers(-7, 8, n) * W for n in elems] for _ in range(W)]
        grads = [[oracle.f32_to_bf16_rne(a.astype(np.float32)) for a in row] for row in ints]
    oracle.allreduce(plan, grads)
    for t, n in enumerate(elems):
        mean = sum(ints[w][t] for w in range(W)) / W
        for w in range(W):
            got = grads[w][t] if dtype == F32 else oracle.bf16_to_f32(grads[w][t])
            assert np.array_equal(got.astype(np.float64), mean)


def test_power_of_two_scaling_commutes():
    cfg, plan, grads = small_case(seed=5, W=8)
    scaled = [[a * np.float32(2.0 ** -9) for a in row] for row in grads]
    oracle.allreduce(plan, grads)
    oracle.allreduce(plan, scaled)
    for t in range(len(grads[0])):
        assert np.array_equal(grads[0][t] * np.float32(2.0 ** -9), scaled[0][t])


@pytest.mark.parametrize("W", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_identical_replicas_reduce_to_the_input(W, dtype):
    """k*x is exact in fp32 for every k <= W when x has at most 24 - log2(W) significant bits;
    the chain x, 2x, 3x, ... is then exact and so is the final scaling.  Arbitrary fp32 values
    survive a chain of up to four terms (3x may round, but 4x is recovered), not longer ones,
    so for W = 8 and 16 the low four mantissa bits of the fp32 inputs are cleared first.
    bf16 values (8 significant bits) are always exact."""
    elems = [10, 700, 33, 5000, 257]
    one = gradients.replica_set(11, 1, elems, bf16=(dtype == BF16))[0]
    if dtype == F32 and W > 4:
        one = [(a.view(np.uint32) & np.uint32(0xFFFFFFF0)).view(np.float32) for a in one]
    grads = [[a.copy() for a in one] for _ in range(W)]
    plan = build_plan(Config(W, dtype, 2048, SPLIT_FIXED, 8, 4096), elems)
    oracle.allreduce(plan, grads)
    for w in range(W):
        for t in range(len(elems)):
            assert np.array_equal(grads[w][t], one[t])


# ------------------------------------------------------------------ accuracy
@pytest.mark.parametrize("name,dtype", [("mlp", F32), ("mlp", BF16)])
def test_error_bound_against_float64(name, dtype):
    wl = workload(name)
    W = 8
    cfg = Config(W, dtype, wl.batch_threshold_bytes, SPLIT_FIXED, 8, 64 << 10)
    plan = build_plan(cfg, wl.elems())
    grads = gradients.replica_set(1, W, wl.elems(), bf16=(dtype == BF16))
    ref = [oracle.mean_f64(plan, grads, t) for t in range(len(wl.elems()))]
    mag = [oracle.abs_sum_f64(plan, grads, t) for t in range(len(wl.elems()))]
    oracle.allreduce(plan, grads)
    for t in range(len(ref)):
        for w in (0, W - 1):
            if dtype == F32:
                err = np.abs(grads[w][t].astype(np.float64) - ref[t])
                assert (err <= 4e-7 * mag[t]).all()
            else:
                got = oracle.bf16_to_f32(grads[w][t]).astype(np.float64)
                err = np.abs(got - ref[t])
                assert (err <= 2.0 ** -8 * np.abs(ref[t]) + 4e-7 * mag[t] + 1e-45).all()


def test_all_replicas_end_up_equal_and_close_to_mean():
    cfg, plan, grads = small_case(seed=9, W=5, T=1024, mode=SPLIT_NONE, S=0)
    ref = [oracle.mean_f64(plan, grads, t) for t in range(len(grads[0]))]
    mag = [oracle.abs_sum_f64(plan, grads, t) for t in range(len(grads[0]))]
    oracle.allreduce(plan, grads)
    for t in range(len(ref)):
        for w in range(1, 5):
            assert np.array_equal(grads[w][t], grads[0][t])
        assert (np.abs(grads[0][t] - ref[t]) <= 4e-7 * mag[t]).all()


# ------------------------------------------------------------------ bf16 conversion
def test_bf16_widening_is_exact():
    bits = np.arange(1 << 16, dtype=np.uint16)
    f = oracle.bf16_to_f32(bits)
    assert np.array_equal(f.view(np.uint32) >> 16, bits.astype(np.uint32))
    assert not (f.view(np.uint32) & 0xFFFF).any()


def test_bf16_rounding_is_nearest_even_by_definition():
    # for each finite bf16 value v with successor v+: the midpoint and its fp32 neighbours
    bits = np.arange(1 << 16, dtype=np.int64)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    lo = bits[finite]
    mid = (lo << 16) | 0x8000
    for delta, expect in ((-1, lo), (+1, lo + 1)):
        x = (mid + delta).astype(np.uint32).view(np.float32)
        assert np.array_equal(oracle.f32_to_bf16_rne(x), expect.astype(np.uint16))
    tie = oracle.f32_to_bf16_rne(mid.astype(np.uint32).view(np.float32))
    assert np.array_equal(tie, np.where(lo & 1, lo + 1, lo).astype(np.uint16))
    # representable values are fixed points; largest finite rounds up to infinity at the tie
    exact = (lo << 16).astype(np.uint32).view(np.float32)
    assert np.array_equal(oracle.f32_to_bf16_rne(exact), lo.astype(np.uint16))
    assert oracle.f32_to_bf16_rne(np.array([3.4028235e38], dtype=np.float32))[0] == 0x7F80
    nan = oracle.f32_to_bf16_rne(np.array([np.nan, -np.nan], dtype=np.float32))
    assert ((nan & 0x7F80) == 0x7F80).all() and (nan & 0x7F).all()


def test_bf16_rounding_agrees_with_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    raw = rng.integers(0, 1 << 32, 2_000_000, dtype=np.uint64).astype(np.uint32)
    x = raw.view(np.float32)
    x = x[np.isfinite(x)]
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16_rne(x), ref)
