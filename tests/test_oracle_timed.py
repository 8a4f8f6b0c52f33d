"""Pins for the timing-aware batcher and the threshold rule of paper section 4.2 (CPU only)."""
import json
import os
import random
from fractions import Fraction

import pytest

import oracle
from oracle import F32, KIND_BATCH, KIND_CHUNK, SPLIT_NONE, Config, build_plan

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_walked_example():
    with open(os.path.join(GOLDEN, "timed_plan.json")) as f:
        gold = json.load(f)
    cfg = Config(2, F32, 1024, SPLIT_NONE, 8, 0, 16, 2)
    plan = build_plan(cfg, gold["elems"], gold["ready_time"], gold["net_a"], gold["net_b"])
    assert plan.fused_elems == gold["fused_elems"] and len(plan.units) == len(gold["units"])
    kinds = {"batch": KIND_BATCH, "chunk": KIND_CHUNK}
    for i, (u, g) in enumerate(zip(plan.units, gold["units"])):
        assert (u.kind, u.elems, u.fused_off) == (kinds[g["kind"]], g["elems"], g["fused_off"])
        members = [[e.tensor, e.unit_off] for e in plan.entries[u.first_entry:u.first_entry + u.n_entries]]
        assert members == g["members"]
        assert plan.enqueue_time[i] == pytest.approx(g["enqueue"], abs=1e-9)
        assert plan.start_time[i] == pytest.approx(g["start"], abs=1e-9)
        assert plan.finish_time[i] == pytest.approx(g["finish"], abs=1e-9)


def random_sizes(rng, n):
    return [rng.choice([1, 3, 8, 17, 64, 100, 255, 256, 257, 1000, 5000]) for _ in range(n)]


def test_a_network_that_is_always_busy_gives_the_size_only_plan():
    rng = random.Random(1)
    for _ in range(200):
        elems = random_sizes(rng, rng.randint(1, 12))
        cfg = Config(4, F32, rng.choice([256, 1024, 4096]))
        t, times = 0.0, []
        for _ in elems:
            t += rng.random()
            times.append(t)
        slow = build_plan(cfg, elems, times, 1e9, 0.0)       # every transfer takes "forever"
        plain = build_plan(cfg, elems)
        # the first small parameter may still go at once (nothing queued yet); compare from there on
        if slow.units == plain.units:
            continue
        first = slow.units[0]
        assert first.kind == KIND_BATCH and first.n_entries == 1
        rest = build_plan(cfg, elems[1:])
        assert [(u.kind, u.elems) for u in slow.units[1:]] == [(u.kind, u.elems) for u in rest.units]


def test_an_infinitely_fast_network_never_batches():
    rng = random.Random(2)
    for _ in range(100):
        elems = random_sizes(rng, rng.randint(1, 12))
        times = sorted(rng.random() * 10 for _ in elems)
        plan = build_plan(Config(4, F32, 4096), elems, times, 0.0, 0.0)
        assert len(plan.units) == len(elems)
        assert all(u.n_entries == 1 for u in plan.units)
        assert plan.start_time == [float(x) for x in times]


def test_schedule_invariants():
    rng = random.Random(3)
    for _ in range(300):
        elems = random_sizes(rng, rng.randint(1, 14))
        T = rng.choice([256, 1024, 4096])
        cfg = Config(rng.choice([2, 8]), F32, T)
        times = sorted(rng.random() * 50 for _ in elems)
        a, b = rng.choice([0.0, 0.5, 5.0]), rng.choice([0.0, 0.001, 0.01])
        plan = build_plan(cfg, elems, times, a, b)
        # transfers are served one at a time, in queue order, never before they are queued
        for i in range(len(plan.units)):
            assert plan.start_time[i] >= plan.enqueue_time[i]
            if i:
                assert plan.start_time[i] >= plan.finish_time[i - 1]
                assert plan.enqueue_time[i] >= plan.enqueue_time[i - 1]
            assert plan.finish_time[i] == plan.start_time[i] + (a + b * float(plan.units[i].elems * 4))
        # a unit is queued at the update time of its last member; what is still open after the
        # last parameter goes out then
        for i, u in enumerate(plan.units):
            last = plan.entries[u.first_entry + u.n_entries - 1].tensor
            leftover = i == len(plan.units) - 1 and u.kind == KIND_BATCH
            assert plan.enqueue_time[i] == (times[-1] if leftover else times[last])
        # a batch below the threshold was sent because the network was about to idle (or at the end)
        for i, u in enumerate(plan.units):
            leftover = i == len(plan.units) - 1
            if u.kind == KIND_BATCH and u.elems * 4 < T and not leftover:
                last = plan.entries[u.first_entry + u.n_entries - 1].tensor
                if last + 1 < len(elems):
                    busy_until = plan.finish_time[i - 1] if i else 0.0
                    assert busy_until <= times[last + 1]
        # and an open batch is never kept while the network is idle ahead
        for i, u in enumerate(plan.units):
            if u.kind != KIND_BATCH:
                continue
            members = plan.entries[u.first_entry:u.first_entry + u.n_entries]
            for m in members[:-1]:                         # after each earlier member the batch stayed open
                queued = [j for j in range(len(plan.units)) if plan.enqueue_time[j] <= times[m.tensor] and j < i]
                busy_until = max([plan.finish_time[j] for j in queued], default=0.0)
                assert busy_until > times[m.tensor + 1]


def test_rejects_bad_timing_arguments():
    cfg = Config(2, F32, 1024)
    with pytest.raises(ValueError):
        build_plan(cfg, [10, 10], [1.0, 0.5], 1.0, 1.0)
    with pytest.raises(ValueError):
        build_plan(cfg, [10, 10], [1.0], 1.0, 1.0)
    with pytest.raises(ValueError):
        build_plan(cfg, [10, 10], [0.0, 1.0], -1.0, 1.0)


# ------------------------------------------------------------------ threshold rule
def ratio(a, b, x):
    f = lambda d: Fraction(a) + Fraction(b) * d
    return f(2 * x) / (2 * f(x))


def test_threshold_is_the_smallest_size_past_the_ratio():
    rng = random.Random(4)
    for _ in range(300):
        a = rng.choice([0.0, 1e-6, 37.5, 100.0, rng.random() * 1000])
        b = rng.choice([1e-3, 0.01, 0.125, rng.random() + 1e-6])
        x = oracle.threshold_from_model(a, b)
        assert x >= 1 and ratio(a, b, x) > Fraction(4, 5)
        if x > 1:
            assert ratio(a, b, x - 1) <= Fraction(4, 5)


def test_threshold_by_brute_force_scan_and_closed_form():
    # f = 40 + 0.5 d: 1.5 a / b = 120, and the ratio at exactly 120 is 0.8, so the answer is 121
    assert oracle.threshold_from_model(40.0, 0.5) == 121
    scan = next(x for x in range(1, 10000) if ratio(40.0, 0.5, x) > Fraction(4, 5))
    assert scan == 121
    for a, b in ((3.0, 0.25), (10.0, 0.01), (0.0, 1.0), (7.0, 3.0)):
        scan = next(x for x in range(1, 100000) if ratio(a, b, x) > Fraction(4, 5))
        assert oracle.threshold_from_model(a, b) == scan


def test_linear_fit_through_the_two_measured_sizes():
    # section 4.2 measures 64 B and 4 MB transfers
    a, b = oracle.fit_linear(64, 50.0 + 64 * 0.002, 4 << 20, 50.0 + (4 << 20) * 0.002)
    assert abs(float(a) - 50.0) < 1e-6 and abs(float(b) - 0.002) < 1e-12
    assert oracle.threshold_from_model(a, b) == int(Fraction(3) * a / (2 * b)) + 1
    with pytest.raises(ValueError):
        oracle.fit_linear(64, 1.0, 64, 2.0)
    with pytest.raises(ValueError):
        oracle.threshold_from_model(1.0, 0.0)
