"""Pins for the transfer scheduler of paper section 4.3 (CPU only)."""
import json
import os
import random

import pytest

from oracle import (BIN_BACKWARD, BIN_FORWARD, F32, Config, build_plan, group_windows, schedule_transfers)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_walked_example():
    with open(os.path.join(GOLDEN, "transfer_schedule.json")) as f:
        gold = json.load(f)
    g = gold["groups"]
    s = schedule_transfers([x["bytes"] for x in g], [x["ready"] for x in g], [x["need"] for x in g],
                           gold["bp_len"], gold["fp_len"], gold["net_a"], gold["net_b"])
    bins = {"backward": BIN_BACKWARD, "forward": BIN_FORWARD}
    for got, want in zip(s.slots, gold["slots"]):
        assert (got.bin, got.start, got.end, got.stage) == (bins[want["bin"]], want["start"], want["end"], want["stage"])
    assert (s.comm_time, s.compute_time, s.bp_overrun, s.fp_overrun, s.iteration_time) == \
        (gold["comm_time"], gold["compute_time"], gold["bp_overrun"], gold["fp_overrun"], gold["iteration_time"])
    assert s.overlap == pytest.approx(gold["overlap_num"] / gold["overlap_den"], rel=1e-15)
    assert s.utilization == pytest.approx(gold["utilization_num"] / gold["utilization_den"], rel=1e-15)


def random_case(rng, n, integer=False):
    bp, fp = float(rng.randint(5, 40)), float(rng.randint(5, 40))
    nbytes = [rng.randint(1, 12) for _ in range(n)]
    if integer:
        ready = [float(rng.randint(0, int(bp))) for _ in range(n)]
        need = [float(rng.randint(0, int(fp))) for _ in range(n)]
        a, b = float(rng.randint(0, 2)), 1.0
    else:
        ready = [rng.random() * bp for _ in range(n)]
        need = [rng.random() * fp for _ in range(n)]
        a, b = rng.random() * 2, rng.random() + 0.01
    return nbytes, ready, need, bp, fp, a, b


def test_invariants_on_random_cases():
    rng = random.Random(43)
    for _ in range(400):
        n = rng.randint(1, 14)
        nbytes, ready, need, bp, fp, a, b = random_case(rng, n)
        s = schedule_transfers(nbytes, ready, need, bp, fp, a, b)
        assert len(s.slots) == n
        for g, sl in enumerate(s.slots):
            assert sl.end - sl.start == pytest.approx(a + b * nbytes[g], abs=1e-9)
            if sl.bin == BIN_BACKWARD:
                assert sl.start >= ready[g]                      # never before the last member's update
                assert sl.stage == 3 or sl.end <= bp
            else:
                assert sl.end <= need[g]                         # never after the first member is read
                assert sl.stage == 3 or sl.start >= 0.0
        for which in (BIN_BACKWARD, BIN_FORWARD):                # one transfer at a time
            iv = sorted((sl.start, sl.end) for sl in s.slots if sl.bin == which)
            for (s0, e0), (s1, e1) in zip(iv, iv[1:]):
                assert e0 <= s1
        # bookkeeping: iteration time, and the utilization law of section 3
        assert s.iteration_time == pytest.approx(bp + fp + s.bp_overrun + s.fp_overrun)
        assert s.bp_overrun >= 0 and s.fp_overrun >= 0 and 0.0 <= s.overlap <= 1.0 + 1e-12
        rho = s.comm_time / s.compute_time
        assert s.utilization == pytest.approx(1.0 / (1.0 + rho - s.overlap * min(rho, 1.0)), rel=1e-12)
        # overruns are caused by stage-3 slots only
        if all(sl.stage == 2 for sl in s.slots):
            assert s.bp_overrun == 0.0 and s.fp_overrun == 0.0 and s.utilization == 1.0


def occupied(slots, which, t0, t1):
    return any(sl is not None and sl.bin == which and sl.start < t1 and t0 < sl.end for sl in slots)


def test_integer_cases_against_a_time_step_search():
    """With whole-number times every feasible start is a whole number, so a scan over all of
    them finds the true earliest (backward) or latest (forward) place; replay the greedy
    order with that scan and compare."""
    rng = random.Random(44)
    for _ in range(300):
        n = rng.randint(1, 10)
        nbytes, ready, need, bp, fp, a, b = random_case(rng, n, integer=True)
        if a + b * min(nbytes) <= 0:
            continue
        s = schedule_transfers(nbytes, ready, need, bp, fp, a, b)
        dur = [int(a + b * x) for x in nbytes]
        horizon = int(bp + fp) + sum(dur) + 2

        class S:
            def __init__(self, bin, start, end):
                self.bin, self.start, self.end = bin, start, end
        placed = [None] * n
        order = sorted(range(n), key=lambda g: (-nbytes[g], g))

        def scan_bp(g, limit):
            for t in range(int(ready[g]), limit + 1):
                if t + dur[g] <= limit and not occupied(placed, BIN_BACKWARD, t, t + dur[g]):
                    return t
            return None

        def scan_fp(g, limit):
            for e in range(int(need[g]), limit - 1, -1):
                if e - dur[g] >= limit and not occupied(placed, BIN_FORWARD, e - dur[g], e):
                    return e
            return None

        for g in order:
            t = scan_bp(g, int(bp))
            if t is not None:
                placed[g] = S(BIN_BACKWARD, t, t + dur[g])
                continue
            e = scan_fp(g, 0)
            if e is not None:
                placed[g] = S(BIN_FORWARD, e - dur[g], e)
        for g in order:
            if placed[g] is not None:
                continue
            end_now = max([int(bp)] + [p.end for p in placed if p is not None and p.bin == BIN_BACKWARD])
            begin_now = min([0] + [p.start for p in placed if p is not None and p.bin == BIN_FORWARD])
            t = scan_bp(g, horizon)
            e = scan_fp(g, -horizon)
            grow_bp = max(0, t + dur[g] - end_now)
            grow_fp = max(0, begin_now - (e - dur[g]))
            placed[g] = S(BIN_BACKWARD, t, t + dur[g]) if grow_bp <= grow_fp else S(BIN_FORWARD, e - dur[g], e)
        for g in range(n):
            assert (s.slots[g].bin, s.slots[g].start, s.slots[g].end) == (placed[g].bin, placed[g].start, placed[g].end)


def test_everything_fits_behind_the_backward_pass_start():
    """All groups ready at time 0 and a long backward pass: back to back in size order."""
    nbytes = [3, 9, 1, 9, 5]
    s = schedule_transfers(nbytes, [0.0] * 5, [0.0] * 5, 100.0, 1.0, 0.5, 2.0)
    t = 0.0
    for g in [1, 3, 4, 0, 2]:
        assert (s.slots[g].bin, s.slots[g].start, s.slots[g].stage) == (BIN_BACKWARD, t, 2)
        t += 0.5 + 2.0 * nbytes[g]
    assert s.iteration_time == 101.0 and s.overlap == 1.0 and s.utilization == 1.0


def test_nothing_fits_beside_the_computation():
    """Every transfer is longer than either pass: all of them lengthen the iteration; the first
    goes behind the backward pass (equal cost), the later ones wherever the overrun grows less."""
    s = schedule_transfers([10, 8, 6], [2.0, 1.0, 0.0], [1.0, 2.0, 3.0], 4.0, 3.0, 0.0, 1.0)
    # g0 (10): backward [2, 12] adds 8; forward [-9, 1] adds 9 -> backward
    # g1 (8):  backward after g0 [12, 20] adds 8; forward [-6, 2] adds 6 -> forward
    # g2 (6):  backward [12, 18] adds 6; forward before g1 [-12, -6] adds 6 -> backward
    assert [(x.bin, x.start, x.end, x.stage) for x in s.slots] == \
        [(BIN_BACKWARD, 2.0, 12.0, 3), (BIN_FORWARD, -6.0, 2.0, 3), (BIN_BACKWARD, 12.0, 18.0, 3)]
    assert (s.bp_overrun, s.fp_overrun, s.iteration_time) == (14.0, 6.0, 27.0)
    assert s.overlap == pytest.approx((24 + 7 - 27) / 7)


def test_forward_window_is_the_mirror_image_of_the_backward_window():
    """Groups that can only go forward (ready when the backward pass ends), against the mirrored
    problem where they can only go backward: the slots are reflections of each other."""
    rng = random.Random(45)
    done = 0
    while done < 100:
        n = rng.randint(1, 8)
        fp = float(rng.randint(20, 60))
        nbytes = [rng.randint(1, 6) for _ in range(n)]
        need = [float(rng.randint(0, int(fp))) for _ in range(n)]
        fwd = schedule_transfers(nbytes, [5.0] * n, need, 5.0, fp, 0.0, 1.0)
        if any(sl.stage != 2 for sl in fwd.slots):
            continue
        done += 1
        assert all(sl.bin == BIN_FORWARD for sl in fwd.slots)
        bwd = schedule_transfers(nbytes, [fp - x for x in need], [0.0] * n, fp, 5.0, 0.0, 1.0)
        for f, m in zip(fwd.slots, bwd.slots):
            assert (m.bin, m.start, m.end) == (BIN_BACKWARD, fp - f.end, fp - f.start)


def test_a_later_boundary_is_respected_even_when_earlier_room_is_free():
    s = schedule_transfers([4], [7.5], [0.0], 20.0, 5.0, 1.0, 0.25)
    assert (s.slots[0].bin, s.slots[0].start, s.slots[0].end) == (BIN_BACKWARD, 7.5, 9.5)
    s = schedule_transfers([4], [19.5], [3.25], 20.0, 5.0, 1.0, 0.25)     # backward would end at 21.5
    assert (s.slots[0].bin, s.slots[0].start, s.slots[0].end) == (BIN_FORWARD, 1.25, 3.25)


def test_windows_of_a_batch_come_from_its_last_updated_and_first_read_member():
    # three small tensors form one batch, the fourth goes alone
    plan = build_plan(Config(2, F32, 1024), [16, 32, 208, 4096])
    assert [u.n_entries for u in plan.units] == [3, 1]
    nbytes, ready, need = group_windows(plan, [1.0, 2.0, 3.0, 4.0], [9.0, 8.0, 7.0, 6.0])
    assert nbytes == [256 * 4, 4096 * 4] and ready == [3.0, 4.0] and need == [7.0, 6.0]


def test_chunks_of_a_split_tensor_share_its_boundaries():
    from oracle import SPLIT_FIXED
    plan = build_plan(Config(2, F32, 1024, SPLIT_FIXED, 8, 4096), [3000, 16])     # 12000 B -> chunks of 4096 B
    assert [u.elems for u in plan.units] == [1024, 1024, 952, 16]
    nbytes, ready, need = group_windows(plan, [2.5, 3.5], [8.0, 1.0])
    assert nbytes == [4096, 4096, 3808, 64]
    assert ready == [2.5, 2.5, 2.5, 3.5] and need == [8.0, 8.0, 8.0, 1.0]


def test_argument_errors():
    with pytest.raises(ValueError):
        schedule_transfers([1], [0.0], [0.0, 1.0], 1.0, 1.0, 1.0, 1.0)
    with pytest.raises(ValueError):
        schedule_transfers([1], [2.0], [0.0], 1.0, 1.0, 1.0, 1.0)        # ready after the pass ended
    with pytest.raises(ValueError):
        schedule_transfers([1], [0.0], [2.0], 1.0, 1.0, 1.0, 1.0)
    with pytest.raises(ValueError):
        schedule_transfers([1], [0.0], [0.0], 1.0, 1.0, 0.0, 0.0)        # zero-length transfers
    with pytest.raises(ValueError):
        schedule_transfers([1], [0.0], [0.0], 1.0, 1.0, -1.0, 1.0)
