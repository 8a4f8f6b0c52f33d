"""Pins for the oracle's transfer plan (CPU only).

The batcher of paper section 4.2 and the depth rule of section 4.4 are checked
against (i) a plan enumerated by hand, (ii) properties that together determine
the result uniquely, and (iii) the per-configuration shapes worked out when the
workloads were defined.
"""
import json
import os
import random

import pytest

import oracle
from oracle import (BF16, F32, KIND_BATCH, KIND_CHUNK, SPLIT_ADAPTIVE, SPLIT_FIXED, SPLIT_NONE,
                    Config, build_plan)
from workloads.shapes import ALL, EXTRA, workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def cfg_of(wl):
    return Config(wl.world, wl.dtype, wl.batch_threshold_bytes, wl.split_mode, wl.max_depth,
                  wl.split_bytes, wl.align_bytes, wl.num_streams)


# ------------------------------------------------------------------ hand case
def test_mlp_plan_matches_hand_enumeration():
    with open(os.path.join(GOLDEN, "mlp_plan.json")) as f:
        gold = json.load(f)
    wl = workload("mlp")
    assert [n for n, _ in wl.update_order()] == gold["update_order"]
    assert wl.elems() == gold["elems"]
    plan = build_plan(cfg_of(wl), wl.elems())
    assert plan.fused_elems == gold["fused_elems"]
    kinds = {"batch": KIND_BATCH, "chunk": KIND_CHUNK}
    assert len(plan.units) == len(gold["units"])
    for u, g in zip(plan.units, gold["units"]):
        assert (u.kind, u.elems, u.fused_off, u.stream, u.seg_start) == \
               (kinds[g["kind"]], g["elems"], g["fused_off"], g["stream"], g["seg_start"])
    assert len(plan.entries) == len(gold["entries"])
    for e, g in zip(plan.entries, gold["entries"]):
        assert (e.tensor, e.tensor_off, e.unit, e.unit_off, e.elems) == \
               (g["tensor"], g["tensor_off"], g["unit"], g["unit_off"], g["elems"])


# ------------------------------------------------------------------ invariants
def check_invariants(cfg: Config, elems, plan):
    s, g, T, W = cfg.elem_size, cfg.granule, cfg.batch_threshold_bytes, cfg.world
    # entries are grouped by unit, in unit order
    pos = 0
    for ui, u in enumerate(plan.units):
        assert u.first_entry == pos and u.n_entries >= 1
        for e in plan.entries[pos:pos + u.n_entries]:
            assert e.unit == ui
        pos += u.n_entries
        assert u.stream == ui % cfg.num_streams
    assert pos == len(plan.entries)

    # every element of every tensor is covered exactly once, in order
    cover = {t: [] for t in range(len(elems))}
    for e in plan.entries:
        assert e.elems > 0
        cover[e.tensor].append((e.tensor_off, e.elems))
    for t, n in enumerate(elems):
        at = 0
        for off, cnt in sorted(cover[t]):
            assert off == at
            at += cnt
        assert at == n

    # batches: members small, in update order, granule-aligned, tightly packed;
    # a batch is sent by the FIRST member that lifts it to the threshold
    fused_at = 0
    batches = [u for u in plan.units if u.kind == KIND_BATCH]
    last_tensor = -1
    for bi, u in enumerate(batches):
        assert T > 0
        members = plan.entries[u.first_entry:u.first_entry + u.n_entries]
        fill = 0
        for m in members:
            assert m.tensor > last_tensor
            last_tensor = m.tensor
            assert m.tensor_off == 0 and m.elems == elems[m.tensor]
            assert m.elems * s < T
            assert m.unit_off % g == 0
            assert m.unit_off == (fill + g - 1) // g * g
            fill = m.unit_off + m.elems
        padded = (fill + g - 1) // g * g
        assert u.elems == padded
        before_last = members[-1].unit_off          # already granule aligned
        assert before_last * s < T                  # not yet due before its last member
        if bi < len(batches) - 1:
            assert padded * s >= T                  # due once the last member is in
        assert padded * s < 2 * T
        assert u.fused_off == fused_at
        fused_at += u.elems
    assert plan.fused_elems == fused_at
    # only the very last emitted batch may be below the threshold, and then it is the last unit
    for bi, u in enumerate(batches):
        if u.elems * s < T:
            assert bi == len(batches) - 1 and u is plan.units[-1]

    # chunks: large tensors only; consecutive pieces; sizes per split mode
    by_tensor = {}
    for u in plan.units:
        if u.kind == KIND_CHUNK:
            assert u.n_entries == 1 and u.fused_off == 0
            e = plan.entries[u.first_entry]
            assert e.unit_off == 0 and e.elems == u.elems
            by_tensor.setdefault(e.tensor, []).append(e)
    for t, pieces in by_tensor.items():
        nbytes = elems[t] * s
        assert T == 0 or nbytes >= T
        sizes = [p.elems for p in pieces]
        if cfg.split_mode == SPLIT_NONE or nbytes <= cfg.split_bytes:
            assert sizes == [elems[t]]
        elif cfg.split_mode == SPLIT_FIXED:
            piece = cfg.split_bytes // s
            assert all(x == piece for x in sizes[:-1]) and 0 < sizes[-1] <= piece
            assert len(sizes) == -(-elems[t] // piece)
        else:
            depth = min(max(nbytes // cfg.split_bytes, 1), cfg.max_depth)
            assert 1 <= len(sizes) <= depth <= cfg.max_depth
            assert all(x == sizes[0] for x in sizes[:-1]) and 0 < sizes[-1] <= sizes[0]
            assert sizes[0] % g == 0 or len(sizes) == 1
            assert sizes[0] * depth >= elems[t] and (sizes[0] - g) * depth < elems[t]
            if depth > 1:
                assert sizes[0] * s >= cfg.split_bytes     # no piece drops below the threshold
        for p in pieces:
            assert p.tensor_off % g == 0
    # small tensors never become chunks, large never join batches
    for t, n in enumerate(elems):
        is_large = T == 0 or n * s >= T
        assert (t in by_tensor) == is_large

    # unit emission order: a chunk unit appears at its tensor's position, a batch unit at
    # the position of the member that closed it (or at the end)
    def emit_key(u):
        return plan.entries[u.first_entry + u.n_entries - 1].tensor
    keys = [emit_key(u) for u in plan.units]
    if batches and batches[-1].elems * s < T:
        keys = keys[:-1]
    assert keys == sorted(keys)

    # ring segments: W contiguous pieces on granule boundaries, sizes within one granule,
    # larger ones first
    for u in plan.units:
        seg = u.seg_start
        assert len(seg) == W + 1 and seg[0] == 0 and seg[-1] == u.elems
        gran = []
        for c in range(W):
            assert seg[c] <= seg[c + 1]
            assert seg[c] % g == 0 or seg[c] == u.elems
            gran.append(-(-(seg[c + 1] - seg[c]) // g))
        assert max(gran) - min(gran) <= 1
        assert gran == sorted(gran, reverse=True)


def random_case(rng):
    dtype = rng.choice([F32, BF16])
    s = 4 if dtype == F32 else 2
    align = rng.choice([16, 16, 16, 32, 64, s])
    W = rng.choice([1, 2, 3, 4, 5, 7, 8, 16])
    T = rng.choice([0, 64, 256, 1024, 4096, 1000])
    mode = rng.choice([SPLIT_NONE, SPLIT_FIXED, SPLIT_ADAPTIVE])
    S = rng.choice([1, 2, 4, 16, 64]) * max(align, 64) if mode != SPLIT_NONE else 0
    cfg = Config(W, dtype, T, mode, rng.choice([1, 2, 8]), S, align, rng.choice([1, 2]))
    n = rng.randint(1, 14)
    elems = [rng.choice([1, 2, 3, 5, 8, 17, 64, 100, 255, 256, 257, 1000, 4096, 5000, 70000])
             for _ in range(n)]
    return cfg, elems


def test_invariants_random(rounds=500):
    rng = random.Random(20041402)
    for _ in range(rounds):
        cfg, elems = random_case(rng)
        plan = build_plan(cfg, elems)
        check_invariants(cfg, elems, plan)
        again = build_plan(cfg, elems)
        assert again == plan                     # deterministic


@pytest.mark.parametrize("name", ALL + EXTRA)
def test_invariants_workloads(name):
    wl = workload(name)
    cfg = cfg_of(wl)
    check_invariants(cfg, wl.elems(), build_plan(cfg, wl.elems()))


# ------------------------------------------------------------------ special cases
def test_batching_off_gives_one_unit_per_tensor():
    elems = [5, 100, 7, 3000]
    plan = build_plan(Config(4, F32, 0), elems)
    assert [u.kind for u in plan.units] == [KIND_CHUNK] * 4
    assert [u.elems for u in plan.units] == elems and plan.fused_elems == 0


def test_size_equal_to_threshold_is_large():
    plan = build_plan(Config(2, F32, 1024), [100, 256, 100])
    assert [u.kind for u in plan.units] == [KIND_CHUNK, KIND_BATCH]
    assert plan.entries[0].tensor == 1


def test_large_tensor_does_not_flush_open_batch():
    # small, LARGE, small: the large one is queued at once, the two small ones share a batch
    plan = build_plan(Config(2, F32, 4096), [10, 5000, 10])
    assert [u.kind for u in plan.units] == [KIND_CHUNK, KIND_BATCH]
    assert [e.tensor for e in plan.entries] == [1, 0, 2]


def test_split_threshold_above_all_tensors_is_depth_one():
    for mode in (SPLIT_FIXED, SPLIT_ADAPTIVE):
        plan = build_plan(Config(4, F32, 64, mode, 8, 1 << 20), [100, 2000, 50000])
        assert len(plan.units) == 3


def test_adaptive_depth_grows_with_size_and_saturates():
    S = 1 << 20
    cfg = Config(8, F32, S, SPLIT_ADAPTIVE, 8, S)
    sizes = {1: S // 4, 2: 2 * S // 4, 3: 7 * S // 8, 5: 5 * S // 4 + 12, 8: 8 * S // 4, 100: 100 * S // 4}
    expect = {1: 1, 2: 2, 3: 3, 5: 5, 8: 8, 100: 8}    # section 4.4: from 1 up to a maximum of 8
    for k, n in sizes.items():
        plan = build_plan(cfg, [n])
        assert len(plan.units) == expect[k], k
    # just below twice the threshold: still one piece
    assert len(build_plan(cfg, [2 * S // 4 - 1]).units) == 1


def test_fixed_split_vgg_fc1_is_98_exact_chunks():
    wl = workload("vgg16")
    plan = build_plan(cfg_of(wl), wl.elems())
    t = [n for n, _ in wl.update_order()].index("fc1.w")
    pieces = [e.elems for e in plan.entries if e.tensor == t]
    assert pieces == [1 << 20] * 98


def test_workload_plan_shapes():
    # (units, batch units, chunk units, small elems) per configuration
    expect = {"mlp": (3, 1, 2, 3084), "resnet50": (35, 6, 29, 1620008), "vgg16": (140, 2, 138, 273192),
              "inception_v3": (30, 21, 9, 14208968), "transformer": (101, 49, 52, 102560768)}
    for name in ALL:
        wl = workload(name)
        plan = build_plan(cfg_of(wl), wl.elems())
        nb = sum(u.kind == KIND_BATCH for u in plan.units)
        assert (len(plan.units), nb, len(plan.units) - nb, plan.fused_elems) == expect[name]


@pytest.mark.parametrize("bad", [
    dict(world=0), dict(dtype=7), dict(align_bytes=24), dict(align_bytes=2), dict(num_streams=3),
    dict(split_mode=SPLIT_FIXED, split_bytes=0), dict(split_mode=SPLIT_FIXED, split_bytes=40),
    dict(split_mode=9),
])
def test_bad_config_rejected(bad):
    kw = dict(world=4, dtype=F32, batch_threshold_bytes=1024)
    kw.update(bad)
    with pytest.raises(ValueError):
        build_plan(Config(**kw), [10, 20])


def test_bad_tensor_list_rejected():
    with pytest.raises(ValueError):
        build_plan(Config(4), [])
    with pytest.raises(ValueError):
        build_plan(Config(4), [4, 0, 4])
