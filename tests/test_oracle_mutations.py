"""Do the pins bite?  Plausible mistakes are planted in a copy of the oracle's source (on the
CPU only) and the pin tests are run against the damaged copy: for every mistake at least one
pin must fail.  The undamaged oracle must pass all of them through the same harness."""
import importlib
import os
import sys
import types

import pytest

import oracle
import oracle.aggregate
import oracle.plan
import oracle.schedule

import test_oracle_aggregate as pins_agg
import test_oracle_patterns as pins_pat
import test_oracle_plan as pins_plan
import test_oracle_schedule as pins_sched
import test_oracle_timed as pins_timed

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PLAN_PINS = [
    pins_plan.test_mlp_plan_matches_hand_enumeration,
    lambda: pins_plan.test_invariants_random(100),
    pins_plan.test_size_equal_to_threshold_is_large,
    pins_plan.test_large_tensor_does_not_flush_open_batch,
    pins_plan.test_adaptive_depth_grows_with_size_and_saturates,
    pins_plan.test_fixed_split_vgg_fc1_is_98_exact_chunks,
    pins_plan.test_workload_plan_shapes,
    pins_plan.test_batching_off_gives_one_unit_per_tensor,
]
AGG_PINS = [
    pins_agg.test_worked_examples,
    lambda: pins_agg.test_formula_equals_message_passing_simulation(4),
    lambda: pins_agg.test_formula_equals_message_passing_simulation(5),
    lambda: pins_agg.test_integer_inputs_give_exact_mean(8, oracle.F32),
    lambda: pins_agg.test_integer_inputs_give_exact_mean(4, oracle.BF16),
    lambda: pins_agg.test_identical_replicas_reduce_to_the_input(16, oracle.BF16),
    lambda: pins_agg.test_pack_then_unpack_is_identity_and_padding_is_zero(oracle.F32),
    lambda: pins_agg.test_pack_then_unpack_is_identity_and_padding_is_zero(oracle.BF16),
    pins_agg.test_pack_places_position_codes,
    lambda: pins_agg.test_error_bound_against_float64("mlp", oracle.BF16),
    pins_agg.test_bf16_rounding_is_nearest_even_by_definition,
    pins_agg.test_bf16_widening_is_exact,
    pins_pat.test_worked_example_values,
    lambda: pins_pat.test_halving_doubling_formula_equals_protocol_simulation(8),
    lambda: pins_pat.test_shuffle_formula_equals_protocol_simulation(5),
    pins_timed.test_hand_walked_example,
    pins_timed.test_an_infinitely_fast_network_never_batches,
    pins_timed.test_schedule_invariants,
    pins_timed.test_threshold_by_brute_force_scan_and_closed_form,
]
SCHED_PINS = [
    pins_sched.test_hand_walked_example,
    pins_sched.test_invariants_on_random_cases,
    pins_sched.test_integer_cases_against_a_time_step_search,
    pins_sched.test_everything_fits_behind_the_backward_pass_start,
    pins_sched.test_nothing_fits_beside_the_computation,
    pins_sched.test_forward_window_is_the_mirror_image_of_the_backward_window,
    pins_sched.test_a_later_boundary_is_respected_even_when_earlier_room_is_free,
    pins_sched.test_windows_of_a_batch_come_from_its_last_updated_and_first_read_member,
]

# (file, text to replace, replacement, what the mistake is)
MUTATIONS = [
    ("plan.py", "if t_bytes == 0 or n * s >= t_bytes:", "if t_bytes == 0 or n * s > t_bytes:", "equality with the threshold counted as small"),
    ("plan.py", "        at = _align_up(open_elems, g)\n        open_batch.append", "        at = open_elems\n        open_batch.append", "members not aligned to granules"),
    ("plan.py", "        full = _align_up(open_elems, g) * s >= t_bytes", "        full = _align_up(open_elems, g) * s > 2 * t_bytes", "batch sent too late"),
    ("plan.py", "        at = _align_up(open_elems, g)\n", "        if open_batch and _align_up(open_elems, g) * s + n * s >= t_bytes:\n            emit(KIND_BATCH, open_batch, _align_up(open_elems, g), now)\n            open_batch, open_elems = [], 0\n        at = _align_up(open_elems, g)\n", "batch sent before the member that fills it"),
    ("plan.py", "            off = 0\n            for piece in chunk_sizes(cfg, n):", "            if open_batch:\n                emit(KIND_BATCH, open_batch, _align_up(open_elems, g), now)\n                open_batch, open_elems = [], 0\n            off = 0\n            for piece in chunk_sizes(cfg, n):", "a large tensor flushes the open batch"),
    ("plan.py", "        gran = c * base + min(c, rem)", "        gran = c * base + max(0, c - (w - rem))", "surplus granules given to the last owners"),
    ("plan.py", "        depth = min(max(nbytes // cfg.split_bytes, 1), cfg.max_depth)", "        depth = min(max(-(-nbytes // cfg.split_bytes), 1), cfg.max_depth)", "depth rounded up"),
    ("plan.py", "        depth = min(max(nbytes // cfg.split_bytes, 1), cfg.max_depth)", "        depth = max(nbytes // cfg.split_bytes, 1)", "depth not capped"),
    ("plan.py", "        piece = cfg.split_bytes // s\n", "        piece = cfg.split_bytes\n", "chunk size in bytes used as elements"),
    ("plan.py", "                          u % cfg.num_streams, ring_segments(cfg, n)))", "                          0, ring_segments(cfg, n)))", "every unit on stream 0"),
    ("plan.py", "            fused_off = fused_elems\n", "            fused_off = 0\n", "fused offsets not accumulated"),
    ("aggregate.py", "            acc = val(c + 1).copy()\n            for k in range(2, W + 1):\n                acc = acc + val(c + k)", "            acc = val(c).copy()\n            for k in range(1, W):\n                acc = acc + val(c + k)", "chain starts at the owner"),
    ("aggregate.py", "                acc = acc + val(c + k)", "                acc = acc + val(c + 2 - k)", "ring walked in the other direction"),
    ("aggregate.py", "            for k in range(2, W + 1):", "            for k in range(2, W):", "last term dropped"),
    ("aggregate.py", "                part = [part[i] + part[i + 1] for i in range(0, len(part), 2)]", "                h = len(part) // 2\n                part = [part[i] + part[i + h] for i in range(h)]", "halving-doubling pairs the far partner first"),
    ("aggregate.py", "            acc = val(0).copy()\n            for w in range(1, W):\n                acc = acc + val(w)", "            acc = val(c).copy()\n            for w in range(1, W):\n                acc = acc + val(c + w)", "shuffle sums starting from the owner"),
    ("plan.py", "        idle_ahead = timed and t + 1 < len(elems) and free_at <= float(ready_time[t + 1])", "        idle_ahead = timed and t + 1 < len(elems) and free_at <= now", "idle test against the current update time"),
    ("plan.py", "            begin = max(now, free_at)", "            begin = now", "transfers overlap instead of queueing"),
    ("plan.py", "    x = (3 * a) // (2 * b) + 1", "    x = -((-3 * a) // (2 * b))", "threshold at the ratio instead of past it"),
    ("aggregate.py", "        y = acc * inv_w", "        y = acc", "no scaling"),
    ("aggregate.py", "        y = acc * inv_w", "        y = acc / np.float32(W)", "division instead of multiplication by the rounded reciprocal"),
    ("aggregate.py", "    lsb = (b >> np.uint64(16)) & np.uint64(1)", "    lsb = np.uint64(1)", "ties rounded away from zero"),
    ("aggregate.py", "    r = ((b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)", "    r = (b >> np.uint64(16)).astype(np.uint16)", "bf16 truncation instead of rounding"),
    ("aggregate.py", "    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)", "    return (bits.astype(np.uint32) << np.uint32(15)).view(np.float32)", "wrong widening shift"),
    ("aggregate.py", "            region[...] = 0\n", "", "padding not cleared"),
    ("aggregate.py", "                region[e.unit_off:e.unit_off + e.elems] = \\\n                    grads[w][e.tensor][e.tensor_off:e.tensor_off + e.elems]", "                region[e.unit_off:e.unit_off + e.elems] = \\\n                    grads[0][e.tensor][e.tensor_off:e.tensor_off + e.elems]", "pack reads worker 0 for every replica"),
    ("schedule.py", "key=lambda g: (-nbytes[g], g))", "key=lambda g: (nbytes[g], g))", "groups taken smallest first"),
    ("schedule.py", "key=lambda g: (-nbytes[g], g))", "key=lambda g: g)", "groups taken in queue order"),
    ("schedule.py", "        s = _earliest_start(slots, ready[g], dur[g], bp_len)\n        if s is not None:\n            slots[g] = Slot(BIN_BACKWARD, s, s + dur[g], 2)\n            continue\n        e = _latest_end(slots, need[g], dur[g], 0.0)\n        if e is not None:\n            slots[g] = Slot(BIN_FORWARD, e - dur[g], e, 2)\n",
     "        e = _latest_end(slots, need[g], dur[g], 0.0)\n        if e is not None:\n            slots[g] = Slot(BIN_FORWARD, e - dur[g], e, 2)\n            continue\n        s = _earliest_start(slots, ready[g], dur[g], bp_len)\n        if s is not None:\n            slots[g] = Slot(BIN_BACKWARD, s, s + dur[g], 2)\n", "forward pass tried before the backward pass"),
    ("schedule.py", "        if cost_bp <= cost_fp:", "        if cost_bp < cost_fp:", "equal cost resolved towards the forward pass"),
    ("schedule.py", "        if cost_bp <= cost_fp:", "        if cost_bp >= cost_fp:", "the side that adds MORE time is taken"),
    ("schedule.py", "        cost_bp = max(0.0, (s + dur[g]) - bp_end)", "        cost_bp = max(0.0, (s + dur[g]) - bp_len)", "overrun measured from the unextended backward pass"),
    ("schedule.py", "        cost_fp = max(0.0, fp_begin - (e - dur[g]))", "        cost_fp = dur[g]", "forward cost taken as the whole transfer time"),
    ("schedule.py", "    return max(good) if good else None", "    return min(good) if good else None", "forward slots packed from the start of the pass"),
    ("schedule.py", "    cands = [float(ready)] + [s.end for s in placed if s is not None and s.bin == BIN_BACKWARD and s.end >= ready]", "    cands = [0.0] + [s.end for s in placed if s is not None and s.bin == BIN_BACKWARD]", "backward boundary ignored"),
    ("schedule.py", "    return all(not (s.start < end and start < s.end) for s in placed if s is not None and s.bin == which)", "    return all(not (s.start <= end and start <= s.end) for s in placed if s is not None and s.bin == which)", "touching transfers treated as overlapping"),
    ("schedule.py", "    return all(not (s.start < end and start < s.end) for s in placed if s is not None and s.bin == which)", "    return all(not (s.start < end and start < s.end) for s in placed if s is not None)", "the two windows share one timeline"),
    ("schedule.py", "    dur = [net_a + net_b * float(b) for b in nbytes]", "    dur = [net_b * float(b) for b in nbytes]", "fixed cost per transfer dropped"),
    ("schedule.py", "        ready.append(max(ready_time[t] for t in members))", "        ready.append(min(ready_time[t] for t in members))", "batch boundary from its first updated member"),
    ("schedule.py", "        need.append(min(read_time[t] for t in members))", "        need.append(max(read_time[t] for t in members))", "batch boundary from its last read member"),
    ("schedule.py", "    overlap = (comm + compute - total) / lesser if lesser > 0.0 else 0.0", "    overlap = (comm + compute - total) / compute if lesser > 0.0 else 0.0", "overlap normalised by the computation time only"),
]


def load_variant(fname, old, new):
    """Both oracle modules re-executed from source under a private package name, one of them edited."""
    pkg = types.ModuleType("oracle_variant")
    pkg.__path__ = []
    mods = {}
    for name in ("plan.py", "aggregate.py", "ring_sim.py", "schedule.py"):
        with open(os.path.join(ROOT, "oracle", name)) as f:
            src = f.read()
        if name == fname:
            assert src.count(old) == 1, f"mutation target not found exactly once in {name}: {old!r}"
            src = src.replace(old, new)
        mod = types.ModuleType("oracle_variant." + name[:-3])
        mod.__package__ = "oracle_variant"
        sys.modules[mod.__name__] = mod
        sys.modules["oracle_variant"] = pkg
        exec(compile(src, os.path.join("oracle_variant", name), "exec"), mod.__dict__)
        mods[name[:-3]] = mod
        setattr(pkg, name[:-3], mod)
    return mods


def install(monkeypatch, mods):
    """Point every name the pin tests use at the variant."""
    exported = {}
    for mod in mods.values():
        for k, v in vars(mod).items():
            if not k.startswith("_") and callable(v) and getattr(v, "__module__", "").startswith("oracle_variant"):
                exported[k] = v
    for target in (oracle, oracle.plan, oracle.aggregate, oracle.schedule, pins_plan, pins_agg, pins_pat, pins_timed, pins_sched):
        for k, v in exported.items():
            if hasattr(target, k):
                monkeypatch.setattr(target, k, v)


def run_pins(fname=None):
    """All pins, or only those that look at the edited file."""
    pins = PLAN_PINS + AGG_PINS + SCHED_PINS
    if fname == "schedule.py":
        pins = SCHED_PINS
    elif fname is not None:
        pins = PLAN_PINS + AGG_PINS
    failed = []
    for pin in pins:
        try:
            pin()
        except AssertionError:
            failed.append(pin)
        except Exception:                      # a crash also counts as "noticed"
            failed.append(pin)
    return failed


def test_harness_passes_on_the_undamaged_oracle(monkeypatch):
    install(monkeypatch, load_variant(None, None, None))
    assert run_pins() == []


@pytest.mark.parametrize("fname,old,new,what", MUTATIONS, ids=[m[3] for m in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, fname, old, new, what):
    install(monkeypatch, load_variant(fname, old, new))
    assert run_pins(fname), f"no pin noticed: {what}"
