"""GPU parity: the HIP path against the CPU oracle, bit for bit, through the C ABI.

Integer/byte work (plan, pack, unpack) and the fixed-order fp32 ring sums both have exactly
one correct bit pattern per element, so every comparison is on raw bits.  The float64 bound
|y - mean| <= 4e-7 * sum_w |g_w| is checked as well.
"""
import numpy as np
import pytest

import oracle
import paper_2004_14020_amd as cm
from paper_2004_14020_amd.device import Replicas
from workloads.shapes import ALL, workload

from gpu_util import assert_same_bits, bits, clone, lib_plan, make_inputs, oracle_result

pytestmark = pytest.mark.gpu

# spans several reduce tiles (1024 vectors = 4096 fp32 each), ragged tails, members that are
# smaller than one granule, and units with fewer granules than workers (empty ring segments)
SMALL_ELEMS = (10, 700, 33, 50000, 1, 257, 30011, 64, 129, 3, 4097, 100000, 7, 20000)


def small_cfg(W, dtype, streams=2, T=8192, mode=oracle.SPLIT_FIXED, S=65536, align=16):
    return oracle.Config(W, dtype, T, mode, 8, S, align, streams)


@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 8, 16, 33])
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_each_stage_matches_the_oracle(W, dtype):
    print(f"case: stages W={W} dtype={dtype}", flush=True)
    cfg = small_cfg(W, dtype)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=W)
    oplan = oracle.build_plan(cfg, elems)
    ref = clone(grads)
    ofused = oracle.new_fused(oplan)

    plan = lib_plan(cfg, elems)
    dev = Replicas(plan, elems)
    dev.upload(grads)
    dev.fill_fused(0xA5)

    plan.pack()
    oracle.pack(oplan, ref, ofused)
    assert np.array_equal(bits(dev.download_fused()), bits(ofused)), "fused buffer after pack"
    assert_same_bits(dev.download(), ref, "tensors after pack")

    plan.ring_reduce()
    oracle.ring_reduce(oplan, ref, ofused)
    assert np.array_equal(bits(dev.download_fused()), bits(ofused)), "fused buffer after ring_reduce"
    assert_same_bits(dev.download(), ref, "tensors after ring_reduce")

    plan.unpack()
    oracle.unpack(oplan, ref, ofused)
    assert_same_bits(dev.download(), ref, "tensors after unpack")
    plan.close()


MODES = [(cm.LAUNCH_PER_UNIT, cm.BATCH_STAGED), (cm.LAUNCH_PER_UNIT, cm.BATCH_DIRECT),
         (cm.LAUNCH_PER_STREAM, cm.BATCH_STAGED), (cm.LAUNCH_PER_STREAM, cm.BATCH_DIRECT)]


@pytest.mark.parametrize("W,dtype", [(4, oracle.F32), (8, oracle.F32), (8, oracle.BF16), (16, oracle.F32),
                                     (5, oracle.F32), (3, oracle.BF16)])
@pytest.mark.parametrize("launch,batch", MODES)
@pytest.mark.parametrize("streams", [1, 2])
def test_allreduce_all_modes(W, dtype, launch, batch, streams):
    print(f"case: allreduce W={W} dtype={dtype} launch={launch} batch={batch} streams={streams}", flush=True)
    cfg = small_cfg(W, dtype, streams)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=100 + W)
    ref = oracle_result(cfg, elems, grads)
    plan = lib_plan(cfg, elems, {cm.OPT_LAUNCH_MODE: launch, cm.OPT_BATCH_PATH: batch})
    dev = Replicas(plan, elems)
    dev.upload(grads)
    plan.allreduce()
    assert_same_bits(dev.download(), ref, "allreduce")
    plan.close()


@pytest.mark.parametrize("opts", [
    {cm.OPT_TILE_VECS: 64}, {cm.OPT_TILE_VECS: 256, cm.OPT_UNROLL: 4}, {cm.OPT_TILE_VECS: 4096, cm.OPT_UNROLL: 1},
    {cm.OPT_MAX_GRID: 7}, {cm.OPT_NONTEMPORAL: 0}, {cm.OPT_UNROLL: 2, cm.OPT_MAX_GRID: 300},
    {cm.OPT_LAUNCH_MIN_BYTES: 1 << 16}, {cm.OPT_LAUNCH_MIN_BYTES: 1 << 30, cm.OPT_BATCH_PATH: cm.BATCH_STAGED},
    {cm.OPT_LAUNCH_MIN_BYTES: 200000, cm.OPT_BATCH_PATH: cm.BATCH_STAGED},
    {cm.OPT_STREAM_MAJOR: 4, cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TILE_VECS: 4096}, {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TILE_VECS: 8192},
    {cm.OPT_STREAM_MAJOR: 4, cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TILE_VECS: 8192}, {cm.OPT_STREAM_MAJOR: 8, cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TILE_VECS: 2048, cm.OPT_BLOCK: 256},
    {cm.OPT_STREAM_MAJOR: 2, cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TILE_VECS: 512, cm.OPT_BLOCK: 256},
    {cm.OPT_STREAM_MAJOR: 4, cm.OPT_LONG_RUN_BYTES: 4096, cm.OPT_TILE_VECS: 1024, cm.OPT_BLOCK: 256, cm.OPT_BATCH_PATH: cm.BATCH_STAGED},
    {cm.OPT_LONG_RUN_BYTES: 1}, {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_STREAM_MAJOR: 0}, {cm.OPT_LONG_RUN_BYTES: 1 << 40},
    {cm.OPT_LONG_RUN_BYTES: 4096, cm.OPT_TAIL_TILES: 0}, {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TAIL_TILES: 5, cm.OPT_TILE_VECS: 2048, cm.OPT_BLOCK: 256},
    {cm.OPT_LONG_RUN_BYTES: 4096, cm.OPT_MERGE_SMALL_BYTES: 0}, {cm.OPT_LONG_RUN_BYTES: 4096, cm.OPT_MERGE_SMALL_BYTES: 1 << 30},
    {cm.OPT_LAUNCH_MODE: cm.LAUNCH_PER_UNIT, cm.OPT_LONG_RUN_BYTES: 4096, cm.OPT_LONG_LAUNCH_MIN_BYTES: 0},
    {cm.OPT_LONG_RUN_BYTES: 4096, cm.OPT_MERGE_SMALL_BYTES: 1 << 30, cm.OPT_SMALL_TILE_VECS: 1024, cm.OPT_STREAM_MAJOR: 2, cm.OPT_TILE_VECS: 2048},
    {cm.OPT_LONG_RUN_BYTES: 100000, cm.OPT_SMALL_TILE_VECS: 64}, {cm.OPT_LONG_RUN_BYTES: 2048, cm.OPT_LONG_LAUNCH_MIN_BYTES: 0},
    {cm.OPT_LONG_RUN_BYTES: 65536, cm.OPT_SMALL_BLOCK: 512, cm.OPT_SMALL_TILE_VECS: 1024, cm.OPT_BATCH_PATH: cm.BATCH_STAGED},
    {cm.OPT_BLOCK: 256}, {cm.OPT_BLOCK: 1024, cm.OPT_TILE_VECS: 2048}, {cm.OPT_BLOCK: 1024, cm.OPT_TILE_VECS: 128},
])
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_launch_options_do_not_change_results(opts, dtype):
    print(f"case: options {opts} dtype={dtype}", flush=True)
    cfg = small_cfg(8, dtype)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=7)
    ref = oracle_result(cfg, elems, grads)
    plan = lib_plan(cfg, elems, opts)
    dev = Replicas(plan, elems)
    dev.upload(grads)
    plan.allreduce()
    assert_same_bits(dev.download(), ref, f"options {opts}")
    plan.close()


@pytest.mark.parametrize("align", [16, 64, 256])
@pytest.mark.parametrize("mode,S", [(oracle.SPLIT_NONE, 0), (oracle.SPLIT_ADAPTIVE, 16384)])
def test_alignment_and_split_modes(align, mode, S):
    print(f"case: align={align} mode={mode}", flush=True)
    cfg = small_cfg(8, oracle.F32, 2, 16384, mode, S, align)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=align)
    ref = oracle_result(cfg, elems, grads)
    for batch in (cm.BATCH_STAGED, cm.BATCH_DIRECT):
        plan = lib_plan(cfg, elems, {cm.OPT_BATCH_PATH: batch})
        dev = Replicas(plan, elems)
        dev.upload(grads)
        plan.allreduce()
        assert_same_bits(dev.download(), ref, f"align {align} batch path {batch}")
        plan.close()


# Segment boundaries wherever odd tensor sizes put them, for every kernel (the specialised chain
# kernels, stream-major with 2, 4 and 8 vectors per lane and all-at-once, and the kernel for any
# world size, whose tiles may straddle a boundary): tiles of every length from one vector up, whole
# groups of vectors, the rows left over after them, ragged ends, the boundary in any of those.
BOUNDARY_SHAPES = [
    {cm.OPT_LONG_RUN_BYTES: 1}, {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TILE_VECS: 8192},
    {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_STREAM_MAJOR: 4, cm.OPT_TILE_VECS: 8192},
    {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_STREAM_MAJOR: 2, cm.OPT_TILE_VECS: 1024, cm.OPT_BLOCK: 256},
    {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_STREAM_MAJOR: 0, cm.OPT_TILE_VECS: 2048},
    {cm.OPT_LONG_RUN_BYTES: 1 << 40}, {cm.OPT_LONG_RUN_BYTES: 1 << 40, cm.OPT_SMALL_TILE_VECS: 1024, cm.OPT_SMALL_BLOCK: 512},
    {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TAIL_TILES: 0, cm.OPT_TILE_VECS: 2560},
    # no pieces at the end of a stream: whole 64 KiB and 128 KiB tiles, i.e. whole groups of vectors per lane
    {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TAIL_TILES: 0}, {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TAIL_TILES: 0, cm.OPT_TILE_VECS: 8192},
    {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TAIL_TILES: 2, cm.OPT_TILE_VECS: 16384},
]


@pytest.mark.parametrize("W", [2, 3, 4, 5, 7, 8, 12, 16, 24])
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_segment_boundaries_at_odd_positions(W, dtype):
    print(f"case: odd segment boundaries W={W} dtype={dtype}", flush=True)
    # chunks only (no batching, no splitting of tensors): segment boundaries wherever the sizes put them
    cfg = oracle.Config(W, dtype, 0, oracle.SPLIT_NONE, 1, 0, 16, 1)
    elems = [100000, 4099, 70001, 16384, 262144 + 4, 50, 33333, 8192 * W, 1 << 20]
    grads = make_inputs(cfg, elems, seed=900 + W)
    ref = oracle_result(cfg, elems, grads)
    # world sizes without a kernel of their own get tiles across the boundaries, unless switched off
    splits = (1,) if W in (2, 4, 8, 16) else (1, 0)
    for opts in [{**o, cm.OPT_SPLIT_TILES: sp} for o in BOUNDARY_SHAPES for sp in splits]:
        for phase in (0, 1280):
            plan = lib_plan(cfg, elems, opts)
            dev = Replicas(plan, elems, arena_phase=phase)
            dev.upload(grads)
            plan.allreduce()
            assert_same_bits(dev.download(), ref, f"options {opts}, arena phase {phase}")
            plan.close()


@pytest.mark.parametrize("phase", [0, 256, 1280, 4096 - 256, 65536 - 512])
@pytest.mark.parametrize("align_tiles", [0, 1, 2, 3])
def test_tiles_cut_on_aligned_blocks_give_the_same_bits(phase, align_tiles):
    """Every replica at the same position inside an aligned block: small tiles (bit 0) and long
    tiles (bit 1) are then cut on multiples of their size in memory, with a short first tile."""
    print(f"case: aligned tiles phase={phase} align_tiles={align_tiles}", flush=True)
    cfg = small_cfg(8, oracle.F32)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=11)
    ref = oracle_result(cfg, elems, grads)
    for extra in ({}, {cm.OPT_LONG_RUN_BYTES: 8192, cm.OPT_TILE_VECS: 256, cm.OPT_BLOCK: 256, cm.OPT_BATCH_PATH: cm.BATCH_STAGED}):
        plan = lib_plan(cfg, elems, {cm.OPT_ALIGN_TILES: align_tiles, cm.OPT_SMALL_TILE_VECS: 64, **extra})
        dev = Replicas(plan, elems, slot_align=256, large_align=256, arena_phase=phase)
        dev.upload(grads)
        plan.allreduce()
        assert_same_bits(dev.download(), ref, f"phase {phase}, align_tiles {align_tiles}, {extra}")
        plan.close()


@pytest.mark.parametrize("phase", [0, 256, 1280, 20480, 39936, 65536 - 512])
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_long_tiles_cut_on_aligned_blocks_give_the_same_bits(phase, dtype):
    """Long launches over tensors that do not start on a tile boundary in memory: the first and
    last tile of every run are short (1 to 4 rows of lanes, the last row ragged) and are walked
    by the stream-major kernel like the whole ones."""
    print(f"case: long tiles phase={phase} dtype={dtype}", flush=True)
    cfg = oracle.Config(8, dtype, 8192, oracle.SPLIT_FIXED, 8, 1 << 20, 16, 2)
    elems = [600000, 33, 262144 + 4, 5000, 1 << 20]
    grads = make_inputs(cfg, elems, seed=12)
    ref = oracle_result(cfg, elems, grads)
    for tile, block, sm in ((4096, 1024, 4), (1024, 256, 4), (2048, 1024, 2), (8192, 1024, 8), (0, 1024, 8), (2048, 256, 8)):
        plan = lib_plan(cfg, elems, {cm.OPT_LONG_RUN_BYTES: 4096,
                                     cm.OPT_TILE_VECS: tile, cm.OPT_BLOCK: block, cm.OPT_STREAM_MAJOR: sm})
        dev = Replicas(plan, elems, slot_align=256, large_align=256, arena_phase=phase)
        dev.upload(grads)
        plan.allreduce()
        assert_same_bits(dev.download(), ref, f"phase {phase}, tile {tile}, block {block}")
        plan.close()


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_replicas_at_different_positions_inside_aligned_blocks(dtype):
    """Replicas that disagree on where a tensor sits inside an aligned block of memory: tiles are
    cut for the position most of them share (or for none); the bits do not depend on it."""
    print(f"case: replicas at different phases dtype={dtype}", flush=True)
    cfg = oracle.Config(8, dtype, 8192, oracle.SPLIT_FIXED, 8, 1 << 20, 16, 2)
    elems = [600000, 33, 262144 + 4, 5000]
    grads = make_inputs(cfg, elems, seed=13)
    ref = oracle_result(cfg, elems, grads)
    for phases in ([0, 0, 256, 0, 4096, 0, 0, 512], [256 * w for w in range(8)], [1024] * 4 + [2048] * 4):
        plan = lib_plan(cfg, elems, {cm.OPT_LONG_RUN_BYTES: 4096})
        dev = Replicas(plan, elems, slot_align=256, large_align=256, arena_phases=phases)
        dev.upload(grads)
        plan.allreduce()
        assert_same_bits(dev.download(), ref, f"phases {phases}")
        plan.close()


def test_batching_off_and_single_tiny_tensor():
    for elems, T in (([1], 0), ([3, 5], 0), ([2], 1 << 20), ([5, 3, 9], 1 << 20)):
        for W in (1, 4, 16):
            print(f"case: tiny elems={elems} T={T} W={W}", flush=True)
            cfg = oracle.Config(W, oracle.F32, T, oracle.SPLIT_NONE, 8, 0, 16, 2)
            grads = make_inputs(cfg, elems, seed=1)
            ref = oracle_result(cfg, elems, grads)
            plan = lib_plan(cfg, elems)
            dev = Replicas(plan, elems)
            dev.upload(grads)
            plan.allreduce()
            assert_same_bits(dev.download(), ref, "tiny")
            plan.close()


def test_special_values_follow_ieee():
    """Denormals are kept (no flush to zero), infinities propagate, and the hand-worked
    rotation example gives the four distinct per-segment results."""
    W, n = 4, 52
    cfg = oracle.Config(W, oracle.F32, 0)
    tiny = np.float32(1e-45)
    rows = [np.full(n, v, dtype=np.float32) for v in (tiny, tiny * 3, -tiny, tiny * 5)]
    rows[0][5] = np.inf
    rows[1][6] = -np.inf
    rows[2][7] = np.float32(3.0e38)
    rows[3][7] = np.float32(3.0e38)
    grads = [[r] for r in rows]
    ref = oracle_result(cfg, [n], grads)
    plan = lib_plan(cfg, [n])
    dev = Replicas(plan, [n])
    dev.upload(grads)
    plan.allreduce()
    got = dev.download()
    assert_same_bits(got, ref, "special values")
    assert got[0][0][0] == tiny * 2 and np.isinf(got[0][0][5]) and np.isinf(got[0][0][7])
    plan.close()

    ex = [1.0, 33554432.0, -33554432.0, 5.0]
    grads = [[np.full(n, g, dtype=np.float32)] for g in ex]
    plan = lib_plan(cfg, [n])
    dev = Replicas(plan, [n])
    dev.upload(grads)
    plan.allreduce()
    got = dev.download()
    seg = plan.segments(0)
    for c, want in enumerate([1.5, 1.0, 2.0, 1.25]):
        for w in range(W):
            assert (got[w][0][seg[c]:seg[c + 1]] == np.float32(want)).all()
    plan.close()


def test_bf16_special_values_follow_ieee():
    """bf16 in and out: infinities propagate, Inf - Inf and NaN inputs (quiet or signalling) give
    a NaN (payload bits are not compared), an fp32 sum that overflows gives Inf, bf16 denormals
    are widened, added and rounded without a flush to zero, and signed zeros keep their sign.
    Everything that is not a NaN is compared bit for bit."""
    W, n = 4, 72
    cfg = oracle.Config(W, oracle.BF16, 0)
    rows = [np.full(n, b, dtype=np.uint16) for b in (0x0001, 0x0003, 0x8001, 0x0005)]   # denormals
    rows[0][5] = 0x7F80                       # +Inf and finite values
    rows[1][6] = 0xFF80                       # -Inf
    rows[2][8], rows[3][8] = 0x7F80, 0xFF80   # Inf - Inf
    rows[0][9] = 0x7FC1                       # quiet NaN with a payload
    rows[3][10] = 0x7F81                      # signalling NaN
    for r in rows:
        r[12] = 0x7F7F                        # 4 x the largest bf16: the fp32 sum overflows
        r[13] = 0x8000                        # -0 + -0 + -0 + -0
    rows[1][14], rows[2][14] = 0x8000, 0x0000  # mixed zeros (the others are denormals there)
    rows[0][15], rows[1][15], rows[2][15], rows[3][15] = 0x0000, 0x8000, 0x8000, 0x0000
    rows[0][16], rows[1][16], rows[2][16], rows[3][16] = 0x007F, 0x007F, 0x0001, 0x0001   # denormals summing to a normal
    rows[0][17], rows[1][17], rows[2][17], rows[3][17] = 0x3F80, 0x3B80, 0x0000, 0x0000   # ties at the bf16 rounding:
    rows[0][18], rows[1][18], rows[2][18], rows[3][18] = 0x3F80, 0x3B80, 0x3B80, 0x3B80   # one down, one up, to even
    grads = [[r] for r in rows]
    ref = oracle_result(cfg, [n], grads)
    for opts in ({}, {cm.OPT_LONG_RUN_BYTES: 1}):
        plan = lib_plan(cfg, [n], opts)
        dev = Replicas(plan, [n])
        dev.upload(grads)
        plan.allreduce()
        got = dev.download()
        plan.close()
        want = ref[0][0]
        is_nan = ((want & 0x7F80) == 0x7F80) & ((want & 0x007F) != 0)
        assert is_nan[[8, 9, 10]].all() and is_nan.sum() == 3
        for w in range(W):
            g = got[w][0]
            assert (((g & 0x7F80) == 0x7F80) & ((g & 0x007F) != 0))[is_nan].all(), "NaN in, NaN out"
            assert np.array_equal(g[~is_nan], want[~is_nan])
        g = got[0][0]
        assert g[5] == 0x7F80 and g[6] == 0xFF80 and g[12] == 0x7F80 and g[13] == 0x8000 and g[15] == 0x0000
        assert g[0] == 0x0002                     # (1 + 3 - 1 + 5) / 4 denormal units
        assert g[17] == 0x3E80 and g[18] == 0x3E82


def test_repeated_calls_are_race_free_and_idempotent_on_the_result():
    """20 back-to-back allreduce calls on one and on two streams: after the first call all
    replicas are equal, so for W = 4 every further call must leave the bits unchanged
    (x + x, 3x -> 4x is recovered exactly); any stream-ordering mistake would show."""
    import torch
    for streams in (1, 2):
        print(f"case: repeat streams={streams}", flush=True)
        cfg = small_cfg(4, oracle.F32, streams)
        elems = list(SMALL_ELEMS)
        grads = make_inputs(cfg, elems, seed=5)
        ref = oracle_result(cfg, elems, grads)
        plan = lib_plan(cfg, elems, {cm.OPT_BATCH_PATH: cm.BATCH_STAGED, cm.OPT_LAUNCH_MODE: cm.LAUNCH_PER_UNIT})
        dev = Replicas(plan, elems)
        dev.upload(grads)
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            for _ in range(20):
                plan.allreduce(s.cuda_stream)
        s.synchronize()
        assert_same_bits(dev.download(), ref, "repeat")
        plan.close()


def test_accuracy_bound_against_float64():
    cfg = small_cfg(16, oracle.F32)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=3)
    oplan = oracle.build_plan(cfg, elems)
    mean = [oracle.mean_f64(oplan, grads, t) for t in range(len(elems))]
    mag = [oracle.abs_sum_f64(oplan, grads, t) for t in range(len(elems))]
    plan = lib_plan(cfg, elems)
    dev = Replicas(plan, elems)
    dev.upload(grads)
    plan.allreduce()
    got = dev.download()
    for t in range(len(elems)):
        assert (np.abs(got[0][t].astype(np.float64) - mean[t]) <= 4e-7 * mag[t]).all()
    plan.close()


def test_profile_counters():
    cfg = small_cfg(8, oracle.F32)
    elems = list(SMALL_ELEMS)
    plan = lib_plan(cfg, elems, {cm.OPT_BATCH_PATH: cm.BATCH_STAGED, cm.OPT_LAUNCH_MODE: cm.LAUNCH_PER_STREAM})
    dev = Replicas(plan, elems)
    dev.upload(make_inputs(cfg, elems, seed=3))
    for level in (1, 2):
        plan.profile(level)
        for _ in range(3):
            plan.allreduce()
        st = plan.profile_read()
        # every run of this small case is short: one launch over small tiles per stream and call,
        # none over long tiles; pack/unpack only on streams that own batch units
        red = st[cm.K_REDUCE_SMALL]
        assert red["launches"] == 6 and st[cm.K_REDUCE]["launches"] == 0
        units = plan.units()
        assert red["elements"] == 3 * sum(u.elems for u in units)        # batch units with their padding
        assert st[cm.K_PACK]["launches"] == st[cm.K_UNPACK]["launches"] and st[cm.K_PACK]["launches"] in (3, 6)
        seq = st[cm.K_SEQUENCE]
        assert seq["launches"] == 6 and seq["calls"] == 3 and seq["total_ms"] > 0 and seq["span_ms"] > 0
        if level == 2:
            assert red["calls"] == 3 and red["total_ms"] > 0
            assert red["total_ms"] <= seq["total_ms"]
        else:
            assert red["total_ms"] == 0
    # with a lower limit the long runs go out in launches of their own
    plan.close()
    plan = lib_plan(cfg, elems, {cm.OPT_LONG_RUN_BYTES: 4096})
    dev = Replicas(plan, elems)
    dev.upload(make_inputs(cfg, elems, seed=3))
    plan.profile(1)
    plan.allreduce()
    st = plan.profile_read()
    # AUTO: one launch per class on the caller's stream, and the few small tiles join the long ones
    assert st[cm.K_REDUCE]["launches"] == 1 and st[cm.K_REDUCE_SMALL]["launches"] == 0
    assert st[cm.K_REDUCE]["elements"] == sum(elems)                                      # in place: no padding
    plan.set_option(cm.OPT_MERGE_SMALL_BYTES, 0)
    plan.profile(1)
    plan.allreduce()
    st = plan.profile_read()
    assert st[cm.K_REDUCE]["launches"] == 1 and st[cm.K_REDUCE_SMALL]["launches"] == 1
    assert st[cm.K_REDUCE]["elements"] + st[cm.K_REDUCE_SMALL]["elements"] == sum(elems)
    assert st[cm.K_REDUCE]["elements"] > 0 and st[cm.K_REDUCE_SMALL]["elements"] > 0
    plan.profile(0)
    plan.close()


# ------------------------------------------------------------------ other patterns, timed plans
@pytest.mark.parametrize("pattern", [oracle.PATTERN_HALVING_DOUBLING, oracle.PATTERN_SHUFFLE])
@pytest.mark.parametrize("W,dtype", [(1, oracle.F32), (2, oracle.F32), (4, oracle.F32), (8, oracle.F32), (16, oracle.F32),
                                     (4, oracle.BF16), (8, oracle.BF16), (16, oracle.BF16),
                                     (32, oracle.F32), (64, oracle.F32), (32, oracle.BF16), (64, oracle.BF16)])
def test_other_patterns_match_the_oracle(pattern, W, dtype):
    print(f"case: pattern={pattern} W={W} dtype={dtype}", flush=True)
    cfg = oracle.Config(W, dtype, 8192, oracle.SPLIT_FIXED, 8, 65536, 16, 2, pattern)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=40 + W)
    ref = oracle_result(cfg, elems, grads)
    for batch in (cm.BATCH_DIRECT, cm.BATCH_STAGED):
        plan = lib_plan(cfg, elems, {cm.OPT_BATCH_PATH: batch})
        dev = Replicas(plan, elems)
        dev.upload(grads)
        plan.allreduce()
        assert_same_bits(dev.download(), ref, f"pattern {pattern} batch path {batch}")
        plan.close()


@pytest.mark.parametrize("W", [6, 12, 24, 64])
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_world_sizes_of_the_generic_kernel_including_the_maximum(W, dtype):
    """World sizes without a specialised kernel, up to CARAMEL_MAX_WORLD, with large tiles too."""
    print(f"case: generic W={W} dtype={dtype}", flush=True)
    cfg = small_cfg(W, dtype)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=60 + W)
    ref = oracle_result(cfg, elems, grads)
    for opts in ({}, {cm.OPT_LONG_RUN_BYTES: 1, cm.OPT_TILE_VECS: 4096}, {cm.OPT_LONG_RUN_BYTES: 1 << 40}):
        plan = lib_plan(cfg, elems, opts)
        dev = Replicas(plan, elems)
        dev.upload(grads)
        plan.allreduce()
        assert_same_bits(dev.download(), ref, f"W {W} options {opts}")
        plan.close()


def test_two_plans_on_two_streams_at_once():
    """Two independent plans queued on two caller streams with no synchronisation between them:
    each has its own tables, internal stream and events, so both results must be exact."""
    import torch
    print("case: two plans at once", flush=True)
    cases = []
    for i, (W, dtype) in enumerate(((8, oracle.F32), (4, oracle.BF16))):
        cfg = small_cfg(W, dtype)
        elems = list(SMALL_ELEMS) + [300000 + i]
        grads = make_inputs(cfg, elems, seed=70 + i)
        plan = lib_plan(cfg, elems, {cm.OPT_PIPELINE_MIN_BYTES: 0})
        dev = Replicas(plan, elems)
        dev.upload(grads)
        cases.append((cfg, elems, grads, plan, dev, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for _, _, _, plan, _, stream in cases:
        plan.allreduce(stream.cuda_stream)
    torch.cuda.synchronize()
    for cfg, elems, grads, plan, dev, _ in cases:
        assert_same_bits(dev.download(), oracle_result(cfg, elems, grads), f"plan with W {cfg.world}")
        plan.close()


@pytest.mark.parametrize("W", [3, 5, 33])
def test_shuffle_with_any_world_size(W):
    cfg = oracle.Config(W, oracle.F32, 8192, oracle.SPLIT_FIXED, 8, 65536, 16, 2, oracle.PATTERN_SHUFFLE)
    elems = list(SMALL_ELEMS)
    grads = make_inputs(cfg, elems, seed=W)
    ref = oracle_result(cfg, elems, grads)
    plan = lib_plan(cfg, elems)
    dev = Replicas(plan, elems)
    dev.upload(grads)
    plan.allreduce()
    assert_same_bits(dev.download(), ref, "shuffle")
    plan.close()


def test_pattern_worked_example_on_the_gpu():
    n = 52
    ex = [1.0, 33554432.0, -33554432.0, 5.0]
    for pattern, want in ((oracle.PATTERN_HALVING_DOUBLING, 1.0), (oracle.PATTERN_SHUFFLE, 1.25)):
        cfg = oracle.Config(4, oracle.F32, 0, pattern=pattern)
        plan = lib_plan(cfg, [n])
        dev = Replicas(plan, [n])
        dev.upload([[np.full(n, g, dtype=np.float32)] for g in ex])
        plan.allreduce()
        got = dev.download()
        for w in range(4):
            assert (got[w][0] == np.float32(want)).all()
        plan.close()


def test_timing_aware_plan_runs_bit_exact():
    elems = list(SMALL_ELEMS)
    cfg = small_cfg(8, oracle.F32)
    times = [float(3 * i) for i in range(len(elems))]
    grads = make_inputs(cfg, elems, seed=9)
    oplan = oracle.build_plan(cfg, elems, times, 2.0, 0.0005)
    assert len(oplan.units) != len(oracle.build_plan(cfg, elems).units)      # the timing changes the batches
    ref = clone(grads)
    oracle.allreduce(oplan, ref)
    plan = cm.Plan(cfg.world, elems, dtype=cfg.dtype, batch_threshold_bytes=cfg.batch_threshold_bytes,
                   split_mode=cfg.split_mode, split_bytes=cfg.split_bytes, ready_time=times, net_a=2.0, net_b=0.0005)
    assert plan.counts()[0] == len(oplan.units)
    dev = Replicas(plan, elems)
    dev.upload(grads)
    plan.allreduce()
    assert_same_bits(dev.download(), ref, "timed plan")
    plan.close()


def test_trace_log_names_every_launch():
    """CARAMEL_TRACE=1 is read once per process, so the traced call runs in a child process."""
    import os
    import subprocess
    import sys
    print("case: CARAMEL_TRACE host log", flush=True)
    code = (
        "import torch, paper_2004_14020_amd as cm\n"
        "elems = [300000, 100, 5000]\n"
        "plan = cm.Plan(4, elems, batch_threshold_bytes=65536, split_mode=cm.SPLIT_FIXED, split_bytes=1 << 19, num_streams=2)\n"
        "g = [[torch.ones(n, device='cuda:0') for n in elems] for _ in range(4)]\n"
        "plan.bind([[t.data_ptr() for t in r] for r in g], None)\n"
        "plan.allreduce(torch.cuda.current_stream().cuda_stream)\n"
        "torch.cuda.synchronize()\n"
        "assert all(float(t.min()) == 1.0 and float(t.max()) == 1.0 for r in g for t in r)\n"
    )
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, CARAMEL_TRACE="1", PYTHONPATH=root)
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=240)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stderr.splitlines() if l.startswith("caramel:")]
    units = [l for l in lines if l.startswith("caramel: unit ")]
    launches = [l for l in lines if " reduce " in l]
    assert len(units) == 4 and any("batch" in l for l in units) and sum("chunk" in l for l in units) == 3, lines
    assert launches and all("call 1 " in l for l in launches), lines
