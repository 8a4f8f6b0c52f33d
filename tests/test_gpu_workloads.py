"""GPU parity at the benchmark's full sizes: all five configurations, in the launch
configuration bench.py times (defaults), every element of every replica against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2004_14020_amd as cm
from paper_2004_14020_amd.device import Replicas
from workloads.shapes import ALL, workload

from gpu_util import assert_same_bits, clone, lib_plan, make_inputs

pytestmark = pytest.mark.gpu


def cfg_of(wl):
    return oracle.Config(wl.world, wl.dtype, wl.batch_threshold_bytes, wl.split_mode, wl.max_depth,
                         wl.split_bytes, wl.align_bytes, wl.num_streams)


SEEDS = (0, 1, 200414020)


@pytest.mark.parametrize("name,seeds", [("mlp", SEEDS), ("resnet50", SEEDS), ("inception_v3", SEEDS), ("vgg16", SEEDS),
                                        ("transformer", SEEDS), ("alexnet_v2", (0,)), ("resnet_v2_152", (0,))])
@pytest.mark.parametrize("large_align", [256])
def test_workload_bit_exact(name, seeds, large_align):
    """Default launch options, tensors placed as bench.py places them (large tensors on 256-byte
    boundaries: tiles are cut on aligned blocks, with short first and last tiles)."""
    wl = workload(name)
    cfg = cfg_of(wl)
    elems = wl.elems()
    oplan = oracle.build_plan(cfg, elems)
    plan = lib_plan(cfg, elems)
    dev = Replicas(plan, elems, large_align=large_align)
    for seed in seeds:
        print(f"case: workload {name} seed {seed}: generating", flush=True)
        grads = make_inputs(cfg, elems, seed)
        dev.upload(grads)
        print("  device allreduce", flush=True)
        plan.allreduce()
        got = dev.download()
        print("  oracle", flush=True)
        # accuracy bound on a few tensors before the inputs are overwritten in place
        check = sorted(set([0, len(elems) // 2, len(elems) - 1]))
        mean = {t: oracle.mean_f64(oplan, grads, t) for t in check}
        mag = {t: oracle.abs_sum_f64(oplan, grads, t) for t in check}
        oracle.allreduce(oplan, grads)
        print("  compare", flush=True)
        assert_same_bits(got, grads, f"{name} seed {seed}")
        for t in check:
            y = got[0][t]
            y = (oracle.bf16_to_f32(y) if cfg.dtype == oracle.BF16 else y).astype(np.float64)
            slack = 2.0 ** -8 * np.abs(mean[t]) if cfg.dtype == oracle.BF16 else 0.0
            assert (np.abs(y - mean[t]) <= 4e-7 * mag[t] + slack).all()
        del grads, got
    plan.close()


@pytest.mark.parametrize("name", ["vgg16", "transformer"])
def test_workload_bit_exact_with_the_two_stream_pipeline_and_aligned_tensors(name):
    """The two-stream pipeline (units alternating over the caller's and the internal stream,
    launches of at least 64 MiB) on tensors that start on 64 KiB boundaries."""
    wl = workload(name)
    cfg = cfg_of(wl)
    elems = wl.elems()
    print(f"case: workload {name} pipelined: generating", flush=True)
    grads = make_inputs(cfg, elems, 3)
    plan = lib_plan(cfg, elems, {cm.OPT_LAUNCH_MODE: cm.LAUNCH_PER_UNIT})
    dev = Replicas(plan, elems, large_align=65536)
    dev.upload(grads)
    plan.allreduce()
    got = dev.download()
    oracle.allreduce(oracle.build_plan(cfg, elems), grads)
    assert_same_bits(got, grads, f"{name} pipelined")
    plan.close()


def test_staged_path_on_a_full_workload():
    """The pack -> reduce -> unpack route through the fused workspace, per-unit launches, on
    the configuration dominated by small tensors."""
    wl = workload("inception_v3")
    cfg = cfg_of(wl)
    elems = wl.elems()
    print("case: inception_v3 staged/per-unit", flush=True)
    grads = make_inputs(cfg, elems, 2)
    plan = lib_plan(cfg, elems, {cm.OPT_BATCH_PATH: cm.BATCH_STAGED, cm.OPT_LAUNCH_MODE: cm.LAUNCH_PER_UNIT})
    dev = Replicas(plan, elems)
    dev.upload(grads)
    plan.allreduce()
    got = dev.download()
    oracle.allreduce(oracle.build_plan(cfg, elems), grads)
    assert_same_bits(got, grads, "inception staged")
    plan.close()


def test_offsets_beyond_4_gib():
    """One tensor of 4.5 GiB per replica (W = 2): byte offsets inside a tensor exceed 32 bits."""
    n = (4608 << 20) // 4 + 3
    W = 2
    cfg = oracle.Config(W, oracle.F32, 1 << 20, oracle.SPLIT_FIXED, 8, 1 << 30, 16, 2)
    print("case: 4.5 GiB tensor", flush=True)
    base = np.arange(n, dtype=np.uint32)
    grads = []
    for w in range(W):
        v = ((base * np.uint32(2654435761) + np.uint32(w * 977)) >> np.uint32(9)).astype(np.float32)
        v *= np.float32(2.0 ** -10 * (w + 1))
        grads.append([v])
    plan = lib_plan(cfg, [n])
    dev = Replicas(plan, [n])
    dev.upload(grads)
    plan.allreduce()
    got = dev.download()
    oracle.allreduce(oracle.build_plan(cfg, [n]), grads)
    assert_same_bits(got, grads, "4.5 GiB tensor")
    plan.close()
