"""caramel_allreduce under HIP graph capture: the call allocates nothing and issues only kernel
launches and event records/waits, so it can be recorded once and replayed.  Every replay, with
fresh inputs and the program's own eager work and synchronisation in between, must give the
oracle's bits."""
import pytest
import torch

import oracle
import paper_2004_14020_amd as cm
from paper_2004_14020_amd.device import Replicas

from gpu_util import assert_same_bits, lib_plan, make_inputs, oracle_result

pytestmark = pytest.mark.gpu

ELEMS = (10, 700, 33, 50000, 1, 257, 30011, 64, 129, 3, 4097, 100000, 7, 20000)


@pytest.mark.parametrize("pipelined", [False, True], ids=["one_stream", "two_streams"])
@pytest.mark.parametrize("batch_path", [cm.BATCH_STAGED, cm.BATCH_DIRECT], ids=["staged", "direct"])
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16], ids=["f32", "bf16"])
def test_captured_allreduce_replays_bit_exact(pipelined, batch_path, dtype):
    print(f"case: graph capture pipelined={pipelined} batch_path={batch_path} dtype={dtype}", flush=True)
    cfg = oracle.Config(8, dtype, 8192, oracle.SPLIT_FIXED, 8, 65536, 16, 2)
    elems = list(ELEMS)
    plan = lib_plan(cfg, elems, {cm.OPT_PIPELINE_MIN_BYTES: 0 if pipelined else 1 << 40,
                                 cm.OPT_BATCH_PATH: batch_path})
    dev = Replicas(plan, elems)
    dev.upload(make_inputs(cfg, elems, seed=0))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                      # captures on a side stream; nothing runs yet
        plan.allreduce(torch.cuda.current_stream().cuda_stream)
    for seed in (1, 2, 3):
        grads = make_inputs(cfg, elems, seed=seed)
        dev.upload(grads)                              # eager copies and a synchronise between replays
        dev.fill_fused(0xA5)
        graph.replay()
        torch.cuda.synchronize()
        assert_same_bits(dev.download(), oracle_result(cfg, elems, grads), f"replay with seed {seed}")
    # the plan still works eagerly afterwards
    grads = make_inputs(cfg, elems, seed=4)
    dev.upload(grads)
    plan.allreduce(torch.cuda.current_stream().cuda_stream)
    assert_same_bits(dev.download(), oracle_result(cfg, elems, grads), "eager call after the replays")
    del graph
    plan.close()
