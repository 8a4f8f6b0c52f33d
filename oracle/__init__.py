"""CPU oracle for the Caramel aggregation hot path.

TEST INFRASTRUCTURE: a plain, single-threaded numpy/Python statement of what the
path computes, written from the paper (sections 2, 4.2, 4.3 and 4.4).  It exists so
the GPU library can be checked bit for bit.  Only tests, the smoke check and the
benchmark's CPU-baseline leg import it; the library never does and shares no
code with it.
"""
from .plan import (BF16, F32, KIND_BATCH, KIND_CHUNK, PATTERN_HALVING_DOUBLING, PATTERN_RING, PATTERN_SHUFFLE, SPLIT_ADAPTIVE, SPLIT_FIXED, SPLIT_NONE,
                   Config, Entry, Plan, Unit, build_plan, chunk_sizes, fit_linear, ring_segments,
                   threshold_from_model)
from .aggregate import (abs_sum_f64, allreduce, bf16_to_f32, f32_to_bf16_rne, mean_f64, new_fused,
                        pack, reduce_unit, ring_reduce, unit_views, unpack)
from .ring_sim import halving_doubling_sim, ring_allreduce_sim, shuffle_sim
from .schedule import BIN_BACKWARD, BIN_FORWARD, Schedule, Slot, group_windows, schedule_transfers
