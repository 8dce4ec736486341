"""CPU oracle for the multi-ring allreduce (test infrastructure, not product code).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It shares no code with the HIP library and never imports it.
"""
from .ddl_oracle import (  # noqa: F401
    coords,
    rank_of,
    neighbour,
    granule,
    split,
    level_segment,
    fine_chunks,
    schedule,
    schedule_bytes,
    allreduce_steps,
    reduce_scatter_steps,
    allgather_steps,
    allreduce_fold,
    allreduce_fold_range,
    sum_fp64,
    schedule_tensors,
    allreduce_tensors,
    bf16_add,
    bf16_to_f32,
    f32_to_bf16,
    ring_time_model,
    multiring_time_model,
    choose_dims_bruteforce,
)
