"""MI355X-native simulated multi-ring allreduce (PowerAI DDL's data-parallel hot path).

Thin ctypes binding over the C ABI of libddlsim (see include/ddlsim.h); every step of the
path runs in the library's HIP kernels.  There is no CPU fallback: if the shared library
has not been built, importing the binding raises.
"""
from .binding import (  # noqa: F401
    DDL_F32,
    DDL_F64,
    DDL_I32,
    DDL_OK,
    DDL_ERR_ARG,
    DDL_ERR_DIMS,
    DDL_ERR_DTYPE,
    DDL_ERR_ALIGN,
    DDL_ERR_PLAN_MISMATCH,
    DDL_ERR_NOMEM,
    DDL_ERR_HIP,
    DDL_STEP_REDUCE,
    DDL_STEP_GATHER,
    DdlError,
    Plan,
    ddl_ring_plan,
    ddl_plan_free,
    ddl_plan_prepare,
    ddl_allreduce_sim,
    ddl_reduce_scatter_sim,
    ddl_allgather_sim,
    ddl_allreduce_sim_profile,
    ddl_plan_num_steps,
    ddl_plan_num_learners,
    ddl_plan_bytes_moved,
    ddl_plan_step_bytes,
    ddl_plan_get_step,
    ddl_plan_owned_chunk,
    ddl_plan_model_time,
    ddl_status_string,
    library_path,
)
