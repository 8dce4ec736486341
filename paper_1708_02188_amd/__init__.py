"""MI355X-native simulated multi-ring allreduce (PowerAI DDL's data-parallel hot path).

Thin ctypes binding over the C ABI of libddlsim (see include/ddlsim.h); every step of the
path runs in the library's HIP kernels.  There is no CPU fallback: the first use of any
entry point loads the shared library and raises ImportError if it has not been built
(`python -m paper_1708_02188_amd.build`).  The load is deferred to first use so that the
build module itself can be run from a tree whose library is missing or stale.
"""
import importlib

_BINDING_NAMES = (
    "DDL_F32", "DDL_F64", "DDL_I32", "DDL_F16", "DDL_BF16",
    "DDL_OK", "DDL_ERR_ARG", "DDL_ERR_DIMS", "DDL_ERR_DTYPE", "DDL_ERR_ALIGN",
    "DDL_ERR_PLAN_MISMATCH", "DDL_ERR_NOMEM", "DDL_ERR_HIP", "DDL_ERR_UNSUPPORTED",
    "DDL_STEP_REDUCE", "DDL_STEP_GATHER", "DDL_WALK_AUTO", "DDL_WALK_OFF", "DDL_WALK_ON",
    "DdlError", "Plan",
    "ddl_ring_plan", "ddl_ring_plan_tensors", "ddl_plan_free", "ddl_plan_prepare", "ddl_plan_reserve_bindings", "ddl_plan_set_walk", "ddl_plan_walk_bytes",
    "ddl_plan_num_tensors", "ddl_plan_owned_chunk_tensor",
    "ddl_assign_sim", "ddl_allreduce_sim", "ddl_allreduce_sim_noalloc", "ddl_reduce_scatter_sim", "ddl_allgather_sim",
    "ddl_allreduce_sim_profile", "ddl_allreduce_sim_timed", "ddl_allreduce_fused_sim", "ddl_reduce_scatter_fused_sim", "ddl_allgather_fused_sim",
    "ddl_plan_fused_bytes",
    "ddl_plan_verify", "ddl_plan_num_steps", "ddl_plan_num_learners", "ddl_plan_bytes_moved", "ddl_plan_step_bytes",
    "ddl_plan_get_step", "ddl_plan_owned_chunk", "ddl_plan_model_time", "ddl_choose_dims", "ddl_device_memory_info", "ddl_status_string",
    "library_path", "pointer_array",
)
__all__ = list(_BINDING_NAMES)


def __getattr__(name):
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
