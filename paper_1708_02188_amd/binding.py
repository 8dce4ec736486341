"""ctypes binding of libddlsim: same names as the C ABI, argument marshalling only."""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))

DDL_F32, DDL_F64, DDL_I32, DDL_F16, DDL_BF16 = 0, 1, 2, 3, 4
DDL_OK = 0
DDL_ERR_ARG, DDL_ERR_DIMS, DDL_ERR_DTYPE, DDL_ERR_ALIGN = -1, -2, -3, -4
DDL_ERR_PLAN_MISMATCH, DDL_ERR_NOMEM, DDL_ERR_HIP, DDL_ERR_UNSUPPORTED = -5, -6, -7, -8
DDL_STEP_REDUCE, DDL_STEP_GATHER = 0, 1
DDL_WALK_AUTO, DDL_WALK_OFF, DDL_WALK_ON = 0, 1, 2


def library_path():
    """Where the built library is expected (DDLSIM_LIBRARY overrides the in-tree file)."""
    return os.environ.get("DDLSIM_LIBRARY") or os.path.join(_PKG, "libddlsim.so")


def _one_hip_runtime():
    """PyTorch wheels bundle their own libamdhip64 under the same SONAME as the system's; the
    first one loaded serves the whole process.  If this library came first, torch would run on
    a runtime it was not built for (its launches then fail), so torch, when present, is
    imported before the library is opened."""
    try:
        import torch  # noqa: F401
    except ImportError:
        pass


def _load():
    _one_hip_runtime()
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_1708_02188_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(path)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    pi, psz = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_size_t)
    sim_args = [ctypes.POINTER(vp), i, vp, sz, i, vp]
    sigs = {
        "ddl_ring_plan": (vp, [pi, i, i, sz, i, pi]),
        "ddl_ring_plan_tensors": (vp, [pi, i, i, psz, psz, i, sz, i, pi]),
        "ddl_plan_num_tensors": (i, [vp]),
        "ddl_plan_owned_chunk_tensor": (i, [vp, i, i, psz, psz]),
        "ddl_plan_free": (None, [vp]),
        "ddl_plan_prepare": (i, [vp]),
        "ddl_plan_reserve_bindings": (i, [vp, i]),
        "ddl_plan_set_walk": (i, [vp, i]),
        "ddl_plan_walk_bytes": (sz, [vp]),
        "ddl_allreduce_sim": (i, sim_args),
        "ddl_allreduce_sim_noalloc": (i, sim_args),
        "ddl_reduce_scatter_sim": (i, sim_args),
        "ddl_allgather_sim": (i, sim_args),
        "ddl_assign_sim": (i, [vp, vp, sz, i, vp]),
        "ddl_allreduce_fused_sim": (i, sim_args),
        "ddl_reduce_scatter_fused_sim": (i, sim_args),
        "ddl_allgather_fused_sim": (i, sim_args),
        "ddl_plan_fused_bytes": (sz, [vp]),
        "ddl_allreduce_sim_profile": (i, sim_args + [ctypes.POINTER(ctypes.c_float)]),
        "ddl_allreduce_sim_timed": (i, sim_args + [ctypes.POINTER(ctypes.c_float),
                                                   ctypes.POINTER(ctypes.c_float)]),
        "ddl_plan_verify": (i, [vp]),
        "ddl_plan_num_steps": (i, [vp]),
        "ddl_plan_num_learners": (i, [vp]),
        "ddl_plan_bytes_moved": (sz, [vp]),
        "ddl_plan_step_bytes": (sz, [vp, i]),
        "ddl_plan_get_step": (i, [vp, i, pi, pi, pi, pi, psz, psz]),
        "ddl_plan_owned_chunk": (i, [vp, i, psz, psz]),
        "ddl_plan_model_time": (ctypes.c_double, [vp, ctypes.POINTER(ctypes.c_double),
                                                  ctypes.POINTER(ctypes.c_double)]),
        "ddl_choose_dims": (i, [i, sz, i, ctypes.POINTER(ctypes.c_double),
                                ctypes.POINTER(ctypes.c_double), pi, pi,
                                ctypes.POINTER(ctypes.c_double)]),
        "ddl_device_memory_info": (i, [pi, pi]),
        "ddl_status_string": (ctypes.c_char_p, [i]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()


class DdlError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {ddl_status_string(status)} ({status})")


class Plan:
    """Owner of a ddl_plan_t*; freed on garbage collection or by ddl_plan_free."""

    def __init__(self, handle, dims, P, count, dtype):
        self.handle, self.dims, self.P, self.count, self.dtype = handle, list(dims), P, count, dtype

    def __del__(self):
        try:
            ddl_plan_free(self)
        except Exception:  # interpreter shutdown: the module may already be torn down
            pass


def _h(plan):
    return plan.handle if isinstance(plan, Plan) else plan


def pointer_array(bufs):
    """The host array of device pointers the ddl_*_sim calls take, made once from ints or
    objects with data_ptr(); pass it instead of the list to marshal nothing per call."""
    return _ptr_array(bufs)


def _ptr_array(bufs):
    """Host array of device pointers from ints or objects with data_ptr()."""
    if bufs is None or isinstance(bufs, ctypes.Array):
        return bufs
    vals = [b.data_ptr() if hasattr(b, "data_ptr") else b for b in bufs]
    return (ctypes.c_void_p * len(vals))(*vals)


def _stream(stream):
    if stream is None:
        return None
    return getattr(stream, "cuda_stream", stream)


def ddl_status_string(status):
    return _lib.ddl_status_string(int(status)).decode()


def ddl_ring_plan(dims, P, count, dtype=DDL_F32):
    arr = (ctypes.c_int * max(len(dims), 1))(*dims) if dims is not None else None
    status = ctypes.c_int(0)
    handle = _lib.ddl_ring_plan(arr, len(dims) if dims is not None else 0, P, count, dtype,
                                ctypes.byref(status))
    if not handle:
        raise DdlError(status.value, "ddl_ring_plan")
    return Plan(handle, dims, P, count, dtype)


def ddl_ring_plan_tensors(dims, P, tensor_off, tensor_count, count, dtype=DDL_F32):
    """Plan for a buffer of `count` elements holding several independently reduced tensors."""
    arr = (ctypes.c_int * max(len(dims), 1))(*dims)
    S = len(tensor_off)
    offs = (ctypes.c_size_t * max(S, 1))(*tensor_off)
    cnts = (ctypes.c_size_t * max(S, 1))(*tensor_count)
    status = ctypes.c_int(0)
    handle = _lib.ddl_ring_plan_tensors(arr, len(dims), P, offs, cnts, S, count, dtype, ctypes.byref(status))
    if not handle:
        raise DdlError(status.value, "ddl_ring_plan_tensors")
    return Plan(handle, dims, P, count, dtype)


def ddl_plan_num_tensors(plan):
    return _lib.ddl_plan_num_tensors(_h(plan))


def ddl_plan_owned_chunk_tensor(plan, tensor, learner):
    off, n = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(_lib.ddl_plan_owned_chunk_tensor(_h(plan), tensor, learner, ctypes.byref(off), ctypes.byref(n)),
           "ddl_plan_owned_chunk_tensor")
    return off.value, n.value


def ddl_plan_free(plan):
    if isinstance(plan, Plan):
        if plan.handle:
            _lib.ddl_plan_free(plan.handle)
            plan.handle = None
    elif plan:
        _lib.ddl_plan_free(plan)


def _check(status, where):
    if status != DDL_OK:
        raise DdlError(status, where)


def ddl_plan_prepare(plan):
    _check(_lib.ddl_plan_prepare(_h(plan)), "ddl_plan_prepare")


def ddl_plan_reserve_bindings(plan, slots):
    _check(_lib.ddl_plan_reserve_bindings(_h(plan), slots), "ddl_plan_reserve_bindings")


def ddl_plan_set_walk(plan, mode):
    _check(_lib.ddl_plan_set_walk(_h(plan), mode), "ddl_plan_set_walk")


def ddl_plan_walk_bytes(plan):
    return _lib.ddl_plan_walk_bytes(_h(plan))


def ddl_allreduce_sim(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    _check(_lib.ddl_allreduce_sim(_ptr_array(bufs), P, _h(plan), count, dtype, _stream(stream)),
           "ddl_allreduce_sim")


def ddl_allreduce_sim_noalloc(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    _check(_lib.ddl_allreduce_sim_noalloc(_ptr_array(bufs), P, _h(plan), count, dtype, _stream(stream)),
           "ddl_allreduce_sim_noalloc")


def ddl_reduce_scatter_sim(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    _check(_lib.ddl_reduce_scatter_sim(_ptr_array(bufs), P, _h(plan), count, dtype,
                                       _stream(stream)), "ddl_reduce_scatter_sim")


def ddl_allgather_sim(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    _check(_lib.ddl_allgather_sim(_ptr_array(bufs), P, _h(plan), count, dtype, _stream(stream)),
           "ddl_allgather_sim")


def ddl_allreduce_fused_sim(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    _check(_lib.ddl_allreduce_fused_sim(_ptr_array(bufs), P, _h(plan), count, dtype, _stream(stream)),
           "ddl_allreduce_fused_sim")


def ddl_assign_sim(dst, src, count, dtype=DDL_F32, stream=None):
    d = dst.data_ptr() if hasattr(dst, "data_ptr") else dst
    s = src.data_ptr() if hasattr(src, "data_ptr") else src
    _check(_lib.ddl_assign_sim(d, s, count, dtype, _stream(stream)), "ddl_assign_sim")


def ddl_reduce_scatter_fused_sim(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    _check(_lib.ddl_reduce_scatter_fused_sim(_ptr_array(bufs), P, _h(plan), count, dtype, _stream(stream)),
           "ddl_reduce_scatter_fused_sim")


def ddl_allgather_fused_sim(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    _check(_lib.ddl_allgather_fused_sim(_ptr_array(bufs), P, _h(plan), count, dtype, _stream(stream)),
           "ddl_allgather_fused_sim")


def ddl_plan_fused_bytes(plan):
    return _lib.ddl_plan_fused_bytes(_h(plan))


def ddl_allreduce_sim_profile(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    """Returns the list of per-step milliseconds."""
    n = max(ddl_plan_num_steps(plan), 0)
    ms = (ctypes.c_float * max(n, 1))()
    _check(_lib.ddl_allreduce_sim_profile(_ptr_array(bufs), P, _h(plan), count, dtype,
                                          _stream(stream), ms), "ddl_allreduce_sim_profile")
    return list(ms)[:n]


def ddl_allreduce_sim_timed(bufs, P, plan, count, dtype=DDL_F32, stream=None):
    """Returns (reduce_ms, gather_ms): elapsed time of the two halves."""
    r, g = ctypes.c_float(0), ctypes.c_float(0)
    _check(_lib.ddl_allreduce_sim_timed(_ptr_array(bufs), P, _h(plan), count, dtype, _stream(stream),
                                        ctypes.byref(r), ctypes.byref(g)), "ddl_allreduce_sim_timed")
    return r.value, g.value


def ddl_plan_verify(plan):
    _check(_lib.ddl_plan_verify(_h(plan)), "ddl_plan_verify")


def ddl_plan_num_steps(plan):
    return _lib.ddl_plan_num_steps(_h(plan))


def ddl_plan_num_learners(plan):
    return _lib.ddl_plan_num_learners(_h(plan))


def ddl_plan_bytes_moved(plan):
    return _lib.ddl_plan_bytes_moved(_h(plan))


def ddl_plan_step_bytes(plan, step):
    return _lib.ddl_plan_step_bytes(_h(plan), step)


def ddl_plan_get_step(plan, step):
    """Returns (kind, dim, [(src, dst, off, n), ...])."""
    P = max(ddl_plan_num_learners(plan) * max(ddl_plan_num_tensors(plan), 1), 1)
    kind, dim = ctypes.c_int(-1), ctypes.c_int(-1)
    src, dst = (ctypes.c_int * P)(), (ctypes.c_int * P)()
    off, n = (ctypes.c_size_t * P)(), (ctypes.c_size_t * P)()
    _check(_lib.ddl_plan_get_step(_h(plan), step, ctypes.byref(kind), ctypes.byref(dim),
                                  src, dst, off, n), "ddl_plan_get_step")
    return kind.value, dim.value, list(zip(src, dst, off, n))


def ddl_plan_owned_chunk(plan, learner):
    off, n = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(_lib.ddl_plan_owned_chunk(_h(plan), learner, ctypes.byref(off), ctypes.byref(n)),
           "ddl_plan_owned_chunk")
    return off.value, n.value


def ddl_plan_model_time(plan, bw, lat):
    m = len(bw)
    return _lib.ddl_plan_model_time(_h(plan), (ctypes.c_double * m)(*bw), (ctypes.c_double * m)(*lat))


def ddl_choose_dims(P, nbytes, bw, lat, max_dim=None):
    """Returns (dims, modelled seconds)."""
    m = len(bw)
    dims = (ctypes.c_int * max(m, 1))()
    t = ctypes.c_double(0.0)
    caps = (ctypes.c_int * m)(*max_dim) if max_dim is not None else None
    _check(_lib.ddl_choose_dims(P, nbytes, m, (ctypes.c_double * max(m, 1))(*bw),
                                (ctypes.c_double * max(m, 1))(*lat), caps, dims, ctypes.byref(t)),
           "ddl_choose_dims")
    return list(dims)[:m], t.value


def ddl_device_memory_info():
    """Returns (memory clock in kHz, bus width in bits) of the current device."""
    clock, bus = ctypes.c_int(0), ctypes.c_int(0)
    _check(_lib.ddl_device_memory_info(ctypes.byref(clock), ctypes.byref(bus)), "ddl_device_memory_info")
    return clock.value, bus.value
