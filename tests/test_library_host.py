"""Host-side tests of the C-ABI libraries: no GPU needed, no kernel is launched."""
import ctypes
import os
import re
from math import prod

import numpy as np
import pytest

import oracle.ddl_oracle as O
import paper_1708_02188_amd as D
from paper_1708_02188_amd import inputs as I
from conftest import ROOT, read_golden_kv

HEADERS = {"ddlsim.h": D.library_path(), "ddlgen.h": I.library_path()}


def declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"\b(ddl\w*)\s*\(", text)


@pytest.mark.parametrize("header", sorted(HEADERS))
def test_library_exports_every_declared_symbol(header):
    names = declared_functions(header)
    assert len(names) >= 2
    lib = ctypes.CDLL(HEADERS[header])
    for name in names:
        assert hasattr(lib, name), f"{name} declared in {header} but not exported"


def test_binding_has_every_entry_point():
    for name in declared_functions("ddlsim.h"):
        assert hasattr(D, name), name


# ---------------------------------------------------------------------------------------
# planner == oracle's independently written schedule
# ---------------------------------------------------------------------------------------
PLAN_CASES = [
    ([1], 10), ([2], 0), ([4], 1 << 20), ([4], 37), ([5], 3), ([2, 3], 1001), ([3, 1, 2], 64),
    ([4, 4], 25557032), ([4, 16], 25557032), ([4, 8, 8], 25557032), ([4, 8, 8], 87252369),
    ([2, 2, 2, 2], 5), ([16], 1000), ([7, 3], 12345), ([4, 8, 8], 100), ([1, 1], 9),
]


@pytest.mark.parametrize("dims,count", PLAN_CASES)
@pytest.mark.parametrize("dtype,itemsize", [(D.DDL_F32, 4), (D.DDL_F64, 8), (D.DDL_I32, 4),
                                            (D.DDL_F16, 2), (D.DDL_BF16, 2)])
def test_plan_tables_equal_oracle_schedule(dims, count, dtype, itemsize):
    P = prod(dims)
    plan = D.ddl_ring_plan(dims, P, count, dtype)
    steps = O.schedule(dims, count, 16 // itemsize)
    assert D.ddl_plan_num_steps(plan) == len(steps) == 2 * sum(d - 1 for d in dims)
    assert D.ddl_plan_num_learners(plan) == P
    total = 0
    for s, (kind, t, ops) in enumerate(steps):
        k, dim, lib_ops = D.ddl_plan_get_step(plan, s)
        assert k == (D.DDL_STEP_REDUCE if kind == "RS" else D.DDL_STEP_GATHER)
        assert dim == t
        assert lib_ops == [(src, dst, a, b - a) for src, dst, a, b in ops]
        step_bytes = sum(b - a for _, _, a, b in ops) * (3 if kind == "RS" else 2) * itemsize
        assert D.ddl_plan_step_bytes(plan, s) == step_bytes
        total += step_bytes
    assert D.ddl_plan_bytes_moved(plan) == total == O.schedule_bytes(dims, count, itemsize)
    for k, a, b in O.fine_chunks(dims, count, 16 // itemsize):
        assert D.ddl_plan_owned_chunk(plan, O.rank_of(k, dims)) == (a, b - a)
    D.ddl_plan_free(plan)
    D.ddl_plan_free(plan)  # second free of the wrapper is a no-op


@pytest.mark.parametrize("dims,count", PLAN_CASES)
def test_plan_self_check_accepts_every_plan(dims, count):
    P = prod(dims)
    D.ddl_plan_verify(D.ddl_ring_plan(dims, P, count))
    D.ddl_plan_verify(D.ddl_ring_plan(dims, P, count, D.DDL_F16))
    if count >= 64:
        D.ddl_plan_verify(D.ddl_ring_plan_tensors(dims, P, [0, 16, 48], [9, 32, count - 48], count))
    with pytest.raises(D.DdlError):
        D.ddl_plan_verify(None)


def test_bytes_closed_form_at_the_benchmark_sizes():
    # 5 * sizeof * count * (P - 1) needs count divisible by G*P; otherwise within a granule per op
    for cfg in I.CONFIGS:
        plan = D.ddl_ring_plan(cfg["dims"], cfg["P"], cfg["count"])
        closed = 20 * cfg["count"] * (cfg["P"] - 1)
        got = D.ddl_plan_bytes_moved(plan)
        if cfg["count"] % (4 * cfg["P"]) == 0:
            assert got == closed
        assert abs(got - closed) <= 20 * 4 * cfg["P"] * D.ddl_plan_num_steps(plan)


def test_model_time_matches_oracle_and_paper_figures():
    fig = read_golden_kv("paper_figures.txt")
    S = 87252369 * 4
    plan = D.ddl_ring_plan([4, 8, 8], 256, 87252369)
    bw = [fig["bw_dim1"], fig["bw_dim2"], fig["bw_dim3"]]
    for lat in ([0.0] * 3, [1e-5, 2e-5, 5e-5]):
        assert D.ddl_plan_model_time(plan, bw, lat) == pytest.approx(
            O.multiring_time_model(S, [4, 8, 8], bw, lat), rel=1e-12)
    # Sec. 4.3: reduction and distribution of ~350 MB in under 100 ms
    assert abs(S - fig["resnet101_22k_bytes"]) / fig["resnet101_22k_bytes"] < 0.01
    assert D.ddl_plan_model_time(plan, bw, [0.0] * 3) < fig["allreduce_time_max"]
    assert D.ddl_plan_model_time(plan, [0.0, 1.0, 1.0], [0.0] * 3) < 0


# ---------------------------------------------------------------------------------------
# error paths (all decided on the host before anything touches a device)
# ---------------------------------------------------------------------------------------
def status_of(fn, *args, **kw):
    with pytest.raises(D.DdlError) as e:
        fn(*args, **kw)
    return e.value.status


def test_plan_argument_errors():
    assert status_of(D.ddl_ring_plan, [2, 3], 5, 10) == D.DDL_ERR_DIMS
    assert status_of(D.ddl_ring_plan, [0, 4], 4, 10) == D.DDL_ERR_DIMS
    assert status_of(D.ddl_ring_plan, [-2, -2], 4, 10) == D.DDL_ERR_DIMS
    assert status_of(D.ddl_ring_plan, [], 1, 10) == D.DDL_ERR_DIMS
    assert status_of(D.ddl_ring_plan, [2] * 17, 2 ** 17, 10) == D.DDL_ERR_ARG  # P too large
    assert status_of(D.ddl_ring_plan, [1] * 17, 1, 10) == D.DDL_ERR_DIMS        # too many dims
    assert status_of(D.ddl_ring_plan, [4], 0, 10) == D.DDL_ERR_ARG
    assert status_of(D.ddl_ring_plan, [4], 4, 10, 99) == D.DDL_ERR_DTYPE
    assert status_of(D.ddl_ring_plan, None, 4, 10) == D.DDL_ERR_ARG
    assert status_of(D.ddl_ring_plan, [65536], 65536, 10) == D.DDL_ERR_ARG
    # a flat ring of 65535 learners would need 8.6e9 table entries: refused, not attempted
    assert status_of(D.ddl_ring_plan, [65535], 65535, 10) == D.DDL_ERR_NOMEM
    big = D.ddl_ring_plan([15, 17, 257], 65535, 10)   # the largest learner count, as a box
    assert D.ddl_plan_num_steps(big) == 2 * (14 + 16 + 256)
    D.ddl_plan_free(big)
    for code in range(-8, 1):
        assert D.ddl_status_string(code) and D.ddl_status_string(code) != "unknown status"
    assert D.ddl_status_string(-99) == "unknown status"
    assert D.ddl_plan_num_steps(None) == -1 and D.ddl_plan_bytes_moved(None) == 0
    assert status_of(D.ddl_plan_get_step, D.ddl_ring_plan([4], 4, 8), 6) == D.DDL_ERR_ARG
    assert status_of(D.ddl_plan_owned_chunk, D.ddl_ring_plan([4], 4, 8), 4) == D.DDL_ERR_ARG


@pytest.mark.parametrize("entry", [D.ddl_allreduce_sim, D.ddl_reduce_scatter_sim,
                                   D.ddl_allgather_sim, D.ddl_allreduce_sim_profile,
                                   D.ddl_allreduce_sim_timed, D.ddl_allreduce_fused_sim,
                                   D.ddl_reduce_scatter_fused_sim, D.ddl_allgather_fused_sim])
def test_call_argument_errors(entry):
    count = 64
    plan = D.ddl_ring_plan([2, 2], 4, count)
    good = [0x100000 + j * 0x1000 for j in range(4)]  # never dereferenced: every call below fails
    assert status_of(entry, good, 4, None, count) == D.DDL_ERR_ARG
    assert status_of(entry, good[:3], 3, plan, count) == D.DDL_ERR_PLAN_MISMATCH
    assert status_of(entry, good, 4, plan, count + 1) == D.DDL_ERR_PLAN_MISMATCH
    assert status_of(entry, good, 4, plan, count, D.DDL_F64) == D.DDL_ERR_PLAN_MISMATCH
    assert status_of(entry, good, 4, plan, count, 42) == D.DDL_ERR_DTYPE
    assert status_of(entry, good, 0, plan, count) == D.DDL_ERR_ARG
    assert status_of(entry, [good[0], None, good[2], good[3]], 4, plan, count) == D.DDL_ERR_ARG
    assert status_of(entry, [good[0], good[1] + 8, good[2], good[3]], 4, plan, count) == D.DDL_ERR_ALIGN
    assert status_of(entry, [good[0], good[1], good[1], good[3]], 4, plan, count) == D.DDL_ERR_ARG
    # overlapping, not identical: buffers of 256 bytes only 128 bytes apart
    assert status_of(entry, [good[0], good[0] + 128, good[2], good[3]], 4, plan, count) == D.DDL_ERR_ARG


def test_assign_argument_errors():
    a, b = 0x100000, 0x200000
    assert status_of(D.ddl_assign_sim, a, b, 100, 77) == D.DDL_ERR_DTYPE
    assert status_of(D.ddl_assign_sim, None, b, 100) == D.DDL_ERR_ARG
    assert status_of(D.ddl_assign_sim, a + 4, b, 100) == D.DDL_ERR_ALIGN
    assert status_of(D.ddl_assign_sim, a, a + 16, 100) == D.DDL_ERR_ARG     # overlapping
    assert status_of(D.ddl_assign_sim, a, a, 100) == D.DDL_ERR_ARG
    D.ddl_assign_sim(None, None, 0)                                          # nothing to copy


def test_fused_limits_and_bytes():
    plan = D.ddl_ring_plan([4, 8, 8], 256, 25557032)
    assert D.ddl_plan_fused_bytes(plan) == 4 * 25557032 * (2 * 256 + 2)
    # two passes from 16 learners on (one more write and read of the result), one pass below
    assert D.ddl_plan_fused_bytes(D.ddl_ring_plan([4, 4], 16, 1000)) == 4 * 1000 * (2 * 16 + 2)
    assert D.ddl_plan_fused_bytes(D.ddl_ring_plan([4, 2], 8, 1000)) == 4 * 1000 * 16
    assert D.ddl_plan_fused_bytes(None) == 0
    # rejected on the host, before any device work: too many learners / too many levels
    big = D.ddl_ring_plan([2048], 2048, 64)
    ptrs = [0x100000 + 0x1000 * j for j in range(2048)]
    assert status_of(D.ddl_allreduce_fused_sim, ptrs, 2048, big, 64) == D.DDL_ERR_UNSUPPORTED
    deep = D.ddl_ring_plan([2] * 5, 32, 64)
    assert status_of(D.ddl_allreduce_fused_sim, ptrs[:32], 32, deep, 64) == D.DDL_ERR_UNSUPPORTED
    D.ddl_allreduce_fused_sim([0x100000], 1, D.ddl_ring_plan([1, 1], 1, 100), 100)  # one learner: nothing to do


def test_trivial_calls_need_no_device():
    # one learner, or nothing to move: valid, zero steps, nothing is launched
    plan = D.ddl_ring_plan([1, 1], 1, 100)
    D.ddl_allreduce_sim([0x100000], 1, plan, 100)
    plan0 = D.ddl_ring_plan([2, 2], 4, 0)
    D.ddl_allreduce_sim([0x100000 + 16 * j for j in range(4)], 4, plan0, 0)
    assert D.ddl_allreduce_sim_profile([0x100000 + 16 * j for j in range(4)], 4, plan0, 0) == [0.0] * 4
    assert D.ddl_allreduce_sim_timed([0x100000 + 16 * j for j in range(4)], 4, plan0, 0) == (0.0, 0.0)


# ---------------------------------------------------------------------------------------
# input generator, host side
# ---------------------------------------------------------------------------------------
MASK = (1 << 64) - 1
PHI = 0x9E3779B97F4A7C15


def _mix(x):
    z = (x + PHI) & MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def _reference_value(seed, learner, e, dist):
    """The documented value function of include/ddlgen.h in Python integers."""
    key = _mix((seed + PHI * (learner + 1)) & MASK)
    h0 = _mix((key + 2 * e) & MASK)
    if dist == "int8":
        return np.float32((h0 >> 32) % 17 - 8)
    if dist == "uniform":
        return np.float32((h0 >> 40) - (1 << 23)) * np.float32(2.0 ** -23)
    h1 = _mix((key + 2 * e + 1) & MASK)
    q = sum((h >> (16 * i)) & 0xFFFF for h in (h0, h1) for i in range(4)) - 262140
    return np.float32(q) * np.float32(0.01 / np.sqrt(8.0 * (4294967296.0 - 1.0) / 12.0))


@pytest.mark.parametrize("dist", ["int8", "uniform", "normal"])
def test_generator_matches_documented_function(dist):
    for seed, learner, first in [(0, 0, 0), (I.BASE_SEED + 2, 15, 25557000), (2 ** 63 + 5, 255, 2 ** 33)]:
        got = I.fill_host(40, seed, learner, dist, first)
        want = np.array([_reference_value(seed, learner, first + i, dist) for i in range(40)],
                        dtype=np.float32)
        assert got.tobytes() == want.tobytes()


def test_generator_properties():
    n = 400000
    a = I.fill_host(n, 7, 3, "int8")
    assert np.array_equal(a, np.round(a)) and a.min() == -8 and a.max() == 8
    assert len(np.unique(a)) == 17
    u = I.fill_host(n, 7, 3, "uniform")
    assert -1 <= u.min() and u.max() < 1 and abs(u.mean()) < 0.01 and abs(u.std() - 3 ** -0.5) < 0.01
    g = I.fill_host(n, 7, 3, "normal")
    assert abs(g.mean()) < 1e-4 and abs(g.std() - 1e-2) < 1e-4
    # slices agree with the whole, learners and seeds differ
    assert np.array_equal(I.fill_host(100, 7, 3, "uniform", first=1234), u[1234:1334])
    assert not np.array_equal(I.fill_host(100, 7, 4, "uniform"), u[:100])
    assert not np.array_equal(I.fill_host(100, 8, 3, "uniform"), u[:100])
    assert I.fill_host(0, 1, 1, "uniform").size == 0
    with pytest.raises(ValueError):
        I.fill_host(4, 1, 1, 17)


def test_workload_shapes_match_the_paper_sizes():
    fig = read_golden_kv("paper_figures.txt")
    s50, s101 = I.resnet50_shapes(), I.resnet101_22k_shapes()
    assert len(s50) == 161 and I.numel(s50) == I.RESNET50_COUNT
    assert len(s101) == 314 and I.numel(s101) == I.RESNET101_22K_COUNT
    # Sec. 5.1: about 100 MB of gradients; Sec. 4.3: nearly 90 M entries, about 350 MB
    assert abs(4 * I.RESNET50_COUNT - fig["resnet50_bytes"]) / fig["resnet50_bytes"] < 0.05
    assert abs(I.RESNET101_22K_COUNT - fig["resnet101_22k_entries"]) / fig["resnet101_22k_entries"] < 0.05
    assert abs(4 * I.RESNET101_22K_COUNT - fig["resnet101_22k_bytes"]) / fig["resnet101_22k_bytes"] < 0.01
    for cfg in I.CONFIGS:
        assert prod(cfg["dims"]) == cfg["P"]


# ---------------------------------------------------------------------------------------
# dimension chooser
# ---------------------------------------------------------------------------------------
def test_choose_dims_matches_bruteforce_oracle():
    fig = read_golden_kv("paper_figures.txt")
    bw = [fig["bw_dim1"], fig["bw_dim2"], fig["bw_dim3"]]
    cases = [
        (256, 349e6, bw, [0.0] * 3, None),
        (256, 349e6, bw, [5e-5] * 3, None),
        (256, 349e6, bw, [5e-5] * 3, [4, 16, 0]),
        (256, 349e6, bw, [0.0] * 3, [4, 16, 4]),
        (64, 1e8, bw, [1e-5, 2e-5, 1e-4], [4, 0, 0]),
        (60, 1e6, [1e10, 5e9], [1e-6, 1e-3], None),
        (97, 1e6, [1e10, 5e9, 1e9], [1e-6] * 3, None),
        (1, 1e6, [1e10], [0.0], None),
        (256, 1.0, [1e10] * 8, [1.0] * 8, None),
    ]
    for P, S, B, L, caps in cases:
        dims, t = D.ddl_choose_dims(P, int(S), B, L, caps)
        best, boxes = O.choose_dims_bruteforce(P, float(int(S)), B, L, caps)
        assert prod(dims) == P and dims in boxes, (P, dims, boxes)
        assert t == pytest.approx(best, rel=1e-12)
        plan = D.ddl_ring_plan(dims, P, int(S) // 4)
        assert D.ddl_plan_model_time(plan, B, L) == pytest.approx(t, rel=1e-6)
    # exact ties go to the lexicographically smallest box
    assert D.ddl_choose_dims(64, 10 ** 6, [1e10] * 3, [0.0] * 3)[0] == [1, 1, 64]
    assert status_of(D.ddl_choose_dims, 256, 100, bw, [0.0] * 3, [4, 4, 4]) == D.DDL_ERR_DIMS
    assert status_of(D.ddl_choose_dims, 0, 100, bw, [0.0] * 3) == D.DDL_ERR_ARG
    assert status_of(D.ddl_choose_dims, 4, 100, [0.0], [0.0]) == D.DDL_ERR_ARG
    assert status_of(D.ddl_choose_dims, 4, 100, [1.0], [-1.0]) == D.DDL_ERR_ARG


# ---------------------------------------------------------------------------------------
# several tensors per buffer
# ---------------------------------------------------------------------------------------
def test_tensor_plan_tables_equal_oracle_schedule():
    cases = [
        ([4], [(0, 64), (64, 4), (68, 0), (72, 1000), (1072, 8), (1100, 37)], 1140, D.DDL_F32, 4),
        ([2, 3], [(0, 5), (8, 3), (16, 100000)], 100016, D.DDL_F32, 4),
        ([4, 16], list(zip(*I.tensor_segments(I.resnet50_shapes()))), I.RESNET50_COUNT, D.DDL_F32, 4),
        ([4, 2], [(0, 24), (24, 808), (832, 9)], 841, D.DDL_F16, 2),
    ]
    for dims, segments, count, dtype, itemsize in cases:
        P = prod(dims)
        G = 16 // itemsize
        plan = D.ddl_ring_plan_tensors(dims, P, [o for o, _ in segments], [n for _, n in segments], count, dtype)
        S = len(segments)
        assert D.ddl_plan_num_tensors(plan) == S and D.ddl_plan_num_learners(plan) == P
        steps = O.schedule_tensors(dims, segments, G)
        assert D.ddl_plan_num_steps(plan) == len(steps)
        total = 0
        for i, (kind, t, ops) in enumerate(steps):
            k, dim, lib_ops = D.ddl_plan_get_step(plan, i)
            assert (k, dim) == (D.DDL_STEP_REDUCE if kind == "RS" else D.DDL_STEP_GATHER, t)
            assert lib_ops == [(src, dst, a, b - a) for src, dst, a, b in ops]
            total += sum(b - a for _, _, a, b in ops) * (3 if kind == "RS" else 2) * itemsize
        assert D.ddl_plan_bytes_moved(plan) == total
        for s_i, (off, n) in enumerate(segments):
            for k, a, b in O.fine_chunks(dims, n, G):
                assert D.ddl_plan_owned_chunk_tensor(plan, s_i, O.rank_of(k, dims)) == (off + a, b - a)


def test_tensor_plan_too_large_for_its_work_lists_is_refused():
    # 2^38 fp32 elements over 64 learners would need 8e9 work items: refused before anything is built
    count = 1 << 38
    assert status_of(D.ddl_ring_plan_tensors, [4, 16], 64, [0, count // 2], [count // 2, count // 2], count) \
        == D.DDL_ERR_NOMEM
    D.ddl_plan_free(D.ddl_ring_plan([4, 16], 64, count))   # one tensor needs no lists


def test_tensor_plan_argument_errors():
    ok = dict(dims=[2, 2], P=4, count=100)
    assert status_of(D.ddl_ring_plan_tensors, [2, 2], 4, [0, 10], [10, 10], 100) == D.DDL_ERR_ALIGN   # 10 % 4 != 0
    assert status_of(D.ddl_ring_plan_tensors, [2, 2], 4, [0, 8], [10, 10], 100) == D.DDL_ERR_ARG     # overlap
    assert status_of(D.ddl_ring_plan_tensors, [2, 2], 4, [16, 0], [4, 4], 100) == D.DDL_ERR_ARG      # not ascending
    assert status_of(D.ddl_ring_plan_tensors, [2, 2], 4, [0, 96], [4, 8], 100) == D.DDL_ERR_ARG      # past the end
    assert status_of(D.ddl_ring_plan_tensors, [2, 2], 4, [], [], 100) == D.DDL_ERR_ARG
    assert status_of(D.ddl_ring_plan_tensors, [2, 3], 4, [0], [4], 100) == D.DDL_ERR_DIMS
    plan = D.ddl_ring_plan_tensors([2, 2], 4, [0, 12], [12, 88], 100)
    assert status_of(D.ddl_plan_owned_chunk_tensor, plan, 2, 0) == D.DDL_ERR_ARG
    ptrs = [0x100000 + 0x1000 * j for j in range(4)]
    assert status_of(D.ddl_allreduce_fused_sim, ptrs, 4, plan, 100) == D.DDL_ERR_UNSUPPORTED


# ---------------------------------------------------------------------------------------
# property test: planner tables == oracle schedule on random boxes, lengths and tensor lists
# ---------------------------------------------------------------------------------------
from hypothesis import given, settings, strategies as st  # noqa: E402


@st.composite
def plan_cases(draw):
    dims = draw(st.lists(st.integers(1, 6), min_size=1, max_size=4))
    itemsize = draw(st.sampled_from([2, 4, 8]))
    G = 16 // itemsize
    n_tensors = draw(st.integers(1, 5))
    segments, pos = [], 0
    for _ in range(n_tensors):
        pos += draw(st.integers(0, 3)) * G
        n = draw(st.one_of(st.integers(0, 40), st.integers(0, 5000)))
        segments.append((pos, n))
        pos = -(-(pos + n) // G) * G
    count = pos + draw(st.integers(0, 9))
    return dims, itemsize, segments, count


@settings(max_examples=150, deadline=None)
@given(plan_cases())
def test_planner_matches_oracle_on_random_cases(case):
    dims, itemsize, segments, count = case
    P = prod(dims)
    dtype = {2: D.DDL_F16, 4: D.DDL_F32, 8: D.DDL_F64}[itemsize]
    G = 16 // itemsize
    if len(segments) == 1 and segments[0][0] == 0:
        count = segments[0][1]
        plan = D.ddl_ring_plan(dims, P, count, dtype)
    else:
        plan = D.ddl_ring_plan_tensors(dims, P, [o for o, _ in segments], [n for _, n in segments], count, dtype)
    steps = O.schedule_tensors(dims, segments, G)
    assert D.ddl_plan_num_steps(plan) == len(steps)
    total = 0
    for i, (kind, t, ops) in enumerate(steps):
        k, dim, lib_ops = D.ddl_plan_get_step(plan, i)
        assert (k, dim) == (D.DDL_STEP_REDUCE if kind == "RS" else D.DDL_STEP_GATHER, t)
        assert lib_ops == [(src, dst, a, b - a) for src, dst, a, b in ops]
        total += sum(b - a for _, _, a, b in ops) * (3 if kind == "RS" else 2) * itemsize
    assert D.ddl_plan_bytes_moved(plan) == total
    # within a phase no learner's written range meets a range it is read from
    for _, _, ops in steps:
        writes = {}
        for src, dst, a, b in ops:
            if b > a:
                writes.setdefault(dst, []).append((a, b))
        for src, dst, a, b in ops:
            for wa, wb in writes.get(src, []):
                assert b <= wa or wb <= a or a == b
