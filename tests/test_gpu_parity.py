"""Parity of the HIP path against the CPU oracle, through the C ABI, on a real MI355X.

Bar: bit-exact against the same-order oracle for every dtype; for fp32 additionally
within 1e-5 (relative to sum_j |V_j|, and globally to max |R|) of the fp64 sum.
torch is used for device memory, copies and equality checks only.
"""
import sys
from math import prod

import numpy as np
import pytest
import torch

import oracle.ddl_oracle as O
import paper_1708_02188_amd as D
from paper_1708_02188_amd import inputs as I

pytestmark = pytest.mark.gpu

NP_OF = {D.DDL_F32: np.float32, D.DDL_F64: np.float64, D.DDL_I32: np.int32, D.DDL_F16: np.float16,
         D.DDL_BF16: np.uint16}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a device; run with -m 'not gpu' on a CPU box")
    return torch.device("cuda:0")


def upload(V, dev):
    # bfloat16 bit patterns (numpy uint16) travel as int16: torch is only the carrier
    return [torch.from_numpy(np.ascontiguousarray(v.view(np.int16) if v.dtype == np.uint16 else v)).to(dev)
            for v in V]


def download(bufs, as_dtype=None):
    torch.cuda.synchronize()
    out = [b.cpu().numpy() for b in bufs]
    return [o.view(as_dtype) for o in out] if as_dtype is not None else out


def wide_inputs(rng, P, count, dtype):
    if dtype == D.DDL_I32:
        return [rng.integers(-2 ** 31, 2 ** 31, size=count, dtype=np.int64).astype(np.int32) for _ in range(P)]
    wide = [(rng.uniform(-1, 1, count) * 10.0 ** rng.uniform(-3, 3, count)) for _ in range(P)]
    if dtype == D.DDL_BF16:
        return [O.f32_to_bf16(w.astype(np.float32)) for w in wide]
    return [w.astype(NP_OF[dtype]) for w in wide]


def assert_bitwise(got, want, what):
    assert got.dtype == want.dtype and got.shape == want.shape, what
    if got.tobytes() != want.tobytes():
        bits = {2: np.uint16, 4: np.uint32, 8: np.uint64}[got.dtype.itemsize]
        diff = np.flatnonzero(got.view(bits) != want.view(bits))
        raise AssertionError(f"{what}: {len(diff)} elements differ, first at {diff[:5]} "
                             f"got {got[diff[:5]]} want {want[diff[:5]]}")


def test_library_before_torch_in_a_fresh_process():
    """Import order must not matter: the binding makes sure one HIP runtime serves both."""
    import subprocess
    code = (
        "import paper_1708_02188_amd.binding as B, paper_1708_02188_amd.inputs as I\n"
        "import torch\n"
        "P, n = 4, 5000\n"
        "bufs = [torch.empty(n, dtype=torch.float32, device='cuda') for _ in range(P)]\n"
        "for j, b in enumerate(bufs): I.fill_device(b, 7, j, 'int8')\n"
        "plan = B.ddl_ring_plan([2, 2], P, n)\n"
        "B.ddl_allreduce_sim(bufs, P, plan, n)\n"
        "torch.cuda.synchronize()\n"
        "want = sum(I.fill_host(n, 7, j, 'int8') for j in range(P))\n"
        "assert all((b.cpu().numpy() == want).all() for b in bufs)\n"
        "print('order ok')\n")
    from conftest import ROOT
    run = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=240)
    assert run.returncode == 0 and "order ok" in run.stdout, run.stderr[-2000:]


# ---------------------------------------------------------------------------------------
# the generator: device fill == host fill
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("dist", ["int8", "uniform", "normal"])
def test_generator_device_equals_host(dev, dist):
    for n, seed, learner, first in [(1, 1, 0, 0), (100003, I.BASE_SEED, 7, 12345), (1 << 20, 99, 255, 2 ** 33 + 1)]:
        say(f"generator {dist} n={n} seed={seed} learner={learner} first={first}")
        t = torch.empty(n, dtype=torch.float32, device=dev)
        I.fill_device(t, seed, learner, dist, first)
        torch.cuda.synchronize()
        assert_bitwise(t.cpu().numpy(), I.fill_host(n, seed, learner, dist, first), dist)


# ---------------------------------------------------------------------------------------
# small and medium sizes: every learner, every element, against the step simulator
# ---------------------------------------------------------------------------------------
# one tile of the kernels is 4096 fp32 elements; counts span none, one, several tiles and ragged ends
SMALL_CASES = [
    ([1], 1000), ([2], 1), ([2], 4099), ([3], 100003), ([4], 16), ([4], 37), ([4], 65536 + 5),
    ([5], 3), ([2, 3], 50001), ([4, 4], 8), ([4, 4], 300007), ([3, 1, 2], 70001), ([4, 2, 2], 262144 + 13),
    ([2, 2, 2, 2], 99999), ([16], 150001), ([4, 16], 200003), ([4, 8, 8], 1000), ([4, 8, 8], 300001),
    ([7, 3], 123457), ([2], 0),
]


@pytest.mark.parametrize("dims,count", SMALL_CASES)
def test_allreduce_matches_step_simulator_fp32(dev, dims, count):
    P = prod(dims)
    say(f"allreduce f32 dims={dims} count={count}")
    rng = np.random.default_rng(1000 + count + P)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    got = download(bufs)
    want = O.allreduce_steps(V, dims)
    for j in range(P):
        assert_bitwise(got[j], want[j], f"dims={dims} count={count} learner={j}")
    # value check: fp64 sum within the stated tolerance
    if count:
        ref = O.sum_fp64(V)
        absum = sum(np.abs(v.astype(np.float64)) for v in V)
        assert np.all(np.abs(got[0].astype(np.float64) - ref) <= 1e-5 * absum)


@pytest.mark.parametrize("dims,count", [([4], 1 << 16), ([2, 3], 4097), ([4, 8, 8], 70000), ([3, 5], 12)])
def test_integer_valued_inputs_give_the_exact_sum(dev, dims, count):
    P = prod(dims)
    say(f"allreduce integer-valued dims={dims} count={count}")
    rng = np.random.default_rng(5)
    V = [rng.integers(-8, 9, size=count).astype(np.float32) for _ in range(P)]
    want = sum(v.astype(np.int64) for v in V)
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_allreduce_sim(bufs, P, plan, count)
    for j, g in enumerate(download(bufs)):
        assert np.array_equal(g.astype(np.int64), want), j


@pytest.mark.parametrize("dtype", [D.DDL_F64, D.DDL_I32, D.DDL_F16, D.DDL_BF16])
@pytest.mark.parametrize("dims,count", [([4], 10001), ([2, 3], 65537), ([4, 4], 131072 + 3), ([3], 1),
                                        ([4, 2, 2], 7), ([2, 2], 1 << 20)])
def test_other_dtypes_match_step_simulator(dev, dtype, dims, count):
    P = prod(dims)
    say(f"allreduce dtype={dtype} dims={dims} count={count}")
    rng = np.random.default_rng(77 + count)
    V = wide_inputs(rng, P, count, dtype)
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan(dims, P, count, dtype)
    D.ddl_allreduce_sim(bufs, P, plan, count, dtype)
    got = download(bufs, NP_OF[dtype])
    with np.errstate(over="ignore"):
        want = O.allreduce_steps(V, dims, add=O.bf16_add if dtype == D.DDL_BF16 else None)
    for j in range(P):
        assert_bitwise(got[j], want[j], f"dtype={dtype} dims={dims} learner={j}")


@pytest.mark.parametrize("name", ["ring4_cancellation.txt", "box2x2_dimension_order.txt"])
def test_hand_worked_examples_on_device(dev, name):
    from conftest import read_golden_ring_example
    ex = read_golden_ring_example(name)
    n = len(ex["expected"])
    V = [np.full(n, v, dtype=np.float32) for v in ex["inputs"]]
    want = np.array(ex["expected"], dtype=np.float32)
    plan = D.ddl_ring_plan(ex["dims"], 4, n)
    for entry in (D.ddl_allreduce_sim, D.ddl_allreduce_fused_sim):
        bufs = upload(V, dev)
        entry(bufs, 4, plan, n)
        for g in download(bufs):
            assert np.array_equal(g, want), (name, entry.__name__, g)


# ---------------------------------------------------------------------------------------
# the two halves on their own, streams, repeated calls, views, many learners
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("dims,count", [([4], 20003), ([2, 3], 9001), ([4, 2, 2], 100001)])
def test_reduce_scatter_and_allgather_alone(dev, dims, count):
    P = prod(dims)
    say(f"reduce-scatter / all-gather dims={dims} count={count}")
    rng = np.random.default_rng(31)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    plan = D.ddl_ring_plan(dims, P, count)
    bufs = upload(V, dev)
    D.ddl_reduce_scatter_sim(bufs, P, plan, count)
    got = download(bufs)
    want = O.reduce_scatter_steps(V, dims)
    for j in range(P):
        assert_bitwise(got[j], want[j], f"reduce-scatter learner={j}")
        off, n = D.ddl_plan_owned_chunk(plan, j)
        assert_bitwise(got[j][off:off + n], O.allreduce_fold(V, dims)[off:off + n], f"owned chunk {j}")
    D.ddl_allgather_sim(bufs, P, plan, count)
    got = download(bufs)
    want = O.allgather_steps(want, dims)
    for j in range(P):
        assert_bitwise(got[j], want[j], f"all-gather learner={j}")


def test_side_stream_profile_entry_and_repeat(dev):
    dims, count = [4, 4], 500009
    P = 16
    rng = np.random.default_rng(8)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    want1 = O.allreduce_steps(V, dims)
    want2 = O.allreduce_steps(want1, dims)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_prepare(plan)
    stream = torch.cuda.Stream()
    bufs = upload(V, dev)
    torch.cuda.synchronize()
    say("side stream, two calls back to back")
    with torch.cuda.stream(stream):
        D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, stream)
        D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, stream)
    stream.synchronize()
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want2[j], f"second call learner={j}")
    say("profile entry")
    bufs = upload(V, dev)
    ms = D.ddl_allreduce_sim_profile(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    assert len(ms) == 12 and all(x > 0 for x in ms)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want1[j], f"profile learner={j}")
    say("timed entry")
    bufs = upload(V, dev)
    r_ms, g_ms = D.ddl_allreduce_sim_timed(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    assert r_ms > 0 and g_ms > 0
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want1[j], f"timed learner={j}")


def test_capture_into_a_hip_graph_and_replay(dev):
    """The call is kernel launches only (P <= 256), so it can be stream-captured once the
    plan's device tables exist; every replay must give the eager result."""
    dims, count, P = [4, 2], 300007, 8
    rng = np.random.default_rng(21)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    want = O.allreduce_steps(V, dims)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_prepare(plan)  # allocations happen here, not under capture
    bufs = upload(V, dev)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    say("capturing")
    with torch.cuda.graph(graph, stream=side):
        D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    fused_graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(fused_graph, stream=side):
        D.ddl_allreduce_fused_sim(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    for replay in range(4):
        say(f"replay {replay}")
        for b, v in zip(bufs, V):           # eager work between replays: restore the inputs
            b.copy_(torch.from_numpy(v))
        torch.cuda.synchronize()
        (graph if replay % 2 == 0 else fused_graph).replay()
        for j, g in enumerate(download(bufs)):
            assert_bitwise(g, want[j], f"replay {replay} learner={j}")


@pytest.mark.parametrize("dtype", [D.DDL_F32, D.DDL_F16])
def test_learners_at_different_alignments_within_a_kibibyte(dev, dtype):
    """Learner buffers whose addresses differ modulo 1 KiB (16-byte steps): the kernels lay
    their rows on the destination's 1 KiB boundaries, the source is then misaligned."""
    dims, P = [2, 2, 2], 8
    esz = 4 if dtype == D.DDL_F32 else 2
    G = 16 // esz
    count = 70001
    starts = [j * 80000 + (j * 7 % 64) * G for j in range(P)]   # element offsets, odd multiples of 16 bytes
    rng = np.random.default_rng(52)
    V = wide_inputs(rng, P, count, dtype)
    slab = torch.zeros(P * 80000 + 1024, dtype=torch.float32 if esz == 4 else torch.float16, device=dev)
    bufs = [slab[s0:s0 + count] for s0 in starts]
    assert len({b.data_ptr() % 1024 for b in bufs}) > 4
    for b, v in zip(bufs, V):
        b.copy_(torch.from_numpy(v))
    plan = D.ddl_ring_plan(dims, P, count, dtype)
    D.ddl_allreduce_sim(bufs, P, plan, count, dtype)
    want = O.allreduce_steps(V, dims)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want[j], f"misaligned learner={j}")
    # the fused path on the same layout
    for b, v in zip(bufs, V):
        b.copy_(torch.from_numpy(v))
    D.ddl_allreduce_fused_sim(bufs, P, plan, count, dtype)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want[j], f"misaligned fused learner={j}")
    # nothing outside the learners' ranges was written
    torch.cuda.synchronize()
    mask = torch.ones_like(slab, dtype=torch.bool)
    for s0 in starts:
        mask[s0:s0 + count] = False
    assert not slab[mask].any()


def test_counts_around_row_and_tile_edges(dev):
    """Lengths that end just before, on and after 1 KiB rows, for a 16-bit and a 64-bit type."""
    for dtype, npdt in ((D.DDL_F64, np.float64), (D.DDL_BF16, np.uint16), (D.DDL_F32, np.float32)):
        vl = 16 // np.dtype(npdt).itemsize
        for count in (64 * vl - 1, 64 * vl, 64 * vl + 1, 2 * 64 * vl * 3 + vl - 1, 3 * 64 * vl * 2 + 2 * vl + 1):
            dims, P = [3, 2], 6
            rng = np.random.default_rng(count)
            V = wide_inputs(rng, P, count, dtype)
            bufs = upload(V, dev)
            plan = D.ddl_ring_plan(dims, P, count, dtype)
            D.ddl_allreduce_sim(bufs, P, plan, count, dtype)
            add = O.bf16_add if dtype == D.DDL_BF16 else None
            want = O.allreduce_steps(V, dims, add=add)
            for j, g in enumerate(download(bufs, npdt)):
                assert_bitwise(g, want[j], f"dtype={dtype} count={count} learner={j}")


def test_assignment(dev):
    """Sec. 4.1's basic operation: B copied into A, other memory untouched."""
    for dtype, tdt in ((D.DDL_F32, torch.float32), (D.DDL_F64, torch.float64), (D.DDL_F16, torch.float16)):
        esz = torch.empty(0, dtype=tdt).element_size()
        G = 16 // esz
        for count in (1, G - 1, 64 * G, 64 * G + 1, 100003, 3 * 64 * G * 5 + 7):
            src = (torch.arange(count + 2 * G, device=dev) % 251).to(tdt)
            dst = torch.full((count + 4 * G,), -1, dtype=tdt, device=dev)
            D.ddl_assign_sim(dst[2 * G:], src[G:], count, dtype, torch.cuda.current_stream())
            torch.cuda.synchronize()
            assert torch.equal(dst[2 * G:2 * G + count], src[G:G + count]), (dtype, count)
            assert bool((dst[:2 * G] == -1).all()) and bool((dst[2 * G + count:] == -1).all()), (dtype, count)


def test_denormals_and_infinities_follow_ieee(dev):
    """Subnormal operands and results are kept (no flush to zero), sums that overflow become
    infinite, in every floating type, on both paths."""
    dims, P, count = [2, 2], 4, 4099
    rng = np.random.default_rng(61)
    cases = [
        (D.DDL_F32, np.float32, 1e-41, 3e38),
        (D.DDL_F64, np.float64, 1e-310, 1.5e308),
        (D.DDL_F16, np.float16, 3e-7, 6e4),
    ]
    for dtype, npdt, tiny, huge in cases:
        V = [(rng.uniform(-1, 1, count) * tiny).astype(npdt) for _ in range(P)]
        for v in V:
            v[::7] = npdt(huge)          # some positions overflow when four are added
            v[3::11] = npdt(0.0)
        assert any(np.any((np.abs(v) > 0) & (np.abs(v) < np.finfo(npdt).tiny)) for v in V)
        with np.errstate(over="ignore"):
            want = O.allreduce_steps(V, dims)
        assert np.isinf(want[0]).any()
        assert np.any((np.abs(want[0]) > 0) & (np.abs(want[0]) < np.finfo(npdt).tiny))
        plan = D.ddl_ring_plan(dims, P, count, dtype)
        for entry in (D.ddl_allreduce_sim, D.ddl_allreduce_fused_sim):
            bufs = upload(V, dev)
            entry(bufs, P, plan, count, dtype)
            for j, g in enumerate(download(bufs)):
                assert_bitwise(g, want[j], f"{entry.__name__} dtype={dtype} learner={j}")
    # bf16: subnormal bit patterns through the bit-level helper
    Vb = [O.f32_to_bf16((rng.uniform(-1, 1, count) * 1e-39).astype(np.float32)) for _ in range(P)]
    want = O.allreduce_steps(Vb, dims, add=O.bf16_add)
    plan = D.ddl_ring_plan(dims, P, count, D.DDL_BF16)
    bufs = upload(Vb, dev)
    D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_BF16)
    for j, g in enumerate(download(bufs, np.uint16)):
        assert_bitwise(g, want[j], f"bf16 subnormals learner={j}")


def test_buckets_on_two_streams(dev):
    """A gradient buffer cut into two buckets, each with its own plan on its own stream
    (how a framework would overlap the allreduce of early layers with later compute)."""
    dims, P, count = [2, 4], 8, 400000
    cut = 150000  # multiple of 4 elements: both buckets start 16-byte aligned
    rng = np.random.default_rng(44)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    bufs = upload(V, dev)
    plans = [D.ddl_ring_plan(dims, P, cut), D.ddl_ring_plan(dims, P, count - cut)]
    for p in plans:
        D.ddl_plan_prepare(p)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    views = [[b[:cut] for b in bufs], [b[cut:] for b in bufs]]
    for _ in range(2):  # two rounds back to back on each stream
        for p, st, vw, n in zip(plans, streams, views, (cut, count - cut)):
            D.ddl_allreduce_sim(vw, P, p, n, D.DDL_F32, st)
    for st in streams:
        st.synchronize()
    want_a = O.allreduce_steps(O.allreduce_steps([v[:cut] for v in V], dims), dims)
    want_b = O.allreduce_steps(O.allreduce_steps([v[cut:] for v in V], dims), dims)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g[:cut], want_a[j], f"bucket 0 learner={j}")
        assert_bitwise(g[cut:], want_b[j], f"bucket 1 learner={j}")


def test_one_plan_two_streams_disjoint_buffer_sets(dev):
    """The plan's tables are read-only; every buffer set has its own binding slot, so one
    plan serves two streams at once on disjoint buffers."""
    dims, P, count = [4, 4], 16, 1_000_003
    rng = np.random.default_rng(66)
    VA = wide_inputs(rng, P, count, D.DDL_F32)
    VB = wide_inputs(rng, P, count, D.DDL_F32)
    want_a = O.allreduce_steps(O.allreduce_steps(VA, dims), dims)
    want_b = O.allreduce_steps(O.allreduce_steps(VB, dims), dims)
    plan = D.ddl_ring_plan(dims, P, count)
    A, B = upload(VA, dev), upload(VB, dev)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    say("one plan, two streams, interleaved calls")
    for _ in range(2):
        D.ddl_allreduce_sim(A, P, plan, count, D.DDL_F32, sa)
        D.ddl_allreduce_sim(B, P, plan, count, D.DDL_F32, sb)
    sa.synchronize()
    sb.synchronize()
    for j in range(P):
        assert_bitwise(A[j].cpu().numpy(), want_a[j], f"stream a learner={j}")
        assert_bitwise(B[j].cpu().numpy(), want_b[j], f"stream b learner={j}")
    # the fused path keeps its binding per buffer set as well
    A, B = upload(VA, dev), upload(VB, dev)
    torch.cuda.synchronize()
    D.ddl_allreduce_fused_sim(A, P, plan, count, D.DDL_F32, sa)
    D.ddl_allreduce_fused_sim(B, P, plan, count, D.DDL_F32, sb)
    sa.synchronize()
    sb.synchronize()
    fold_a, fold_b = O.allreduce_fold(VA, dims), O.allreduce_fold(VB, dims)
    for j in range(P):
        assert_bitwise(A[j].cpu().numpy(), fold_a, f"fused stream a learner={j}")
        assert_bitwise(B[j].cpu().numpy(), fold_b, f"fused stream b learner={j}")


def test_one_plan_from_four_host_threads(dev):
    """Four host threads, each with its own stream and buffer set, call through one plan at
    the same time (the binding releases the GIL inside the library): slots are found, created
    and bound under the plan's lock; every thread's result is its own oracle result."""
    import threading
    dims, P, count, rounds = [2, 4], 8, 70001, 6
    plan = D.ddl_ring_plan(dims, P, count)
    rng = np.random.default_rng(5150)
    Vs = [[rng.uniform(-1, 1, count).astype(np.float32) * 1e-2 for _ in range(P)] for _ in range(4)]
    sets = [upload(V, dev) for V in Vs]
    streams = [torch.cuda.Stream() for _ in range(4)]
    torch.cuda.synchronize()
    errors = []

    def work(k):
        try:
            for i in range(rounds):
                entry = D.ddl_allreduce_fused_sim if i % 3 == 2 else D.ddl_allreduce_sim
                entry(sets[k], P, plan, count, D.DDL_F32, streams[k])
            streams[k].synchronize()
        except Exception as e:   # surfaced below: an exception in a thread would otherwise be lost
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for k in range(4):
        want = Vs[k]
        for _ in range(rounds):
            want = O.allreduce_steps(want, dims)
        for j, g in enumerate(download(sets[k])):
            assert_bitwise(g, want[j], f"thread {k} learner={j}")


def test_more_buffer_sets_than_binding_slots(dev):
    """Slots are rebound, least recently used first, once the plan holds its maximum."""
    dims, P, count = [2, 2], 4, 5003
    plan = D.ddl_ring_plan(dims, P, count)
    rng = np.random.default_rng(12)
    sets, wants = [], []
    for i in range(70):  # more than DDL_PLAN_MAX_BINDINGS = 64
        V = [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(P)]
        sets.append(upload(V, dev))
        wants.append(O.allreduce_fold(V, dims))
    for bufs in sets:
        D.ddl_allreduce_sim(bufs, P, plan, count)
    for bufs in sets[:3]:   # evicted by now: bound again; and a second pass over the same set
        D.ddl_allreduce_sim(bufs, P, plan, count)
    torch.cuda.synchronize()
    for i, bufs in enumerate(sets):
        want = wants[i] if i >= 3 else O.allreduce_fold([wants[i]] * P, dims)
        for j in range(P):
            assert_bitwise(bufs[j].cpu().numpy(), want, f"set {i} learner={j}")
    with pytest.raises(D.DdlError) as e:
        D.ddl_plan_reserve_bindings(plan, 65)
    assert e.value.status == D.DDL_ERR_ARG


WALK_CASES = [([4], 1 << 16, D.DDL_F32), ([4], 37, D.DDL_F32), ([2], 1, D.DDL_F32), ([3], 100003, D.DDL_F32),
              ([2, 3], 50001, D.DDL_F32), ([4, 4], 300007, D.DDL_F32), ([3, 1, 2], 70001, D.DDL_F32),
              ([4, 8, 8], 300001, D.DDL_F32), ([4, 8, 8], 1000, D.DDL_F32), ([16], 150001, D.DDL_F32),
              ([20, 2], 99999, D.DDL_F32), ([7, 3], 123457, D.DDL_F64), ([4, 2, 2], 262144 + 13, D.DDL_BF16),
              ([5, 2], 65537, D.DDL_F16), ([9], 4099, D.DDL_I32), ([1, 1], 500, D.DDL_F32), ([2, 2], 0, D.DDL_F32)]


@pytest.mark.parametrize("dims,count,dtype", WALK_CASES)
def test_ring_walk_leaves_every_buffer_as_the_phases_do(dev, dims, count, dtype):
    """One launch per dimension instead of one per phase: after the reduce-scatter every
    learner's whole buffer (partial sums in the chunks it does not own included), after the
    all-gather and after the whole allreduce must equal the step simulator's bit for bit."""
    P = prod(dims)
    say(f"ring walk dims={dims} count={count} dtype={dtype}")
    rng = np.random.default_rng(300 + count + P)
    V = wide_inputs(rng, P, count, dtype)
    add = O.bf16_add if dtype == D.DDL_BF16 else None
    plan = D.ddl_ring_plan(dims, P, count, dtype)
    D.ddl_plan_set_walk(plan, D.DDL_WALK_ON)
    with np.errstate(over="ignore"):
        want_rs = O.reduce_scatter_steps(V, dims, add=add)
        want = O.allgather_steps(want_rs, dims)
    bufs = upload(V, dev)
    D.ddl_reduce_scatter_sim(bufs, P, plan, count, dtype)
    for j, g in enumerate(download(bufs, NP_OF[dtype])):
        assert_bitwise(g, want_rs[j], f"walk reduce-scatter learner={j}")
    D.ddl_allgather_sim(bufs, P, plan, count, dtype)
    for j, g in enumerate(download(bufs, NP_OF[dtype])):
        assert_bitwise(g, want[j], f"walk all-gather learner={j}")
    bufs = upload(V, dev)
    D.ddl_allreduce_sim(bufs, P, plan, count, dtype)
    for j, g in enumerate(download(bufs, NP_OF[dtype])):
        assert_bitwise(g, want[j], f"walk allreduce learner={j}")
    if count:
        assert 0 < D.ddl_plan_walk_bytes(plan) < D.ddl_plan_bytes_moved(plan) or P == 1 or max(dims) == 2


def test_ring_walk_modes_and_limits(dev):
    """AUTO walks launch-bound plans only; the result never depends on the mode; plans without
    the form refuse DDL_WALK_ON."""
    dims, P, count = [4, 2, 2], 16, 20011
    rng = np.random.default_rng(91)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    want = O.allreduce_steps(V, dims)
    for mode in (D.DDL_WALK_AUTO, D.DDL_WALK_OFF, D.DDL_WALK_ON):
        plan = D.ddl_ring_plan(dims, P, count)
        D.ddl_plan_set_walk(plan, mode)
        bufs = upload(V, dev)
        for _ in range(2):
            D.ddl_allreduce_sim(bufs, P, plan, count)
        want2 = O.allreduce_steps(want, dims)
        for j, g in enumerate(download(bufs)):
            assert_bitwise(g, want2[j], f"mode {mode} learner={j}")
        # the measurement entries run phase by phase whatever the mode
        bufs = upload(V, dev)
        ms = D.ddl_allreduce_sim_profile(bufs, P, plan, count)
        assert len(ms) == 10 and all(x > 0 for x in ms)
        for j, g in enumerate(download(bufs)):
            assert_bitwise(g, want[j], f"profile mode {mode} learner={j}")
    with pytest.raises(D.DdlError):
        D.ddl_plan_set_walk(plan, 7)
    # a ring too long for the walk tables: 2 * P * (d + 2) words beyond 2^24
    long_ring = D.ddl_ring_plan([4096], 4096, 64)
    with pytest.raises(D.DdlError) as e:
        D.ddl_plan_set_walk(long_ring, D.DDL_WALK_ON)
    assert e.value.status == D.DDL_ERR_UNSUPPORTED
    assert D.ddl_plan_walk_bytes(long_ring) == 0


def test_capture_with_more_learners_than_the_kernarg_table(dev):
    """Beyond 256 learners the pointers reach the device through kernel arguments too, so
    such a call can be captured; the replay binds its slot itself."""
    dims, count, P = [8, 8, 8], 4099, 512
    V = [I.fill_host(count, 11, j, "uniform") for j in range(P)]
    want = O.allreduce_fold(V, dims)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_prepare(plan)
    bufs = upload(V, dev)
    other = [torch.zeros(count, dtype=torch.float32, device=dev) for _ in range(P)]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    for replay in range(3):
        D.ddl_allreduce_sim(other, P, plan, count)      # eager call on another set in between
        for b, v in zip(bufs, V):
            b.copy_(torch.from_numpy(v))
        torch.cuda.synchronize()
        graph.replay()
        for j, g in enumerate(download(bufs)):
            assert_bitwise(g, want, f"P=512 replay {replay} learner={j}")


def test_buffers_as_aligned_views_of_one_allocation(dev):
    dims, count, P = [2, 2], 10007, 4
    stride = 10240  # elements; multiple of 4 -> 16-byte aligned views, non-overlapping
    rng = np.random.default_rng(9)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    slab = torch.zeros(P * stride, dtype=torch.float32, device=dev)
    bufs = [slab[j * stride: j * stride + count] for j in range(P)]
    for b, v in zip(bufs, V):
        b.copy_(torch.from_numpy(v))
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_allreduce_sim(bufs, P, plan, count)
    want = O.allreduce_steps(V, dims)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want[j], f"view learner={j}")
    # the gaps between the views stay untouched
    torch.cuda.synchronize()
    for j in range(P):
        assert not slab[j * stride + count:(j + 1) * stride].any()
    # misaligned and overlapping views are rejected before anything runs
    with pytest.raises(D.DdlError) as e:
        D.ddl_allreduce_sim([slab[1 + j * stride: 1 + j * stride + count] for j in range(P)], P, plan, count)
    assert e.value.status == D.DDL_ERR_ALIGN
    with pytest.raises(D.DdlError) as e:
        D.ddl_allreduce_sim([slab[j * 5000: j * 5000 + count] for j in range(P)], P, plan, count)
    assert e.value.status == D.DDL_ERR_ARG


def test_more_learners_than_the_kernarg_table_holds(dev):
    dims, count, P = [8, 8, 8], 70001, 512
    say(f"P={P} dims={dims} count={count} (device pointer table path)")
    V = [I.fill_host(count, 3, j, "uniform") for j in range(P)]
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_allreduce_sim(bufs, P, plan, count)
    got = download(bufs)
    want = O.allreduce_fold(V, dims)
    for j in range(P):
        assert_bitwise(got[j], want, f"learner={j}")


# ---------------------------------------------------------------------------------------
# dimension chooser and cost estimate on the GPU machine
# ---------------------------------------------------------------------------------------
def test_chooser_and_estimate_equal_the_oracle_on_this_box():
    """The host-only chooser / estimate checks, run on the GPU machine as well."""
    import test_library_host as H
    H.test_model_time_matches_oracle_and_paper_figures()
    H.test_choose_dims_matches_bruteforce_oracle()


def test_chooser_fed_with_measured_latency_and_rate_picks_a_fast_box(dev):
    """Sec. 4.3's trade-off on one GPU: the latency of a phase is a launch boundary, the
    bandwidth is the memory's.  Time three boxes of 64 learners on one buffer size, fit
    T = phases * L + bytes / B, feed the estimate with the fit: the box ddl_choose_dims
    picks must be within 10 % of the fastest box measured."""
    import time
    P, count = 64, 16384
    bufs = [torch.zeros(count, dtype=torch.float32, device=dev) for _ in range(P)]
    ptrs = D.pointer_array(bufs)
    stream = torch.cuda.current_stream()

    def measure(dims, reps=7, iters=40):
        plan = D.ddl_ring_plan(dims, P, count)
        D.ddl_plan_prepare(plan)
        D.ddl_plan_set_walk(plan, D.DDL_WALK_OFF)
        times = []
        for rep in range(reps + 1):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(iters):
                D.ddl_allreduce_sim(ptrs, P, plan, count, D.DDL_F32, stream)
            torch.cuda.synchronize()
            if rep:   # the first repetition warms up
                times.append((time.perf_counter() - t0) / iters)
        return sorted(times)[len(times) // 2], D.ddl_plan_num_steps(plan), D.ddl_plan_bytes_moved(plan)

    boxes = [[64], [8, 8], [4, 4, 4]]
    rows = [measure(b) for b in boxes]
    A = np.array([[ph, by] for _, ph, by in rows], dtype=np.float64)
    y = np.array([t for t, _, _ in rows])
    (L, invB), *_ = np.linalg.lstsq(A, y, rcond=None)
    say(f"  measured us: {[round(t * 1e6, 1) for t, _, _ in rows]} for {boxes}; fit L = {L * 1e6:.2f} us per phase, "
        f"B = {1e-9 / invB if invB > 0 else float('inf'):.0f} GB/s")
    assert 0.5e-6 < L < 20e-6, "a phase boundary costs microseconds"
    link_bw = (1.0 / invB if invB > 0 else 1e15) / 2.5 / P
    dims, modelled = D.ddl_choose_dims(P, 4 * count, [link_bw] * 6, [float(L)] * 6)
    picked = [d for d in dims if d > 1]
    t_pick, phases, _ = measure(picked)
    fastest = min(min(t for t, _, _ in rows), t_pick)
    say(f"  chooser picks {picked} ({phases} phases): measured {t_pick * 1e6:.1f} us, modelled {modelled * 1e6:.1f} us, "
        f"fastest measured {fastest * 1e6:.1f} us")
    assert t_pick <= 1.10 * fastest
    assert phases <= min(ph for _, ph, _ in rows)   # latency-bound size: fewest phases win


STRIDE_PATHS_CHILD = r"""
import sys
from math import prod
import numpy as np, torch
import oracle.ddl_oracle as O
import paper_1708_02188_amd as D
assert D.library_path().endswith("libddlsim_smallgrid.so"), D.library_path()
dev = torch.device("cuda:0")
rng = np.random.default_rng(2024)
def up(V): return [torch.from_numpy(np.ascontiguousarray(v.view(np.int16) if v.dtype == np.uint16 else v)).to(dev) for v in V]
def check(bufs, want, what):
    torch.cuda.synchronize()
    for j, b in enumerate(bufs):
        g = b.cpu().numpy().view(want[j].dtype) if isinstance(want, list) else b.cpu().numpy().view(want.dtype)
        w = want[j] if isinstance(want, list) else want
        assert g.tobytes() == w.tobytes(), f"{what}: learner {j} differs"
    print("ok", what, flush=True)
# a launch holds 65536 threads: (1023 // P) tiles of 1 KiB per operation, the kernels stride over the rest
for dims, count in (([4, 4], 1_000_003), ([2], 300_001), ([4, 8, 8], 300_001)):
    P = prod(dims)
    V = [(rng.uniform(-1, 1, count) * 10.0 ** rng.uniform(-3, 3, count)).astype(np.float32) for _ in range(P)]
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_set_walk(plan, D.DDL_WALK_OFF)
    want = O.allreduce_fold(V, dims)
    b = up(V); D.ddl_allreduce_sim(b, P, plan, count); check(b, want, f"phases {dims} {count}")
    b = up(V); D.ddl_allreduce_fused_sim(b, P, plan, count); check(b, want, f"fused {dims} {count}")
    b = up(V); D.ddl_allreduce_sim_noalloc(b, P, plan, count); check(b, want, f"noalloc {dims} {count}")
    D.ddl_plan_set_walk(plan, D.DDL_WALK_ON)
    b = up(V); D.ddl_allreduce_sim(b, P, plan, count); check(b, want, f"ring walk {dims} {count}")
# 16-bit elements
dims, count, P = [3, 2], 700_001, 6
V = [O.f32_to_bf16(rng.uniform(-1, 1, count).astype(np.float32)) for _ in range(P)]
plan = D.ddl_ring_plan(dims, P, count, D.DDL_BF16)
b = up(V); D.ddl_allreduce_sim(b, P, plan, count, D.DDL_BF16); check(b, O.allreduce_steps(V, dims, add=O.bf16_add), "bf16 phases")
b = up(V); D.ddl_allreduce_fused_sim(b, P, plan, count, D.DDL_BF16); check(b, O.allreduce_fold(V, dims, add=O.bf16_add), "bf16 fused")
# assignment of one long range
src = torch.arange(2_000_003, device=dev, dtype=torch.float32); dst = torch.zeros_like(src)
D.ddl_assign_sim(dst, src, src.numel()); torch.cuda.synchronize(); assert torch.equal(src, dst); print("ok assign", flush=True)
# several-tensor plan: a phase of more than 1000 workgroups is split into several launches
dims, P = [4, 2], 8
segments, count = [(0, 64), (64, 100_000), (100_064, 7), (100_072, 1_500_001), (1_600_076, 33)], 1_600_076 + 33
V = [(rng.uniform(-1, 1, count) * 10.0 ** rng.uniform(-3, 3, count)).astype(np.float32) for _ in range(P)]
plan = D.ddl_ring_plan_tensors(dims, P, [o for o, _ in segments], [n for _, n in segments], count)
D.ddl_plan_set_walk(plan, D.DDL_WALK_OFF)
b = up(V); D.ddl_allreduce_sim(b, P, plan, count); check(b, O.allreduce_tensors(V, dims, segments), "tensor plan, split launches")
D.ddl_plan_set_walk(plan, D.DDL_WALK_ON)
b = up(V); D.ddl_allreduce_sim(b, P, plan, count); check(b, O.allreduce_tensors(V, dims, segments), "tensor plan, ring walk, split launches")
print("stride paths ok")
"""


def test_striding_and_split_launch_paths_in_a_small_grid_build(dev):
    """Every kernel strides over the tiles its grid does not cover once an operation exceeds
    2^32 / 64 workgroups, and a several-tensor phase of more than 2^26 workgroups is split
    into several launches.  libddlsim_smallgrid.so is the same source built with those
    limits set to 65536 threads and 1000 workgroups, so inputs of test size run exactly
    those paths; a fresh process loads it and is checked against the oracle."""
    import os
    import subprocess
    from conftest import ROOT
    lib = os.path.join(os.path.dirname(D.library_path()), "libddlsim_smallgrid.so")
    assert os.path.exists(lib), "build it with python -m paper_1708_02188_amd.build"
    env = dict(os.environ, DDLSIM_LIBRARY=lib)
    run = subprocess.run([sys.executable, "-c", STRIDE_PATHS_CHILD], cwd=ROOT, capture_output=True, text=True,
                         timeout=600, env=env)
    say(run.stdout)
    assert run.returncode == 0 and "stride paths ok" in run.stdout, run.stderr[-3000:]


def test_four_thousand_learners(dev):
    """4096 learners as the box [16,16,16]: sixteen slices of the pointer table, rings of 16
    (two load batches in the ring walk), chunks of a handful of elements."""
    dims, P, count = [16, 16, 16], 4096, 20001
    say(f"P={P} dims={dims} count={count}")
    V = [I.fill_host(count, 9, j, "uniform") for j in range(P)]
    want = O.allreduce_steps(V, dims)
    for mode in (D.DDL_WALK_OFF, D.DDL_WALK_ON):
        plan = D.ddl_ring_plan(dims, P, count)
        D.ddl_plan_verify(plan)
        D.ddl_plan_set_walk(plan, mode)
        bufs = upload(V, dev)
        D.ddl_allreduce_sim(bufs, P, plan, count)
        torch.cuda.synchronize()
        for j in range(P):
            assert_bitwise(bufs[j].cpu().numpy(), want[j], f"walk mode {mode} learner={j}")
    with pytest.raises(D.DdlError) as e:
        D.ddl_allreduce_fused_sim(bufs, P, plan, count)
    assert e.value.status == D.DDL_ERR_UNSUPPORTED


# ---------------------------------------------------------------------------------------
# seeded random sweep over boxes, lengths, element types and entry points
# ---------------------------------------------------------------------------------------
def random_box(rng, max_P=48):
    dims = []
    P = 1
    for _ in range(int(rng.integers(1, 5))):
        d = int(rng.integers(1, 7))
        if P * d > max_P:
            break
        dims.append(d)
        P *= d
    return dims or [1]


def test_random_sweep_against_oracle(dev):
    rng = np.random.default_rng(20260101)
    dtypes = [D.DDL_F32, D.DDL_F64, D.DDL_I32, D.DDL_F16, D.DDL_BF16]
    for case in range(100):
        dims = random_box(rng)
        P = prod(dims)
        dtype = dtypes[int(rng.integers(0, len(dtypes)))]
        count = int(rng.choice([0, 1, 3, 17, 255, 1024, 4097, 30011, 200003]) + rng.integers(0, 9))
        entry = ["allreduce", "fused", "tensors", "walk", "noalloc"][int(rng.integers(0, 5))]
        levels = sum(d > 1 for d in dims)
        if entry == "fused" and levels > 4:
            entry = "allreduce"
        say(f"case {case}: dims={dims} dtype={dtype} count={count} entry={entry}")
        V = wide_inputs(rng, P, count, dtype)
        add = O.bf16_add if dtype == D.DDL_BF16 else None
        bufs = upload(V, dev)
        with np.errstate(over="ignore"):
            if entry == "tensors":
                G = 16 // V[0].dtype.itemsize
                cuts = sorted(set(int(x) // G * G for x in rng.integers(0, count + 1, 5)) | {0})
                segments = [(a, int(rng.integers(0, b - a + 1))) for a, b in zip(cuts, cuts[1:] + [count])]
                plan = D.ddl_ring_plan_tensors(dims, P, [o for o, _ in segments], [n for _, n in segments],
                                               count, dtype)
                D.ddl_plan_set_walk(plan, D.DDL_WALK_ON if case % 2 else D.DDL_WALK_OFF)
                D.ddl_allreduce_sim(bufs, P, plan, count, dtype)
                want = O.allreduce_tensors(V, dims, segments, add=add)
            else:
                plan = D.ddl_ring_plan(dims, P, count, dtype)
                D.ddl_plan_set_walk(plan, D.DDL_WALK_ON if entry == "walk" else D.DDL_WALK_OFF)
                if entry == "fused":
                    D.ddl_allreduce_fused_sim(bufs, P, plan, count, dtype)
                elif entry == "noalloc":
                    D.ddl_allreduce_sim_noalloc(bufs, P, plan, count, dtype)
                else:
                    D.ddl_allreduce_sim(bufs, P, plan, count, dtype)
                want = O.allreduce_steps(V, dims, add=add)
        for j, g in enumerate(download(bufs, V[0].dtype)):
            assert_bitwise(g, want[j], f"case {case} learner={j}")


# ---------------------------------------------------------------------------------------
# several tensors per buffer, each reduced on its own, transfers batched per phase
# ---------------------------------------------------------------------------------------
TENSOR_CASES = [
    ([4], [(0, 64), (64, 4), (68, 0), (72, 1000), (1072, 8), (1100, 37)], 1140),
    ([2, 3], [(0, 5), (8, 3), (16, 100000)], 100016),
    ([4, 4], [(0, 70000), (70000, 16), (70016, 4), (70020, 300000), (370020, 1)], 370021),
    ([4, 2, 2], [(4 * i * 50, 150 + i) for i in range(40)] + [(8000, 262144 + 5)], 8000 + 262144 + 5),
    ([3], [(0, 1), (4, 2), (8, 3)], 11),
]


@pytest.mark.parametrize("dims,segments,count", TENSOR_CASES)
def test_tensor_plan_matches_per_tensor_oracle(dev, dims, segments, count):
    P = prod(dims)
    say(f"tensor plan dims={dims} tensors={len(segments)} count={count}")
    rng = np.random.default_rng(600 + count)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan_tensors(dims, P, [o for o, _ in segments], [n for _, n in segments], count)
    D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    got = download(bufs)
    want = O.allreduce_tensors(V, dims, segments)   # gaps between tensors keep their input values
    for j in range(P):
        assert_bitwise(got[j], want[j], f"tensor plan dims={dims} learner={j}")
    # the halves on their own
    bufs = upload(V, dev)
    D.ddl_reduce_scatter_sim(bufs, P, plan, count)
    rs = download(bufs)
    steps = O.schedule_tensors(dims, segments, 4)
    want_rs = O._run([v.copy() for v in V], [st for st in steps if st[0] == "RS"])
    for j in range(P):
        assert_bitwise(rs[j], want_rs[j], f"tensor plan reduce-scatter learner={j}")
    D.ddl_allgather_sim(bufs, P, plan, count)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want[j], f"tensor plan all-gather learner={j}")


@pytest.mark.parametrize("dims,segments,count", TENSOR_CASES)
def test_tensor_plan_ring_walk(dev, dims, segments, count):
    """Several tensors, one launch per dimension: whole buffers after the reduce-scatter, the
    all-gather and the allreduce equal the phases' (gaps between tensors untouched)."""
    P = prod(dims)
    say(f"tensor plan, ring walk dims={dims} tensors={len(segments)} count={count}")
    rng = np.random.default_rng(700 + count)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    plan = D.ddl_ring_plan_tensors(dims, P, [o for o, _ in segments], [n for _, n in segments], count)
    D.ddl_plan_verify(plan)
    D.ddl_plan_set_walk(plan, D.DDL_WALK_ON)
    steps = O.schedule_tensors(dims, segments, 4)
    want_rs = O._run([v.copy() for v in V], [st for st in steps if st[0] == "RS"])
    want = O.allreduce_tensors(V, dims, segments)
    bufs = upload(V, dev)
    D.ddl_reduce_scatter_sim(bufs, P, plan, count)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want_rs[j], f"walk reduce-scatter learner={j}")
    D.ddl_allgather_sim(bufs, P, plan, count)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want[j], f"walk all-gather learner={j}")
    bufs = upload(V, dev)
    D.ddl_allreduce_sim(bufs, P, plan, count)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want[j], f"walk allreduce learner={j}")


def test_tensor_plan_sixteen_bit(dev):
    dims, P = [2, 2], 4
    segments, count = [(0, 24), (24, 808), (832, 9), (848, 70001)], 848 + 70001
    rng = np.random.default_rng(71)
    V = wide_inputs(rng, P, count, D.DDL_BF16)
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan_tensors(dims, P, [o for o, _ in segments], [n for _, n in segments], count, D.DDL_BF16)
    D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_BF16)
    want = O.allreduce_tensors(V, dims, segments, add=O.bf16_add)
    for j, g in enumerate(download(bufs, np.uint16)):
        assert_bitwise(g, want[j], f"bf16 tensor plan learner={j}")
    D.ddl_plan_set_walk(plan, D.DDL_WALK_ON)
    bufs = upload(V, dev)
    D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_BF16)
    for j, g in enumerate(download(bufs, np.uint16)):
        assert_bitwise(g, want[j], f"bf16 tensor plan, ring walk learner={j}")


# ---------------------------------------------------------------------------------------
# step-fused allreduce: same final bits as the phase-by-phase schedule
# ---------------------------------------------------------------------------------------
FUSED_CASES = [([1], 100), ([2], 1), ([4], 37), ([4], 65536 + 5), ([3], 100003), ([2, 3], 50001), ([4, 4], 300007),
               ([3, 1, 2], 70001), ([4, 2, 2], 262144 + 13), ([2, 2, 2, 2], 99999), ([16], 150001),
               ([4, 16], 200003), ([4, 8, 8], 1000), ([4, 8, 8], 300001), ([7, 3], 123457), ([5], 3), ([2, 2], 0),
               ([1, 4, 1, 2, 1], 4099)]


@pytest.mark.parametrize("dims,count", FUSED_CASES)
def test_fused_allreduce_matches_fold_fp32(dev, dims, count):
    P = prod(dims)
    say(f"fused allreduce f32 dims={dims} count={count}")
    rng = np.random.default_rng(4000 + count + P)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_allreduce_fused_sim(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    got = download(bufs)
    want = O.allreduce_fold(V, dims)
    for j in range(P):
        assert_bitwise(got[j], want, f"fused dims={dims} count={count} learner={j}")
    # and therefore the same as executing the phases
    bufs2 = upload(V, dev)
    D.ddl_allreduce_sim(bufs2, P, plan, count)
    for j, g in enumerate(download(bufs2)):
        assert_bitwise(g, got[j], f"fused vs phases learner={j}")


@pytest.mark.parametrize("dtype", [D.DDL_F64, D.DDL_I32, D.DDL_F16, D.DDL_BF16])
@pytest.mark.parametrize("dims,count", [([4], 10001), ([2, 3], 65537), ([4, 4], 131072 + 3), ([3], 1), ([4, 2, 2], 7)])
def test_fused_allreduce_other_dtypes(dev, dtype, dims, count):
    P = prod(dims)
    say(f"fused allreduce dtype={dtype} dims={dims} count={count}")
    rng = np.random.default_rng(99 + count)
    V = wide_inputs(rng, P, count, dtype)
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan(dims, P, count, dtype)
    D.ddl_allreduce_fused_sim(bufs, P, plan, count, dtype)
    got = download(bufs, NP_OF[dtype])
    with np.errstate(over="ignore"):
        want = O.allreduce_fold(V, dims, add=O.bf16_add if dtype == D.DDL_BF16 else None)
    for j in range(P):
        assert_bitwise(got[j], want, f"fused dtype={dtype} dims={dims} learner={j}")


@pytest.mark.parametrize("dims,count", [([4], 20003), ([2, 3], 9001), ([4, 2, 2], 100001), ([4, 8, 8], 300001)])
def test_fused_halves_alone(dev, dims, count):
    """ReduceScatter / AllGather as single passes: owner's chunk = the schedule-order sum,
    nothing else written; then every owner's chunk copied everywhere."""
    P = prod(dims)
    say(f"fused halves dims={dims} count={count}")
    rng = np.random.default_rng(77)
    V = wide_inputs(rng, P, count, D.DDL_F32)
    fold = O.allreduce_fold(V, dims)
    plan = D.ddl_ring_plan(dims, P, count)
    bufs = upload(V, dev)
    D.ddl_reduce_scatter_fused_sim(bufs, P, plan, count)
    got = download(bufs)
    for j in range(P):
        want = V[j].copy()
        off, n = D.ddl_plan_owned_chunk(plan, j)
        want[off:off + n] = fold[off:off + n]
        assert_bitwise(got[j], want, f"fused reduce-scatter learner={j}")
    D.ddl_allgather_fused_sim(bufs, P, plan, count)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, fold, f"fused all-gather learner={j}")


def test_fused_allreduce_many_learners_and_limits(dev):
    dims, count, P = [8, 8, 8], 70001, 512
    V = [I.fill_host(count, 5, j, "uniform") for j in range(P)]
    bufs = upload(V, dev)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_allreduce_fused_sim(bufs, P, plan, count)
    want = O.allreduce_fold(V, dims)
    for j, g in enumerate(download(bufs)):
        assert_bitwise(g, want, f"fused P=512 learner={j}")
    # five rings of size 2: more levels than the fused kernel nests
    plan5 = D.ddl_ring_plan([2] * 5, 32, 64)
    small = [torch.zeros(64, dtype=torch.float32, device=dev) for _ in range(32)]
    with pytest.raises(D.DdlError) as e:
        D.ddl_allreduce_fused_sim(small, 32, plan5, 64)
    assert e.value.status == D.DDL_ERR_UNSUPPORTED


# ---------------------------------------------------------------------------------------
# the benchmark configurations at full size, device-generated inputs
# ---------------------------------------------------------------------------------------
def sample_ranges(plan, P, count, width=2048, extra=12):
    """Element ranges the oracle recomputes: both ends of the buffer, both sides of a
    selection of chunk boundaries (kernel tile tails sit there), and random places."""
    rng = np.random.default_rng(count)
    edges = {0, count}
    for j in sorted(set([0, 1, P // 2, P - 1] + list(rng.integers(0, P, 4)))):
        off, n = D.ddl_plan_owned_chunk(plan, int(j))
        edges.update((off, off + n))
    ranges = []
    for e in sorted(edges):
        ranges.append((max(0, e - width // 2), min(count, e + width // 2)))
    for a in rng.integers(0, max(1, count - width), extra):
        ranges.append((int(a), min(count, int(a) + width)))
    return [(a, b) for a, b in ranges if b > a]


PIECE = 1 << 17   # elements the oracle folds per task (P * PIECE * 4 bytes of inputs per worker)
WORKERS = 16      # the GPU machine's CPU share


def compare_whole(results, dims, seed, dist, tensors, what):
    """Every element of `results` (name -> learner 0's buffer on the host) against the oracle's
    nested fold, computed piece by piece on a thread pool straight from the generator
    (numpy and the generator release the GIL).  `tensors` = [(offset, length)]: each is
    chunked and reduced on its own; a one-buffer plan is the single tensor (0, count)."""
    import time
    from concurrent.futures import ThreadPoolExecutor

    P = prod(dims)
    # A tensor short enough that its finest chunks are tiny is cheaper by the step simulator,
    # whole (one task, P * n * 4 bytes of inputs); the nested fold would make P x P small reads.
    short = 8192 * P // 2
    tasks = [(off, n, a, min(n, a + PIECE)) for off, n in tensors if n > short for a in range(0, n, PIECE)]
    tasks += [(off, n, 0, n) for off, n in tensors if n <= short]
    tasks.sort(key=lambda t: t[2] - t[3])   # longest first
    schedules = {}   # phases of a short tensor, by length (layer sizes repeat)

    def one(task):
        off, n, a, b = task
        if n <= short:
            if n not in schedules:
                schedules[n] = O.schedule(dims, n, 4)
            V = [I.fill_host(n, seed, r, dist, first=off) for r in range(P)]
            want = O._run(V, schedules[n])[0]
        else:
            want = O.allreduce_fold_range(lambda r, lo, hi: I.fill_host(hi - lo, seed, r, dist, first=off + lo),
                                          dims, n, a, b, np.float32)
        for name, got in results.items():
            assert_bitwise(got[off + a:off + b], want, f"{what} {name}: tensor at {off}, elements [{a},{b})")
        return b - a

    t0 = time.perf_counter()
    with ThreadPoolExecutor(WORKERS) as pool:
        compared = sum(pool.map(one, tasks))
    say(f"  {what}: {compared} elements x {len(results)} result(s) compared with the oracle, every one equal, "
        f"{len(tasks)} pieces, {time.perf_counter() - t0:.1f} s")
    return compared


def fp64_closeness(got, P, dims, count, seed, dist, ranges):
    """|x - fp64 sum| <= 1e-5 * sum_j |V_j| per element and <= 1e-5 * max|fp64 sum| overall."""
    worst = 0.0
    for a, b in ranges:
        V = [I.fill_host(b - a, seed, r, dist, first=a) for r in range(P)]
        ref = O.sum_fp64(V)
        absum = sum(np.abs(v.astype(np.float64)) for v in V)
        err = np.abs(got[a:b].astype(np.float64) - ref)
        assert np.all(err <= 1e-5 * absum)
        if dist == "int8":
            assert np.array_equal(got[a:b].astype(np.float64), ref)  # integers: exact
        worst = max(worst, float(np.max(err)) / max(float(np.max(np.abs(ref))), 1e-30))
    assert worst <= 1e-5
    return worst


def device_result(dev, cfg, entry, plan):
    """Run `entry` on the configuration's device-generated inputs; all learners must hold the
    same bits; returns learner 0's buffer on the host."""
    P, count, dist, seed = cfg["P"], cfg["count"], cfg["dist"], cfg["seed"]
    bufs = [torch.empty(count, dtype=torch.float32, device=dev) for _ in range(P)]
    for j, b in enumerate(bufs):
        I.fill_device(b, seed, j, dist)
    torch.cuda.synchronize()
    entry(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for j in range(1, P):
        assert torch.equal(bufs[0].view(torch.int32), bufs[j].view(torch.int32)), f"learner {j} differs from 0"
    got = bufs[0].cpu().numpy()
    del bufs
    torch.cuda.empty_cache()
    return got


def run_config(dev, cfg, fused=True, per_tensor=False):
    """One benchmark configuration at full size: the phase-by-phase schedule and the
    step-fused form, whole buffer of learner 0 against the oracle (the other learners are
    compared with learner 0 on the device), fp64 closeness on sampled ranges."""
    P, dims, count, dist, seed = cfg["P"], cfg["dims"], cfg["count"], cfg["dist"], cfg["seed"]
    say(f"config {cfg['name']}: P={P} dims={dims} count={count} dist={dist} seed={seed}")
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_set_walk(plan, D.DDL_WALK_OFF)
    results = {"ddl_allreduce_sim": device_result(dev, cfg, D.ddl_allreduce_sim, plan)}
    walk_plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_set_walk(walk_plan, D.DDL_WALK_ON)
    results["ddl_allreduce_sim, ring walk"] = device_result(dev, cfg, D.ddl_allreduce_sim, walk_plan)
    if fused:
        results["ddl_allreduce_fused_sim"] = device_result(dev, cfg, D.ddl_allreduce_fused_sim, plan)
    assert compare_whole(results, dims, seed, dist, [(0, count)], cfg["name"]) == count
    worst = fp64_closeness(results["ddl_allreduce_sim"], P, dims, count, seed, dist, sample_ranges(plan, P, count))
    say(f"  fp64 closeness on sampled ranges: worst |x - fp64| / max|fp64| = {worst:.2e}")
    if per_tensor:
        shapes = I.resnet50_shapes() if count == I.RESNET50_COUNT else I.resnet101_22k_shapes()
        offs, cnts = I.tensor_segments(shapes)
        tplan = D.ddl_ring_plan_tensors(dims, P, offs, cnts, count)
        D.ddl_plan_set_walk(tplan, D.DDL_WALK_OFF)
        got = {"per-tensor plan": device_result(dev, cfg, D.ddl_allreduce_sim, tplan)}
        D.ddl_plan_set_walk(tplan, D.DDL_WALK_ON)
        got["per-tensor plan, ring walk"] = device_result(dev, cfg, D.ddl_allreduce_sim, tplan)
        n = compare_whole(got, dims, seed, dist, list(zip(offs, cnts)), f"{cfg['name']} as {len(offs)} tensors")
        assert n == count


def test_buffers_beyond_four_gibibytes(dev):
    """Two learners of 4.8 GB each: element and byte offsets that do not fit 32 bits."""
    P, dims, count, seed = 2, [2], 1_200_000_003, 4242
    say(f"large buffers: P={P} count={count} ({4 * count / 2**30:.2f} GiB per learner)")
    bufs = [torch.empty(count, dtype=torch.float32, device=dev) for _ in range(P)]
    plan = D.ddl_ring_plan(dims, P, count)
    rng = np.random.default_rng(1)
    ranges = [(0, 4096), (count - 4099, count), (count // 2 - 2048, count // 2 + 2048),
              (2 ** 30 - 1024, 2 ** 30 + 1024)] + [(int(a), int(a) + 2048) for a in rng.integers(0, count - 2048, 6)]
    for entry in (D.ddl_allreduce_sim, D.ddl_allreduce_fused_sim):
        for j, b in enumerate(bufs):
            I.fill_device(b, seed, j, "uniform")
        entry(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert torch.equal(bufs[0].view(torch.int32), bufs[1].view(torch.int32))
        for a, b in ranges:
            want = O.allreduce_fold_range(lambda r, lo, hi: I.fill_host(hi - lo, seed, r, "uniform", first=lo),
                                          dims, count, a, b, np.float32)
            assert_bitwise(bufs[1][a:b].cpu().numpy(), want, f"{entry.__name__} elements [{a},{b})")


def test_config1_ring4_integer_exact(dev):
    run_config(dev, I.CONFIGS[0])


def test_config2_box4x4_resnet50_whole_buffer(dev):
    run_config(dev, I.CONFIGS[1], per_tensor=True)


def test_config2_first_range_fp64(dev):
    # fp64 closeness over a 4 M element prefix of the ResNet-50-sized buffer
    cfg = I.CONFIGS[1]
    plan = D.ddl_ring_plan(cfg["dims"], cfg["P"], cfg["count"])
    got = device_result(dev, cfg, D.ddl_allreduce_sim, plan)
    fp64_closeness(got, cfg["P"], cfg["dims"], cfg["count"], cfg["seed"], cfg["dist"], [(0, 1 << 22)])


def test_config3_box4x16_resnet50_layers_whole_buffer(dev):
    run_config(dev, I.CONFIGS[2], per_tensor=True)


def test_config4_box4x8x8_resnet50_whole_buffer(dev):
    run_config(dev, I.CONFIGS[3])


def test_config5_box4x8x8_resnet101_22k_whole_buffer(dev):
    run_config(dev, I.CONFIGS[4])


def test_config5_per_tensor_plan_whole_buffer(dev):
    """Configuration 5's buffer as the 314 tensors of ResNet-101 with the 22K-class head."""
    cfg = I.CONFIGS[4]
    offs, cnts = I.tensor_segments(I.resnet101_22k_shapes())
    tplan = D.ddl_ring_plan_tensors(cfg["dims"], cfg["P"], offs, cnts, cfg["count"])
    D.ddl_plan_set_walk(tplan, D.DDL_WALK_OFF)
    got = {"per-tensor plan": device_result(dev, cfg, D.ddl_allreduce_sim, tplan)}
    D.ddl_plan_set_walk(tplan, D.DDL_WALK_ON)
    got["per-tensor plan, ring walk"] = device_result(dev, cfg, D.ddl_allreduce_sim, tplan)
    n = compare_whole(got, cfg["dims"], cfg["seed"], cfg["dist"], list(zip(offs, cnts)),
                      f"{cfg['name']} as {len(offs)} tensors")
    assert n == cfg["count"]
