"""The allocation-free entry point gives ddl_allreduce_sim's result, bit for bit, on two
calls in a row that share its static device array, the second on a smaller input."""
import sys
from math import prod

import numpy as np
import pytest
import torch

import oracle.ddl_oracle as O
import paper_1708_02188_amd as D

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def both_entries(dev, dims, count, seed):
    P = prod(dims)
    rng = np.random.default_rng(seed)
    V = [(rng.uniform(-1, 1, count) * 10.0 ** rng.uniform(-3, 3, count)).astype(np.float32) for _ in range(P)]
    plan = D.ddl_ring_plan(dims, P, count)
    stream = torch.cuda.current_stream()
    ref = [torch.from_numpy(v).to(dev) for v in V]
    D.ddl_allreduce_sim(ref, P, plan, count, D.DDL_F32, stream)
    new = [torch.from_numpy(v).to(dev) for v in V]
    say(f"  ddl_allreduce_sim_noalloc dims={dims} count={count}")
    D.ddl_allreduce_sim_noalloc(new, P, plan, count, D.DDL_F32, stream)
    torch.cuda.synchronize()
    want = O.allreduce_steps(V, dims)
    for j in range(P):
        a, b = ref[j].cpu().numpy(), new[j].cpu().numpy()
        assert a.tobytes() == b.tobytes(), f"dims={dims} count={count}: learner {j} differs from ddl_allreduce_sim"
        assert b.tobytes() == want[j].tobytes(), f"dims={dims} count={count}: learner {j} differs from the oracle"


def test_noalloc_entry_equals_allocating_entry_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a device")
    dev = torch.device("cuda:0")
    # the second call is smaller in learners, phases and elements: records the first call
    # left in the static array beyond the second call's must not matter
    both_entries(dev, [4, 2, 4], 300007, 1)
    both_entries(dev, [3, 2], 4099, 2)
    both_entries(dev, [4, 8, 8], 70001, 3)
    both_entries(dev, [2], 5, 4)


def test_noalloc_entry_under_stream_capture():
    """Its reason to exist: captured into a HIP graph (nothing may allocate there), replayed
    with eager calls of both entry points in between; every replay gives the oracle's bits."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a device")
    dev = torch.device("cuda:0")
    dims, P, count = [4, 2, 2], 16, 50021
    rng = np.random.default_rng(77)
    V = [rng.uniform(-1, 1, count).astype(np.float32) for _ in range(P)]
    want = O.allreduce_steps(V, dims)
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_prepare(plan)   # set-up: looks the static array's address up on this device
    bufs = [torch.from_numpy(v).to(dev) for v in V]
    other = [torch.ones(count, dtype=torch.float32, device=dev) for _ in range(P)]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    say("  capturing ddl_allreduce_sim_noalloc")
    with torch.cuda.graph(graph, stream=side):
        D.ddl_allreduce_sim_noalloc(bufs, P, plan, count, D.DDL_F32, torch.cuda.current_stream())
    for replay in range(3):
        # eager calls in between rewrite the shared static array for other buffers
        D.ddl_allreduce_sim_noalloc(other, P, plan, count)
        D.ddl_allreduce_sim(other, P, plan, count)
        for b, v in zip(bufs, V):
            b.copy_(torch.from_numpy(v))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for j in range(P):
            assert bufs[j].cpu().numpy().tobytes() == want[j].tobytes(), f"replay {replay}: learner {j} differs"


def test_noalloc_entry_limits_are_errors():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a device")
    dev = torch.device("cuda:0")
    # a flat ring of 200 learners has 398 phases x 200 records: beyond the static array
    P, count = 200, 1024
    plan = D.ddl_ring_plan([P], P, count)
    bufs = [torch.zeros(count, dtype=torch.float32, device=dev) for _ in range(P)]
    with pytest.raises(D.DdlError) as e:
        D.ddl_allreduce_sim_noalloc(bufs, P, plan, count)
    assert e.value.status == D.DDL_ERR_UNSUPPORTED
    # more learners than the kernel-argument table holds
    P = 512
    plan = D.ddl_ring_plan([8, 8, 8], P, count)
    bufs = [torch.zeros(count, dtype=torch.float32, device=dev) for _ in range(P)]
    with pytest.raises(D.DdlError) as e:
        D.ddl_allreduce_sim_noalloc(bufs, P, plan, count)
    assert e.value.status == D.DDL_ERR_UNSUPPORTED
    # a several-tensor plan
    plan = D.ddl_ring_plan_tensors([2, 2], 4, [0, 512], [100, 512], count)
    with pytest.raises(D.DdlError) as e:
        D.ddl_allreduce_sim_noalloc(bufs[:4], 4, plan, count)
    assert e.value.status == D.DDL_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert not any(bool(b.any()) for b in bufs[:4])
