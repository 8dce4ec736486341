#!/usr/bin/env python3
"""Benchmark of the simulated multi-ring allreduce on one MI355X.

A step is one whole allreduce (every reduce-scatter and all-gather phase of the schedule)
over one set of P synthetic learner buffers that is already resident in HBM.  Every step
runs between its own pair of HIP events on the stream the kernels are launched on; the
buffers are refilled from the seeded generator before every step, outside the events, so
every step sums fresh N(0, 1e-2) or uniform data and nothing overflows.  Prints ONE JSON
line: allreduce GB/s per virtual learner (`value`, from the median step), the HBM roofline
of the dominant kernel, the other configurations as secondary entries, and the CPU oracle
timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--no-cpu]
    python bench.py --dims 4,8 --count 1000000 --dist uniform --seed 7     # ad-hoc shape
"""
import argparse
import json
import os
import statistics
import sys
import time
from math import prod

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per launch of the dominant kernel from rocprofv3 counter runs (FETCH_SIZE and
# WRITE_SIZE, each in a run of its own, scaled by the same counters' reading for a plain
# copy of known size).  Recorded figures, not measured by this program: a counter run needs
# the profiler around the process.  The summaries that hold them are named beside them.
RECORDED_TRAFFIC = {
    "c5_box4x8x8_resnet101_22k": {
        "bytes_per_launch": 15705330190,
        "source": "profiles/all_kernels_c5_box4x8x8_resnet101_22k_hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE and "
                  "WRITE_SIZE runs of this program, average over reduce_add_step's 17 launches per allreduce "
                  "(algorithmic 15705426420); recorded there, not measured in this run",
    },
}


def time_calls(torch, stream, call, refill, K, W):
    """W untimed calls, then K calls each between its own event pair on `stream`;
    refill(i) runs before call(i), outside the events.  Returns the K times in ms and the
    wall-clock seconds of the timed loop (refills included)."""
    for i in range(W):
        refill(i)
        call(i)
    torch.cuda.synchronize()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
    t0 = time.perf_counter()
    for i in range(K):
        refill(W + i)
        pairs[i][0].record(stream)
        call(W + i)
        pairs[i][1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return [a.elapsed_time(b) for a, b in pairs], wall


def rate(nbytes, ms):
    gbs = nbytes / (ms * 1e-3) / 1e9
    return gbs, gbs / HBM_PEAK_GBS


class Workload:
    """One configuration resident on the device: `n_sets` sets of P learner buffers."""

    def __init__(self, torch, D, I, dev, cfg, n_sets):
        self.torch, self.D, self.I, self.cfg = torch, D, I, cfg
        self.P, self.dims, self.count = cfg["P"], cfg["dims"], cfg["count"]
        self.dist, self.seed = cfg["dist"], cfg["seed"]
        self.stream = torch.cuda.current_stream()
        self.sets = [[torch.empty(self.count, dtype=torch.float32, device=dev) for _ in range(self.P)]
                     for _ in range(n_sets)]
        # pointer arrays are built once: the timed calls marshal nothing
        self.ptrs = [D.pointer_array(s) for s in self.sets]
        self.plan = D.ddl_ring_plan(self.dims, self.P, self.count)
        D.ddl_plan_prepare(self.plan)

    def refill(self, i):
        bufs = self.sets[i % len(self.sets)]
        for j, b in enumerate(bufs):
            self.I.fill_device(b, self.seed + 1000 * i, j, self.dist, 0, self.stream)

    def entry(self, fn, plan=None):
        plan = plan or self.plan
        return lambda i: fn(self.ptrs[i % len(self.sets)], self.P, plan, self.count, self.D.DDL_F32, self.stream)

    def measure(self, fn, K, W, plan=None, nbytes=None):
        ms, wall = time_calls(self.torch, self.stream, self.entry(fn, plan), self.refill, K, W)
        med = statistics.median(ms)
        out = {"ms_per_step": med, "ms_mean": statistics.fmean(ms), "ms_min": min(ms), "ms_max": max(ms),
               "GBs_per_virtual_learner": 4 * self.count / (med * 1e-3) / 1e9,
               "wall_s_with_refills": round(wall, 4)}
        if nbytes:
            out["bytes"] = nbytes
            out["achieved_GBs"], out["frac"] = rate(nbytes, med)
        return out

    def identical(self, i):
        last = self.sets[i % len(self.sets)]
        t = self.torch
        return all(t.equal(last[0].view(t.int32), last[j].view(t.int32)) for j in range(1, self.P))

    def tensor_plan(self):
        I = self.I
        shapes = I.resnet50_shapes() if self.count == I.RESNET50_COUNT else (
            I.resnet101_22k_shapes() if self.count == I.RESNET101_22K_COUNT else None)
        if shapes is None:
            return None, 0
        offs, cnts = I.tensor_segments(shapes)
        tplan = self.D.ddl_ring_plan_tensors(self.dims, self.P, offs, cnts, self.count)
        self.D.ddl_plan_prepare(tplan)
        return tplan, len(offs)

    def close(self):
        self.sets, self.ptrs, self.plan = [], [], None
        self.torch.cuda.empty_cache()


def kernel_roofline(w, passes):
    """Average launch duration of the reduce-add and copy kernels: one event pair round each
    half of the allreduce, so gaps between the launches are in, event overhead is not."""
    D = w.D
    nsteps = D.ddl_plan_num_steps(w.plan)
    kinds = [D.ddl_plan_get_step(w.plan, s)[0] for s in range(nsteps)]
    step_bytes = [D.ddl_plan_step_bytes(w.plan, s) for s in range(nsteps)]
    acc_ms = {D.DDL_STEP_REDUCE: 0.0, D.DDL_STEP_GATHER: 0.0}
    acc_bytes = {D.DDL_STEP_REDUCE: 0, D.DDL_STEP_GATHER: 0}
    launches = {D.DDL_STEP_REDUCE: 0, D.DDL_STEP_GATHER: 0}
    for p in range(passes):
        w.refill(7000 + p)
        r_ms, g_ms = D.ddl_allreduce_sim_timed(w.ptrs[(7000 + p) % len(w.sets)], w.P, w.plan, w.count,
                                               D.DDL_F32, w.stream)
        acc_ms[D.DDL_STEP_REDUCE] += r_ms
        acc_ms[D.DDL_STEP_GATHER] += g_ms
        for s in range(nsteps):
            if step_bytes[s]:
                acc_bytes[kinds[s]] += step_bytes[s]
                launches[kinds[s]] += 1

    def line(kind, name):
        if not launches[kind]:
            return None
        gbs = acc_bytes[kind] / (acc_ms[kind] * 1e-3) / 1e9
        return {"kernel": name, "launches": launches[kind], "avg_launch_us": 1e3 * acc_ms[kind] / launches[kind],
                "avg_launch_bytes": acc_bytes[kind] / launches[kind], "achieved_GBs": gbs,
                "frac": gbs / HBM_PEAK_GBS}

    return (line(D.DDL_STEP_REDUCE, "reduce_add_step (step_kernel<float,true>)"),
            line(D.DDL_STEP_GATHER, "copy_step (step_kernel<float,false>)"))


def secondary(torch, D, I, dev, cfg, K, W, budget_bytes):
    """A configuration other than the headline one: the schedule, the step-fused variant and,
    where the buffer is a layer list, the per-tensor variant, and the ring-walk form (one
    launch per dimension); small ones also back to back."""
    resident = 4 * cfg["count"] * cfg["P"]
    w = Workload(torch, D, I, dev, cfg, 2 if 2 * resident <= budget_bytes else 1)
    out = {"workload": cfg["name"], "P": w.P, "dims": w.dims, "count": w.count,
           "phases": D.ddl_plan_num_steps(w.plan)}
    sched_bytes = D.ddl_plan_bytes_moved(w.plan)
    D.ddl_plan_set_walk(w.plan, D.DDL_WALK_OFF)
    out["schedule"] = w.measure(D.ddl_allreduce_sim, K, W, nbytes=sched_bytes)
    out["learners_identical"] = bool(w.identical(W + K - 1))
    D.ddl_plan_set_walk(w.plan, D.DDL_WALK_ON)
    out["ring_walk_variant"] = w.measure(D.ddl_allreduce_sim, K, W, nbytes=D.ddl_plan_walk_bytes(w.plan))
    out["learners_identical"] = out["learners_identical"] and bool(w.identical(W + K - 1))
    if sched_bytes / max(out["phases"], 1) < (64 << 20):
        # back to back, no refills and no events between the calls: the launch-bound rate
        n = 200
        call = w.entry(D.ddl_allreduce_sim)
        for mode, key in ((D.DDL_WALK_OFF, "phases"), (D.DDL_WALK_ON, "ring_walk")):
            D.ddl_plan_set_walk(w.plan, mode)
            for b in w.sets[0]:
                b.zero_()
            call(0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                call(0)
            torch.cuda.synchronize()
            out.setdefault("back_to_back_us", {})[key] = round((time.perf_counter() - t0) / n * 1e6, 2)
    D.ddl_plan_set_walk(w.plan, D.DDL_WALK_AUTO)
    try:
        out["fused_variant"] = w.measure(D.ddl_allreduce_fused_sim, K, W, nbytes=D.ddl_plan_fused_bytes(w.plan))
    except D.DdlError as e:
        out["fused_variant"] = {"error": str(e)}
    if "layers" in cfg["name"]:
        tplan, ntens = w.tensor_plan()
        if tplan is not None:
            D.ddl_plan_set_walk(tplan, D.DDL_WALK_OFF)
            out["per_tensor_variant"] = w.measure(D.ddl_allreduce_sim, K, W, plan=tplan,
                                                  nbytes=D.ddl_plan_bytes_moved(tplan))
            out["per_tensor_variant"]["tensors"] = ntens
            if D.ddl_plan_walk_bytes(tplan):
                D.ddl_plan_set_walk(tplan, D.DDL_WALK_ON)
                out["per_tensor_variant"]["ring_walk"] = w.measure(D.ddl_allreduce_sim, K, W, plan=tplan,
                                                                   nbytes=D.ddl_plan_walk_bytes(tplan))
    w.close()
    return out


def other_dtypes(torch, D, dev, cfg, K, W):
    """The same kernels through the other element traits (16-, 32- and 64-bit), at one
    configuration's shape; values are drawn by torch before every step, outside the events."""
    P, dims, count = cfg["P"], cfg["dims"], cfg["count"]
    stream = torch.cuda.current_stream()
    out = []
    for name, ddl, tdt in (("f64", D.DDL_F64, torch.float64), ("f16", D.DDL_F16, torch.float16),
                           ("bf16", D.DDL_BF16, torch.bfloat16), ("i32", D.DDL_I32, torch.int32)):
        bufs = [torch.empty(count, dtype=tdt, device=dev) for _ in range(P)]
        ptrs = D.pointer_array(bufs)
        plan = D.ddl_ring_plan(dims, P, count, ddl)
        D.ddl_plan_prepare(plan)
        D.ddl_plan_set_walk(plan, D.DDL_WALK_OFF)

        def refill(i):
            for b in bufs:
                b.random_(-100, 100) if tdt == torch.int32 else b.normal_(0.0, 0.01)

        ms, _ = time_calls(torch, stream, lambda i: D.ddl_allreduce_sim(ptrs, P, plan, count, ddl, stream), refill, K, W)
        med = statistics.median(ms)
        nbytes = D.ddl_plan_bytes_moved(plan)
        gbs, frac = rate(nbytes, med)
        out.append({"dtype": name, "ms_per_step": med, "bytes": nbytes, "achieved_GBs": gbs, "frac": frac,
                    "GBs_per_virtual_learner": count * bufs[0].element_size() / (med * 1e-3) / 1e9})
        del bufs, ptrs, plan
        torch.cuda.empty_cache()
    return {"workload": cfg["name"], "entry": "ddl_allreduce_sim, phase by phase", "results": out}


def overlap_with_compute(torch, D, I, dev, cfg, reps=10):
    """Sec. 5 notes that the Torch integration does not overlap communication with compute.
    Here: the gradient buffer cut into four buckets, each with its own plan, allreduced one
    after the other on a side stream while a dense matrix product (torch's, a stand-in for
    the backward pass of the next layers) runs on the main stream; against both alone."""
    P, dims, count = cfg["P"], cfg["dims"], cfg["count"]
    bufs = [torch.zeros(count, dtype=torch.float32, device=dev) for _ in range(P)]
    cuts = [count * k // 4 // 4 * 4 for k in range(4)] + [count]
    buckets = []
    for a, b in zip(cuts, cuts[1:]):
        plan = D.ddl_ring_plan(dims, P, b - a)
        D.ddl_plan_prepare(plan)
        D.ddl_plan_set_walk(plan, D.DDL_WALK_OFF)
        buckets.append((plan, D.pointer_array([x[a:b] for x in bufs]), b - a))
    n = 8192
    x = torch.randn(n, n, dtype=torch.bfloat16, device=dev)
    y = torch.randn(n, n, dtype=torch.bfloat16, device=dev)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()

    def allreduce(stream):
        for plan, ptrs, nb in buckets:
            D.ddl_allreduce_sim(ptrs, P, plan, nb, D.DDL_F32, stream)

    def timed(comm, compute):
        ms = []
        for _ in range(reps + 2):
            for b in bufs:
                b.zero_()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
            if comm:
                side.wait_event(e0)
                allreduce(side)
            if compute:
                torch.matmul(x, y)
            if comm:
                done = torch.cuda.Event()
                done.record(side)
                main.wait_event(done)
            e1.record(main)
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        return statistics.median(ms[2:])

    t_comm, t_comp, t_both = timed(True, False), timed(False, True), timed(True, True)
    return {"workload": cfg["name"], "buckets": 4, "compute": f"bf16 matmul {n}x{n}x{n} (torch)",
            "allreduce_alone_ms": t_comm, "compute_alone_ms": t_comp, "both_ms": t_both,
            "overlap": (t_comm + t_comp - t_both) / min(t_comm, t_comp)}


def box_sweep(torch, D, dev, P=256, iters=30, counts=(4096, 65536, 1 << 20), boxes=None):
    """Sec. 4.3: a ring's time has a latency term per phase, so for many learners a box with
    fewer phases wins although it moves the same bytes.  On one GPU the latency of a phase
    is a kernel-launch boundary.  Times every box on several buffer sizes, fits
    T = phases * L + bytes / B by least squares and asks ddl_choose_dims with the fit."""
    import numpy as np

    boxes = boxes or [[256], [16, 16], [4, 64], [64, 4], [4, 8, 8], [4, 4, 4, 4], [2] * 8]
    stream = torch.cuda.current_stream()
    rows = []
    for count in counts:
        bufs = [torch.zeros(count, dtype=torch.float32, device=dev) for _ in range(P)]
        ptrs = D.pointer_array(bufs)
        for dims in boxes:
            plan = D.ddl_ring_plan(dims, P, count)
            D.ddl_plan_prepare(plan)
            us = {}
            for mode, key in ((D.DDL_WALK_OFF, "us"), (D.DDL_WALK_ON, "us_ring_walk")):
                D.ddl_plan_set_walk(plan, mode)
                for _ in range(3):
                    D.ddl_allreduce_sim(ptrs, P, plan, count, D.DDL_F32, stream)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(iters):
                    D.ddl_allreduce_sim(ptrs, P, plan, count, D.DDL_F32, stream)
                torch.cuda.synchronize()
                us[key] = round((time.perf_counter() - t0) / iters * 1e6, 1)
            rows.append(dict(count=count, dims=dims, phases=D.ddl_plan_num_steps(plan),
                             bytes=D.ddl_plan_bytes_moved(plan), **us))
        del bufs, ptrs
    A = np.array([[r["phases"], r["bytes"]] for r in rows], dtype=np.float64)
    y = np.array([r["us"] * 1e-6 for r in rows])
    (L, invB), *_ = np.linalg.lstsq(A, y, rcond=None)
    # The estimate charges S_t / (d_t * bw) per phase for ONE learner's transfer of 4-byte
    # elements; here a phase is P such transfers through one memory, each element costing 12
    # (reduce) or 8 (gather) bytes of traffic, 2.5 x 4 on average: bw = fitted rate / (2.5 P).
    link_bw = 1.0 / invB / 2.5 / P
    picks = {}
    for count in counts:
        dims, t = D.ddl_choose_dims(P, 4 * count, [link_bw] * 8, [float(L)] * 8)
        best = min((r for r in rows if r["count"] == count), key=lambda r: r["us"])
        mine = [r for r in rows if r["count"] == count and [d for d in r["dims"] if d > 1] == [d for d in dims if d > 1]]
        picks[str(count)] = {"chooser": [d for d in dims if d > 1], "modelled_us": round(t * 1e6, 1),
                             "chooser_measured_us": mine[0]["us"] if mine else None,
                             "fastest_measured": best["dims"], "fastest_us": best["us"]}
    return {"P": P, "iters": iters, "results": rows,
            "fit": {"latency_per_phase_us": round(L * 1e6, 3), "bandwidth_GBs": round(1e-9 / invB, 1),
                    "note": "the chooser's per-link bandwidth is the fitted rate / (2.5 P): the model counts 4 "
                            "bytes per element of one learner's transfer, a phase here is P transfers at 12 or 8"},
            "chooser": picks}


def cpu_baseline(I, cfg, budget_s=30.0):
    """The oracle's step simulator as it stands, on the host, on a bounded sample."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import allreduce_steps  # the CPU baseline leg: the only use of the oracle here

    P, dims, count, dist, seed = cfg["P"], cfg["dims"], cfg["count"], cfg["dist"], cfg["seed"]
    c_count = count if 4 * count * P <= 8 * 2 ** 30 else count // 16
    workers = max(1, min(16, os.cpu_count() or 1))
    with ThreadPoolExecutor(workers) as pool:   # input generation only; the oracle runs on one core
        V = list(pool.map(lambda j: I.fill_host(c_count, seed, j, dist), range(P)))
    times = []
    t_start = time.perf_counter()
    while len(times) < 5 and time.perf_counter() - t_start < budget_s:
        t0 = time.perf_counter()
        allreduce_steps(V, dims)
        times.append(time.perf_counter() - t0)
    c_s = sorted(times)[len(times) // 2]
    cpu = {"value": 4 * c_count / c_s / 1e9, "unit": "GB/s per virtual learner", "cores": 1, "kind": "oracle",
           "sample": f"numpy step simulator, P={P} dims={dims}, {c_count} of {count} elements per learner "
                     f"(throughput does not depend on the length once out of cache), median of {len(times)} "
                     f"passes, {c_s:.2f} s per pass",
           "hbm_equivalent_GBs": 20 * c_count * (P - 1) / c_s / 1e9,
           "host_cores_available": os.cpu_count()}
    # second figure: the same oracle on slabs of the element range, one slab per host core
    # (the path is element-wise independent; numpy releases the GIL)
    cuts = [c_count * k // workers // 4 * 4 for k in range(workers)] + [c_count]
    slabs = [[v[a:b] for v in V] for a, b in zip(cuts, cuts[1:])]
    with ThreadPoolExecutor(workers) as pool:
        t0 = time.perf_counter()
        list(pool.map(lambda sl: allreduce_steps(sl, dims), slabs))
        a_s = time.perf_counter() - t0
    cpu["all_cores"] = {"value": 4 * c_count / a_s / 1e9, "unit": "GB/s per virtual learner", "cores": workers,
                        "kind": "oracle on element slabs, one thread per slab", "seconds": round(a_s, 3)}
    return cpu


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="1-based index into the five configurations")
    ap.add_argument("--dims", type=str, default=None, help="ad-hoc box, e.g. 4,8,8 (instead of --config)")
    ap.add_argument("--P", type=int, default=None, help="learners of the ad-hoc box (must equal the product of --dims)")
    ap.add_argument("--count", type=int, default=1 << 20, help="elements per learner of the ad-hoc shape")
    ap.add_argument("--seed", type=int, default=None, help="generator seed (default: the configuration's)")
    ap.add_argument("--dist", choices=["int8", "uniform", "normal"], default=None)
    ap.add_argument("--sets-gib", type=float, default=200.0, help="HBM budget for the input sets (two if they fit)")
    ap.add_argument("--profile-passes", type=int, default=10)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-others", action="store_true", help="skip the secondary configurations and the box sweep")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a dispatch of "
                         "known size, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--box-sweep", action="store_true",
                    help="instead of the benchmark line: time P=256 learners arranged as different boxes "
                         "on small buffers (the latency regime the multi-dimensional ring is for)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build simulates the collective inside ONE GPU; "
              "there is no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1708_02188_amd as D
    from paper_1708_02188_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    props = torch.cuda.get_device_properties(0)
    try:
        mem_khz, bus_bits = D.ddl_device_memory_info()
    except D.DdlError:
        mem_khz, bus_bits = None, None
    device_info = {"name": props.name, "memory_clock_khz": mem_khz, "memory_bus_bits": bus_bits,
                   "peak_used_GBs": HBM_PEAK_GBS, "hbm_bytes": props.total_memory,
                   "compute_units": props.multi_processor_count}
    if args.box_sweep:
        print(json.dumps(dict(mode="box_sweep", **box_sweep(torch, D, dev))))
        return

    if args.dims:
        dims = [int(x) for x in args.dims.split(",")]
        P = args.P if args.P is not None else prod(dims)
        dist = args.dist or "uniform"
        cfg = dict(name=f"adhoc_box{'x'.join(map(str, dims))}_count{args.count}_{dist}", P=P, dims=dims,
                   count=args.count, dist=dist, seed=args.seed if args.seed is not None else I.BASE_SEED)
    else:
        cfg = dict(I.CONFIGS[args.config - 1])
        if args.seed is not None:
            cfg["seed"] = args.seed
        if args.dist is not None:
            cfg["dist"] = args.dist
    K, W = args.steps, args.warmup
    budget = int(args.sets_gib * 2 ** 30)
    resident = 4 * cfg["count"] * cfg["P"]
    w = Workload(torch, D, I, dev, cfg, 2 if 2 * resident <= budget else 1)
    P, dims, count = w.P, w.dims, w.count
    nsteps = D.ddl_plan_num_steps(w.plan)
    bytes_total = D.ddl_plan_bytes_moved(w.plan)

    # the schedule itself, phase by phase: `value`
    D.ddl_plan_set_walk(w.plan, D.DDL_WALK_OFF)
    head = w.measure(D.ddl_allreduce_sim, K, W, nbytes=bytes_total)
    same = w.identical(W + K - 1)
    # The same schedule with every dimension's phases walked in one launch: identical buffers,
    # fewer bytes and launches; rated against its own bytes, reported beside `value`.
    walk = None
    if D.ddl_plan_walk_bytes(w.plan):
        D.ddl_plan_set_walk(w.plan, D.DDL_WALK_ON)
        walk = dict(entry="ddl_allreduce_sim with ddl_plan_set_walk(DDL_WALK_ON)",
                    **w.measure(D.ddl_allreduce_sim, K, W, nbytes=D.ddl_plan_walk_bytes(w.plan)))
        walk["speedup_vs_phases"] = head["ms_per_step"] / walk["ms_per_step"]
        same = same and w.identical(W + K - 1)
        D.ddl_plan_set_walk(w.plan, D.DDL_WALK_OFF)
    ms_per_step = head["ms_per_step"]
    per_learner_gbs = head["GBs_per_virtual_learner"]

    # The step-fused variant of the same allreduce, rated against its own byte count;
    # reported beside the schedule's figures, never as `value`.
    try:
        fused = dict(entry="ddl_allreduce_fused_sim",
                     **w.measure(D.ddl_allreduce_fused_sim, K, W, nbytes=D.ddl_plan_fused_bytes(w.plan)))
        fused["speedup_vs_schedule"] = ms_per_step / fused["ms_per_step"]
    except D.DdlError as e:
        fused = {"entry": "ddl_allreduce_fused_sim", "error": str(e)}

    # Per-tensor mode (each layer's tensor reduced on its own, all transfers of a phase in
    # one launch) where the buffer has a network's size; rated against its own schedule's bytes.
    per_tensor = None
    tplan, ntens = w.tensor_plan()
    if tplan is not None:
        D.ddl_plan_set_walk(tplan, D.DDL_WALK_OFF)
        per_tensor = dict(entry="ddl_ring_plan_tensors + ddl_allreduce_sim", tensors=ntens,
                          **w.measure(D.ddl_allreduce_sim, K, W, plan=tplan, nbytes=D.ddl_plan_bytes_moved(tplan)))
        per_tensor["slowdown_vs_one_buffer"] = per_tensor["ms_per_step"] / ms_per_step
        if D.ddl_plan_walk_bytes(tplan):
            D.ddl_plan_set_walk(tplan, D.DDL_WALK_ON)
            per_tensor["ring_walk"] = w.measure(D.ddl_allreduce_sim, K, W, plan=tplan,
                                                nbytes=D.ddl_plan_walk_bytes(tplan))
        del tplan

    red, cpy = kernel_roofline(w, args.profile_passes) if args.profile_passes else (None, None)
    per_step_ms = []
    if args.profile_passes:   # diagnostic only: an event pair round every launch adds a few us each
        w.refill(9999)
        per_step_ms = D.ddl_allreduce_sim_profile(w.ptrs[9999 % len(w.sets)], P, w.plan, count, D.DDL_F32, w.stream)
    recorded = RECORDED_TRAFFIC.get(cfg["name"])
    roofline = {"bound": "hbm", "kernel": red["kernel"] if red else None,
                "achieved": red["achieved_GBs"] if red else None, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": red["frac"] if red else None,
                "traffic": recorded["bytes_per_launch"] if recorded else None,
                "traffic_source": recorded["source"] if recorded else
                "none recorded for this workload (counter runs need rocprofv3 around the process)",
                "bytes_per_element": {"reduce_add_step": 12, "copy_step": 8},
                "avg_launch_us": red["avg_launch_us"] if red else None,
                "avg_launch_bytes": red["avg_launch_bytes"] if red else None,
                "copy_step": cpy,
                "whole_allreduce": {"achieved": head["achieved_GBs"], "frac": head["frac"], "bytes": bytes_total},
                "per_step_us": [round(1e3 * x, 2) for x in per_step_ms]}
    n_sets = len(w.sets)
    w.close()

    # context: a plain 1 GiB device-to-device copy by the HIP runtime (what torch's copy_ calls)
    # and by ddl_assign_sim, the all-gather phase's kernel on one range
    copies = None
    if not args.no_others:
        a = torch.zeros(2 ** 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        stream = torch.cuda.current_stream()
        ms_rt, _ = time_calls(torch, stream, lambda i: b.copy_(a), lambda i: None, 10, 2)
        ms_as, _ = time_calls(torch, stream, lambda i: D.ddl_assign_sim(b, a, a.numel(), D.DDL_F32, stream),
                              lambda i: None, 10, 2)
        copies = {"bytes_read_plus_written": 2 ** 31,
                  "hip_runtime_copy_GBs": 2 ** 31 / (statistics.median(ms_rt) * 1e-3) / 1e9,
                  "ddl_assign_sim_GBs": 2 ** 31 / (statistics.median(ms_as) * 1e-3) / 1e9}
        del a, b
        torch.cuda.empty_cache()

    if args.calib_copy_mib > 0:
        a = torch.zeros(args.calib_copy_mib * 2 ** 18, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    others, fit, dtypes, overlap = None, None, None, None
    if not args.no_others:
        others = [secondary(torch, D, I, dev, c, K, W, budget) for c in I.CONFIGS if c["name"] != cfg["name"]]
        dtypes = other_dtypes(torch, D, dev, I.CONFIGS[1], K, W)
        overlap = overlap_with_compute(torch, D, I, dev, I.CONFIGS[1])
        sweep = box_sweep(torch, D, dev, P=256, iters=20, counts=(4096, 262144),
                          boxes=[[256], [16, 16], [4, 8, 8], [2] * 8])
        fit = {"latency_per_phase_us": sweep["fit"]["latency_per_phase_us"],
               "bandwidth_GBs": sweep["fit"]["bandwidth_GBs"], "chooser": sweep["chooser"],
               "what": "T = phases * L + schedule bytes / B fitted over 4 boxes of 256 learners x 2 sizes, "
                       "phases launched kernel by kernel (Sec. 4.3's latency term = a launch boundary)"}

    cpu = None if args.no_cpu else cpu_baseline(I, cfg)

    out = {
        "metric": "allreduce GB/s per virtual learner + achieved HBM GB/s (% of peak)",
        "value": per_learner_gbs,
        "unit": "GB/s per virtual learner",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg["name"], "P": P, "dims": dims, "count": count, "dist": cfg["dist"],
                   "seed": cfg["seed"], "phases": nsteps, "resident_bytes": resident,
                   "input_sets": n_sets, "refilled_before_every_step": True,
                   "bus_GBs_per_learner": per_learner_gbs * 2 * (P - 1) / P},
        "timing": {"method": "one HIP-event pair per step on the launch stream; ms_per_step = median of the steps",
                   "ms_mean": head["ms_mean"], "ms_min": head["ms_min"], "ms_max": head["ms_max"],
                   "wall_s_with_refills": head["wall_s_with_refills"]},
        "hbm_GBs": head["achieved_GBs"], "hbm_frac_of_peak": head["frac"],
        "learners_identical": bool(same),
        "device": device_info,
        "roofline": roofline,
        "ring_walk_variant": walk,
        "fused_variant": fused,
        "per_tensor_variant": per_tensor,
        "other_configs": others,
        "other_dtypes": dtypes,
        "overlap_with_compute": overlap,
        "plain_copy_1GiB": copies,
        "latency_fit": fit,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    if not same:
        sys.exit(1)


if __name__ == "__main__":
    main()
