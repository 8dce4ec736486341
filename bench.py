#!/usr/bin/env python3
"""Benchmark of the simulated multi-ring allreduce on one MI355X.

A step is one whole allreduce (every reduce-scatter and all-gather phase of the schedule)
over one set of P synthetic learner buffers that is already resident in HBM.  Prints ONE
JSON line: allreduce GB/s per virtual learner (`value`), the HBM roofline of the dominant
kernel measured with HIP events round every phase, and the CPU oracle timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def box_sweep(torch, D, dev, P=256, iters=30):
    """Sec. 4.3: a ring's time has a latency term per phase, so for many learners a box with
    fewer phases wins although it moves the same bytes.  On one GPU the latency of a phase
    is a kernel-launch boundary.  Times every box on three buffer sizes, fits
    T = phases * L + bytes / B by least squares and asks ddl_choose_dims with the fit."""
    import numpy as np

    boxes = [[256], [16, 16], [4, 64], [64, 4], [4, 8, 8], [4, 4, 4, 4], [2] * 8]
    stream = torch.cuda.current_stream()
    rows = []
    for count in (4096, 65536, 1 << 20):
        bufs = [torch.zeros(count, dtype=torch.float32, device=dev) for _ in range(P)]
        for dims in boxes:
            plan = D.ddl_ring_plan(dims, P, count)
            D.ddl_plan_prepare(plan)
            for _ in range(3):
                D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(iters):
                D.ddl_allreduce_sim(bufs, P, plan, count, D.DDL_F32, stream)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) / iters * 1e6
            rows.append({"count": count, "dims": dims, "phases": D.ddl_plan_num_steps(plan),
                         "bytes": D.ddl_plan_bytes_moved(plan), "us": round(us, 1)})
        del bufs
    A = np.array([[r["phases"], r["bytes"]] for r in rows], dtype=np.float64)
    y = np.array([r["us"] * 1e-6 for r in rows])
    (L, invB), *_ = np.linalg.lstsq(A, y, rcond=None)
    picks = {}
    for count in (4096, 65536, 1 << 20):
        dims, t = D.ddl_choose_dims(P, 4 * count, [1.0 / invB / 2.5] * 8, [float(L)] * 8)
        best = min((r for r in rows if r["count"] == count), key=lambda r: r["us"])
        picks[str(count)] = {"chooser": [d for d in dims if d > 1], "modelled_us": round(t * 1e6, 1),
                             "fastest_measured": best["dims"], "fastest_us": best["us"]}
    print(json.dumps({"mode": "box_sweep", "P": P, "iters": iters, "results": rows,
                      "fit": {"latency_per_phase_us": round(L * 1e6, 3), "bandwidth_GBs": round(1e-9 / invB, 1),
                              "note": "the chooser's per-link bandwidth is the fitted rate / 2.5: the model "
                                      "counts 4 bytes per element and transfer, the kernels move 12 or 8"},
                      "chooser": picks}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="1-based index into the five configurations")
    ap.add_argument("--sets-gib", type=float, default=96.0,
                    help="HBM budget for distinct input sets (one per step until it is used up)")
    ap.add_argument("--profile-passes", type=int, default=10)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-fused", action="store_true", help="skip timing the step-fused variant")
    ap.add_argument("--per-tensor", action="store_true",
                    help="also time the per-tensor mode (always done for the per-layer configuration)")
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
        box_sweep(torch, D, dev)
        return
    cfg = I.CONFIGS[args.config - 1]
    P, dims, count, dist, seed = cfg["P"], cfg["dims"], cfg["count"], cfg["dist"], cfg["seed"]
    K, W = args.steps, args.warmup
    plan = D.ddl_ring_plan(dims, P, count)
    D.ddl_plan_prepare(plan)
    nsteps = D.ddl_plan_num_steps(plan)
    bytes_total = D.ddl_plan_bytes_moved(plan)
    resident = 4 * count * P

    # Distinct, freshly seeded input sets, so repeated in-place sums neither overflow nor
    # find the previous step's data in the caches.  If the budget is smaller than K+W sets
    # the sets are reused round-robin (values grow by a factor P per reuse, timing is
    # value-independent).
    n_sets = max(1, min(K + W, int(args.sets_gib * 2 ** 30 // resident)))
    stream = torch.cuda.current_stream()
    sets = []
    for s in range(n_sets):
        bufs = [torch.empty(count, dtype=torch.float32, device=dev) for _ in range(P)]
        for j, b in enumerate(bufs):
            I.fill_device(b, seed + 1000 * s, j, dist, 0, stream)
        sets.append(bufs)
    torch.cuda.synchronize()

    def run(i):
        D.ddl_allreduce_sim(sets[i % n_sets], P, plan, count, D.DDL_F32, stream)

    for i in range(W):
        run(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(W, W + K):
        run(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / K
    per_learner_gbs = 4 * count / (ms_per_step * 1e-3) / 1e9
    hbm_gbs = bytes_total / (ms_per_step * 1e-3) / 1e9

    # The step-fused variant of the same allreduce (one pass, 8*count*P bytes), rated
    # against its own byte count; reported beside the schedule's figures, never as `value`.
    fused = None
    if not args.no_fused:
        try:
            for i in range(W):
                D.ddl_allreduce_fused_sim(sets[i % n_sets], P, plan, count, D.DDL_F32, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(W, W + K):
                D.ddl_allreduce_fused_sim(sets[i % n_sets], P, plan, count, D.DDL_F32, stream)
            torch.cuda.synchronize()
            f_ms = (time.perf_counter() - t0) * 1e3 / K
            f_bytes = D.ddl_plan_fused_bytes(plan)
            fused = {"entry": "ddl_allreduce_fused_sim", "ms_per_step": f_ms,
                     "GBs_per_virtual_learner": 4 * count / (f_ms * 1e-3) / 1e9,
                     "bytes": f_bytes, "achieved_GBs": f_bytes / (f_ms * 1e-3) / 1e9,
                     "frac": f_bytes / (f_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "speedup_vs_schedule": ms_per_step / f_ms}
        except D.DdlError as e:
            fused = {"entry": "ddl_allreduce_fused_sim", "error": str(e)}

    # Per-tensor mode (each layer's tensor reduced on its own, all transfers of a phase in
    # one launch): timed for the configuration that is defined as a per-layer tensor list,
    # or on request; rated against its own schedule's bytes.
    per_tensor = None
    if args.per_tensor or "layers" in cfg["name"]:
        shapes = I.resnet50_shapes() if count == I.RESNET50_COUNT else (
            I.resnet101_22k_shapes() if count == I.RESNET101_22K_COUNT else None)
        if shapes is not None:
            offs, cnts = I.tensor_segments(shapes)
            tplan = D.ddl_ring_plan_tensors(dims, P, offs, cnts, count)
            D.ddl_plan_prepare(tplan)
            for i in range(W):
                D.ddl_allreduce_sim(sets[i % n_sets], P, tplan, count, D.DDL_F32, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(W, W + K):
                D.ddl_allreduce_sim(sets[i % n_sets], P, tplan, count, D.DDL_F32, stream)
            torch.cuda.synchronize()
            t_ms = (time.perf_counter() - t0) * 1e3 / K
            t_bytes = D.ddl_plan_bytes_moved(tplan)
            per_tensor = {"entry": "ddl_ring_plan_tensors + ddl_allreduce_sim", "tensors": len(offs),
                          "ms_per_step": t_ms, "GBs_per_virtual_learner": 4 * count / (t_ms * 1e-3) / 1e9,
                          "bytes": t_bytes, "achieved_GBs": t_bytes / (t_ms * 1e-3) / 1e9,
                          "frac": t_bytes / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "slowdown_vs_one_buffer": t_ms / ms_per_step}
            del tplan

    # quick self-check on the last set used: every learner holds the same bits
    last = sets[(W + K - 1) % n_sets]
    same = all(torch.equal(last[0].view(torch.int32), last[j].view(torch.int32)) for j in range(1, P))

    # Roofline of the dominant kernel (the reduce-add phase kernel carries 12 of every 20
    # bytes): HIP events on the stream the kernels run on, one pair round each half of the
    # allreduce, so that the average launch duration includes kernel-to-kernel gaps but no
    # event overhead between launches.
    kinds = [D.ddl_plan_get_step(plan, s)[0] for s in range(nsteps)]
    step_bytes = [D.ddl_plan_step_bytes(plan, s) for s in range(nsteps)]
    acc_ms = {D.DDL_STEP_REDUCE: 0.0, D.DDL_STEP_GATHER: 0.0}
    acc_bytes = {D.DDL_STEP_REDUCE: 0, D.DDL_STEP_GATHER: 0}
    launches = {D.DDL_STEP_REDUCE: 0, D.DDL_STEP_GATHER: 0}
    for p in range(args.profile_passes):
        for j, b in enumerate(sets[p % n_sets]):
            I.fill_device(b, seed + 7777 + p, j, dist, 0, stream)
        r_ms, g_ms = D.ddl_allreduce_sim_timed(sets[p % n_sets], P, plan, count, D.DDL_F32, stream)
        acc_ms[D.DDL_STEP_REDUCE] += r_ms
        acc_ms[D.DDL_STEP_GATHER] += g_ms
        for s in range(nsteps):
            if step_bytes[s]:
                acc_bytes[kinds[s]] += step_bytes[s]
                launches[kinds[s]] += 1
    # per-phase times (diagnostic only: an event pair round every launch adds a few us each)
    per_step_ms = [0.0] * nsteps
    if args.profile_passes:
        for j, b in enumerate(sets[0]):
            I.fill_device(b, seed + 9999, j, dist, 0, stream)
        per_step_ms = D.ddl_allreduce_sim_profile(sets[0], P, plan, count, D.DDL_F32, stream)

    def kernel_line(kind, name):
        if not launches[kind]:
            return None
        gbs = acc_bytes[kind] / (acc_ms[kind] * 1e-3) / 1e9
        return {"kernel": name, "launches": launches[kind],
                "avg_launch_us": 1e3 * acc_ms[kind] / launches[kind],
                "avg_launch_bytes": acc_bytes[kind] / launches[kind],
                "achieved_GBs": gbs, "frac": gbs / HBM_PEAK_GBS}

    red = kernel_line(D.DDL_STEP_REDUCE, "reduce_add_step (step_kernel<float,true>)")
    cpy = kernel_line(D.DDL_STEP_GATHER, "copy_step (step_kernel<float,false>)")
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tfile):
        try:
            traffic = json.load(open(tfile)).get(cfg["name"])
        except (OSError, ValueError):
            traffic = None
    roofline = {"bound": "hbm", "kernel": red["kernel"] if red else None,
                "achieved": red["achieved_GBs"] if red else None, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": red["frac"] if red else None, "traffic": traffic,
                "bytes_per_element": {"reduce_add_step": 12, "copy_step": 8},
                "avg_launch_us": red["avg_launch_us"] if red else None,
                "avg_launch_bytes": red["avg_launch_bytes"] if red else None,
                "copy_step": cpy,
                "whole_allreduce": {"achieved": hbm_gbs, "frac": hbm_gbs / HBM_PEAK_GBS,
                                    "bytes": bytes_total},
                "per_step_us": [round(1e3 * x, 2) for x in per_step_ms]}

    del sets
    torch.cuda.empty_cache()

    if args.calib_copy_mib > 0:
        a = torch.zeros(args.calib_copy_mib * 2 ** 18, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    cpu = None
    if not args.no_cpu:
        from oracle import allreduce_steps  # the CPU baseline leg: the oracle as it stands

        c_count = count if resident <= 8 * 2 ** 30 else count // 16
        V = [I.fill_host(c_count, seed, j, dist) for j in range(P)]
        times = []
        t_start = time.perf_counter()
        while len(times) < 5 and time.perf_counter() - t_start < 30.0:   # bounded: at most ~30 s
            t0 = time.perf_counter()
            allreduce_steps(V, dims)
            times.append(time.perf_counter() - t0)
        c_s = sorted(times)[len(times) // 2]
        cpu = {"value": 4 * c_count / c_s / 1e9, "unit": "GB/s per virtual learner", "cores": 1,
               "kind": "oracle",
               "sample": f"numpy step simulator, P={P} dims={dims}, {c_count} of {count} elements per "
                         f"learner, median of {len(times)} passes, {c_s:.2f} s per pass",
               "hbm_equivalent_GBs": 20 * c_count * (P - 1) / c_s / 1e9,
               "host_cores_available": os.cpu_count()}
        # optional second figure: the same oracle on slabs of the element range, one slab per
        # host core (the path is element-wise independent; numpy releases the GIL)
        from concurrent.futures import ThreadPoolExecutor
        workers = max(1, min(16, os.cpu_count() or 1))
        cuts = [c_count * w // workers // 4 * 4 for w in range(workers)] + [c_count]
        slabs = [[v[a:b] for v in V] for a, b in zip(cuts, cuts[1:])]
        with ThreadPoolExecutor(workers) as pool:
            t0 = time.perf_counter()
            list(pool.map(lambda sl: allreduce_steps(sl, dims), slabs))
            a_s = time.perf_counter() - t0
        cpu["all_cores"] = {"value": 4 * c_count / a_s / 1e9, "unit": "GB/s per virtual learner",
                            "cores": workers, "kind": "oracle on element slabs, one thread per slab",
                            "seconds": round(a_s, 3)}

    out = {
        "metric": "allreduce GB/s per virtual learner + achieved HBM GB/s (% of peak)",
        "value": per_learner_gbs,
        "unit": "GB/s per virtual learner",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg["name"], "P": P, "dims": dims, "count": count, "dist": dist,
                   "seed": seed, "phases": nsteps, "resident_bytes": resident,
                   "input_sets": n_sets, "bus_GBs_per_learner": per_learner_gbs * 2 * (P - 1) / P},
        "hbm_GBs": hbm_gbs, "hbm_frac_of_peak": hbm_gbs / HBM_PEAK_GBS,
        "learners_identical": bool(same),
        "device": device_info,
        "roofline": roofline,
        "fused_variant": fused,
        "per_tensor_variant": per_tensor,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    if not same:
        sys.exit(1)


if __name__ == "__main__":
    main()
