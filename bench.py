"""Benchmark of the batched plan evaluator on one MI355X.

A step is one pass of the whole hot path over the largest synthetic workload (the
OPT-30B-like cluster with 104 256 000 candidate plans): index decode, table gathers,
per-stage memory check, 1F1B makespan with transfers and gradient all-reduce, cost,
validity mask, and the selection of the 64 best plans for "max throughput under a
budget of 1.2 x the cheapest plan".  Inputs are resident on the device before timing.

Prints one JSON line: candidates/s over the timed steps, the roofline of the dominant
kernel (the full-space scan, timed with HIP events on its own stream inside the
library) and the CPU oracle timed on this host on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# nominal algorithmic work of one candidate: 12 fp32 operations per pipeline stage
# (stage time, two transfers, sum, max, all-reduce, update, price, egress) plus 15 for
# the epilogue, with P the mean pipeline depth over the candidate space
FLOPS_PER_STAGE, FLOPS_EPILOGUE = 12.0, 15.0
PEAK_FP32_VECTOR_TFLOPS = 157.3
# HBM bytes per scan launch on this workload from rocprofv3 FETCH_SIZE / WRITE_SIZE, each
# scaled by a 1 GiB copy of the same run (profiles/k_units_scan_cfg4_counters.md); set to
# None whenever k_units changes after the counters were taken (how many scan units are cut
# into parts depends on times measured at plan creation, so the figures move by a percent or
# two between runs)
SCAN_TRAFFIC_BYTES = 5.79e6
# VALU wave-instructions the scan executes per launch on this workload (SQ_INSTS_VALU, same
# file and same rule); each occupies one of the 1 024 SIMDs for 4 cycles at 2.4 GHz
SCAN_VALU_WAVE_INSTS = 1.081e7
SIMDS, CLOCK_HZ, CYCLES_PER_WAVE_INST = 1024, 2.4e9, 4
# steps of the timed region between two whose scan dispatch carries start / stop events
EVENT_EVERY = 8


def timed_steps(plan, step, steps, sync):
    """Wall time per step (ms) over `steps` calls of step(), and the mean duration (ms) of the
    scan kernel over the calls whose dispatch carried start / stop events: every
    EVENT_EVERY-th one.  A dispatch with events costs the step about 15 us (the runtime
    completes and timestamps it apart from its neighbours), so events on every launch would
    measure mostly that; the steps with events are part of the timed region."""
    scan_ms, n_timed, out = 0.0, 0, None
    sync()
    t0 = time.perf_counter()
    for i in range(steps):
        timed = i % EVENT_EVERY == 0
        plan.set_timing(1 if timed else 0)
        out = step()
        if timed:
            scan_ms += plan.last_timing()[1]
            n_timed += 1
    sync()
    wall = time.perf_counter() - t0
    plan.set_timing(0)
    return wall / steps * 1e3, scan_ms / n_timed, out


def mean_pipeline_depth(prob) -> float:
    """Block-size weighted mean of P over the candidate space (bookkeeping only)."""
    zg = prob.n_zones * prob.n_types
    inner = len(prob.mb_values) * len(prob.tp_values) * len(prob.dp_values) * zg
    tot = wsum = 0
    for ip, P in enumerate(int(x) for x in prob.pp_values):
        for s in (1, 2, 3):
            if s > prob.max_segments or s > P or (s == 3 and P > prob.seg3_max_pp):
                continue
            cuts = 1 if s == 1 else (P - 1 if s == 2 else (P - 1) * (P - 2) // 2)
            size = inner * cuts * (zg - 1) ** (s - 1) * int(prob.n_partitions[ip])
            tot += size
            wsum += size * P
    return wsum / tot


def cpu_baseline(prob, n_sample: int) -> dict:
    """The oracle as it stands, single thread, on uniformly drawn candidates."""
    import numpy as np
    from oracle.oracle import Oracle
    orc = Oracle(prob)
    n = orc.num_candidates
    idx = np.random.default_rng(12345).integers(0, n, n_sample).astype(np.uint64)
    t0 = time.perf_counter()
    orc.eval_batch(indices=idx, n_threads=1)
    dt = time.perf_counter() - t0
    cores = os.cpu_count() or 1
    threads = min(cores, 16)
    t0 = time.perf_counter()
    orc.eval_batch(indices=idx, n_threads=threads)
    dt_mt = time.perf_counter() - t0
    return {"value": n_sample / dt, "unit": "candidates/s", "cores": 1, "kind": "oracle",
            "sample": f"{n_sample} uniformly drawn candidates of the same workload, fp64 C -O2, "
                      f"evaluation only ({dt:.1f} s)",
            "all_cores": {"value": n_sample / dt_mt, "threads": threads, "host_cores": cores}}


def sweep(torch, workloads, Plan, MAX_THROUGHPUT, MIN_COST) -> int:
    """Time to the 64 best plans (max throughput under 1.2 x the cheapest plan's cost) and to
    the best plan, per workload; inputs resident, 32 (top-64) and 30 (best plan) repetitions
    after 5 warm-up calls."""
    from paper_2504_17096_amd.binding import sailor_result
    stream = torch.cuda.current_stream().cuda_stream
    base = {"cfg1": workloads.config1(), "cfg2": workloads.config2(), "cfg3": workloads.config3(),
            "cfg4": workloads.config4()}
    cases = []
    for name, p in base.items():
        cases += [(name, p), (name + "+segment_tp", p.with_per_segment_tp()),
                  (name + "+mixed_types", p.with_mixed_types())]
    cases.append(("cfg3+link_profiles", base["cfg3"].with_bw_poly(workloads.bandwidth_poly(base["cfg3"]))))
    cases.append(("cfg4+segment_tp+mixed_types", base["cfg4"].with_per_segment_tp().with_mixed_types()))
    buf = (sailor_result * 64)()
    for name, p in cases:
        t0 = time.perf_counter()
        plan = Plan(p)
        create_ms = (time.perf_counter() - t0) * 1e3
        budget = 1.2 * plan.best_plan(objective=MIN_COST, stream=stream).cost_per_iter
        plan.set_timing(1)
        for _ in range(5):
            plan.topk_raw(64, MAX_THROUGHPUT, budget, buf, stream)
        top_ms, scan, found = timed_steps(
            plan, lambda: plan.topk_raw(64, MAX_THROUGHPUT, budget, buf, stream), 32,
            torch.cuda.synchronize)
        t0 = time.perf_counter()
        for _ in range(30):
            plan.best_plan(objective=MAX_THROUGHPUT, bound=budget, stream=stream)
        best_ms = (time.perf_counter() - t0) / 30 * 1e3
        n = plan.num_candidates()
        print(json.dumps({"workload": name, "candidates": n, "found": found, "plan_create_ms": create_ms,
                          "time_to_top64_ms": top_ms, "scan_kernel_ms": scan,
                          "time_to_best_plan_ms": best_ms, "candidates_per_s": n / (top_ms * 1e-3)}),
              flush=True)
        plan.destroy()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--cpu-sample", type=int, default=48_000_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: the top-64 query on every synthetic "
                         "workload and its widened variants, one JSON object per line")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy (calibrates FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be at least 1 and --warmup at least 0", file=sys.stderr)
        return 2
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding across GPUs); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2504_17096_amd import workloads
    from paper_2504_17096_amd.binding import MAX_THROUGHPUT, MIN_COST, Plan

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    if args.sweep:
        return sweep(torch, workloads, Plan, MAX_THROUGHPUT, MIN_COST)
    prob = workloads.config4()
    t0 = time.perf_counter()
    plan = Plan(prob)
    create_ms = (time.perf_counter() - t0) * 1e3
    n = plan.num_candidates()
    stream = torch.cuda.current_stream().cuda_stream
    K = 64

    # the budget of the timed query comes from a first pass on the device
    cheapest = plan.best_plan(objective=MIN_COST, stream=stream)
    budget = 1.2 * cheapest.cost_per_iter

    from paper_2504_17096_amd.binding import sailor_result
    buf = (sailor_result * K)()   # results are decoded by the library into this array

    def step():
        return plan.topk_raw(K, MAX_THROUGHPUT, budget, buf, stream)

    # start / stop events ride on the scan kernel's own dispatch in every EVENT_EVERY-th step
    # of the timed region (see timed_steps); those steps are part of `value`
    plan.set_timing(1)
    for _ in range(args.warmup):
        step()
    ms_per_step, scan_ms, n_found = timed_steps(plan, step, args.steps, torch.cuda.synchronize)
    assert n_found == K, n_found
    top1_index = int(buf[0].index)
    counts = plan.last_counts()

    # the selected plans' 1F1B schedules event by event, against the closed form the
    # evaluator uses for T_pp (outside the timed region)
    import numpy as np
    top_idx = np.array([int(buf[j].index) for j in range(K)], dtype=np.uint64)
    d_idx = torch.from_numpy(top_idx.view(np.int64)).to("cuda:0")
    d_ev = torch.empty(K, dtype=torch.float64, device="cuda:0")
    d_cl = torch.empty(K, dtype=torch.float64, device="cuda:0")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(3):
        e0.record()
        plan.simulate_1f1b(K, d_idx, d_ev, d_cl, stream)
        e1.record()
        torch.cuda.synchronize()
    gap = (d_cl / d_ev - 1.0).cpu().numpy()
    event_sched = {"plans": K, "ms": e0.elapsed_time(e1),
                   "closed_over_event_minus_1": {"min": float(gap.min()), "mean": float(gap.mean()),
                                                 "max": float(gap.max())}}

    # time-to-best-plan (single best plan, tolerance tie rule), outside the timed region
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 20
    for _ in range(reps):
        best = plan.best_plan(objective=MAX_THROUGHPUT, bound=budget, stream=stream)
    best_ms = (time.perf_counter() - t0) / reps * 1e3

    # per-candidate outputs for the whole space (20 B per candidate)
    tt = torch.empty(n, dtype=torch.float32, device="cuda:0")
    cc = torch.empty(n, dtype=torch.float32, device="cuda:0")
    mm = torch.empty(n, dtype=torch.int64, device="cuda:0")
    kk = torch.empty(n, dtype=torch.int32, device="cuda:0")
    eval_ms = 0.0
    plan.set_timing(1)
    for i in range(6):
        plan.eval_batch(0, n, objective=MAX_THROUGHPUT, bound=budget, d_time=tt, d_cost=cc,
                        d_mem=mm, d_mask=kk, stream=stream)
        torch.cuda.synchronize()
        if i:
            eval_ms += plan.last_timing()[1] / 5
    plan.set_timing(0)

    # availability stream: 64 snapshots of the 4-zone x 3-type cluster, a full re-plan
    # (6 791 040 candidates) at each: latency of set_avail + best_plan
    prob5 = workloads.config3()
    plan5 = Plan(prob5)
    lat = []
    for snap in workloads.config5_snapshots(prob5):
        t0 = time.perf_counter()
        plan5.set_avail(snap)
        plan5.best_plan(objective=MAX_THROUGHPUT, stream=stream)
        lat.append((time.perf_counter() - t0) * 1e3)
    n5 = plan5.num_candidates()
    plan5.destroy()
    replan = {"snapshots": len(lat), "candidates": n5, "p50_ms": float(np.percentile(lat, 50)),
              "p99_ms": float(np.percentile(lat, 99))}

    # the same query on the widened spaces: a TP digit per segment (915 206 400 candidates),
    # replicas of a stage split over two GPU types (5 zones x 10 extended types)
    def widened(problem, reps):
        p = Plan(problem)
        t0 = time.perf_counter()
        b = 1.2 * p.best_plan(objective=MIN_COST, stream=stream).cost_per_iter
        p.set_timing(1)
        for _ in range(2):
            p.topk_raw(K, MAX_THROUGHPUT, b, buf, stream)
        ms, scan, _ = timed_steps(p, lambda: p.topk_raw(K, MAX_THROUGHPUT, b, buf, stream), reps,
                                  torch.cuda.synchronize)
        out = {"candidates": p.num_candidates(), "time_to_top64_ms": ms, "scan_kernel_ms": scan,
               "candidates_per_s": p.num_candidates() / (ms * 1e-3)}
        p.destroy()
        return out

    segtp = widened(prob.with_per_segment_tp(), 16)
    mixed = widened(prob.with_mixed_types(), 16)

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    pbar = mean_pipeline_depth(prob)
    flops_per_cand = FLOPS_PER_STAGE * pbar + FLOPS_EPILOGUE
    achieved = flops_per_cand * n / (scan_ms * 1e-3) / 1e12
    valu = None
    if SCAN_VALU_WAVE_INSTS is not None:
        issue_ms = SCAN_VALU_WAVE_INSTS * CYCLES_PER_WAVE_INST / SIMDS / CLOCK_HZ * 1e3
        valu = {"wave_insts_per_launch": SCAN_VALU_WAVE_INSTS, "issue_ms": issue_ms,
                "frac_of_kernel_time": issue_ms / scan_ms}
    out = {
        "metric": "candidate plans evaluated/sec (full hot path incl. top-64 selection)",
        "value": n / (ms_per_step * 1e-3), "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg4: OPT-30B-like, 5 zones x 4 GPU types, 48 layers, "
                               "8 layer splits per pp, <=3 segments",
                   "candidates": n, "objective": "max throughput s.t. cost <= 1.2 x cheapest",
                   "top_k": K, "mean_pipeline_depth": pbar},
        "roofline": {"bound": "alu", "kernel": "k_units<SCAN>", "achieved": achieved,
                     "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_VECTOR_TFLOPS, "traffic": SCAN_TRAFFIC_BYTES,
                     "flops_per_candidate": flops_per_cand, "kernel_ms": scan_ms,
                     "valu_issue": valu},
        "extra": {"time_to_top64_ms": ms_per_step, "time_to_best_plan_ms": best_ms,
                  "scan_kernel_ms": scan_ms,
                  "eval_batch_ms": eval_ms,
                  "eval_batch_candidates_per_s": n / (eval_ms * 1e-3),
                  "eval_batch_output_GBps": 20.0 * n / (eval_ms * 1e-3) / 1e9,
                  "plan_create_ms": create_ms, "replan_stream": replan,
                  "per_segment_tp": segtp, "mixed_types": mixed, "event_schedule_top64": event_sched, "survivors_refined_valid": list(counts), "best_index": best.index,
                  "top1_index": top1_index},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(prob, args.cpu_sample)
    plan.destroy()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
