"""Benchmark of the batched plan evaluator on one MI355X.

A step is one pass of the whole hot path over the largest synthetic workload (the
OPT-30B-like cluster with 104 256 000 candidate plans): index decode, table gathers,
per-stage memory check, 1F1B makespan with transfers and gradient all-reduce, cost,
validity mask, and the selection of the 64 best plans for "max throughput under a
budget of 1.2 x the cheapest plan".  Inputs are resident on the device before timing;
every step decides the whole space (nothing is kept from one step to the next): pieces of
the space whose cost bound, computed once per plan, already exceeds the budget are ruled out
by one comparison each, the others are evaluated candidate by candidate.

Prints one JSON line: candidates/s over the timed steps; the roofline of the step's pass over
the space (its duration from HIP events on its own dispatch, its instruction counts from the
committed rocprofv3 counter summary, which is used only while the kernel sources still hash
to what the counters were taken on); the same for the scan of every piece under a budget that
never binds, and for a variant of the workload in which nearly every candidate is valid;
measured FMA and write ceilings; and the CPU oracle timed on this host for the same calls.
"""
from __future__ import annotations

import argparse
import hashlib
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
# vector ALU of the part: 256 compute units x 4 SIMDs x 16 lanes at 2.4 GHz issue 39.3 T
# lane-operations/s; an FMA counts two flops (78.6 TFLOP/s), the published 157.3 TFLOP/s
# needs packed FP32 instructions, which the library is compiled without
CUS, SIMDS_PER_CU, LANES_PER_SIMD, CLOCK_HZ = 256, 4, 16, 2.4e9
PEAK_LANE_OPS = CUS * SIMDS_PER_CU * LANES_PER_SIMD * CLOCK_HZ / 1e12   # T lane-ops/s
PEAK_FP32_FMA_TFLOPS, PEAK_FP32_PACKED_TFLOPS = 78.6, 157.3
PEAK_HBM_GBPS = 8000.0
# rocprofv3 counter summary of the kernels below, with the hash of the sources it was taken on
COUNTERS_JSON = os.path.join(ROOT, "profiles", "kernel_counters.json")
HASHED_SOURCES = ["paper_2504_17096_amd/csrc/sailor_kernels.hip.h",
                  "paper_2504_17096_amd/csrc/sailor_dev.h",
                  "paper_2504_17096_amd/csrc/sailor.hip"]
# steps of the timed region between two whose scan dispatch carries start / stop events
EVENT_EVERY = 8


def source_hash() -> str:
    h = hashlib.sha256()
    for rel in HASHED_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def load_counters():
    """(entries by name, note): the committed counter summary, or ({}, why not) when it is
    missing or was taken on other kernel sources than the ones built now."""
    if not os.path.exists(COUNTERS_JSON):
        return {}, "no counter summary committed"
    with open(COUNTERS_JSON) as f:
        doc = json.load(f)
    if doc.get("source_sha256") != source_hash():
        return {}, "kernel sources changed since the counters were taken"
    return doc.get("kernels", {}), "profiles/kernel_counters.json, sources unchanged"


def alu_roofline(entry, kernel_ms, nominal_flops):
    """Flat roofline keys of an ALU-bound kernel from its counters (per launch) and its
    duration in this run.  `achieved` counts every vector instruction as 64 lane-operations."""
    out = {"bound": "alu", "unit": "T lane-ops/s", "peak": PEAK_LANE_OPS, "kernel_ms": kernel_ms,
           "achieved": None, "frac": None, "traffic": None}
    if nominal_flops is not None:
        nominal = nominal_flops / (kernel_ms * 1e-3) / 1e12
        out["nominal_tflops"] = nominal  # per-stage definition's work / time: NOT a utilisation
        out["nominal_work_ratio"] = nominal / PEAK_FP32_PACKED_TFLOPS
    if not entry:
        return out
    c = entry["counters"]
    valu = c["SQ_INSTS_VALU"]
    out["achieved"] = valu * 64 / (kernel_ms * 1e-3) / 1e12
    out["frac"] = out["achieved"] / PEAK_LANE_OPS
    fp32_flops = (c["SQ_INSTS_VALU_ADD_F32"] + c["SQ_INSTS_VALU_MUL_F32"]
                  + 2 * c["SQ_INSTS_VALU_FMA_F32"]) * 64
    out["fp32_op_rate_tflops"] = fp32_flops / (kernel_ms * 1e-3) / 1e12
    out["fp32_frac_of_78_6"] = out["fp32_op_rate_tflops"] / PEAK_FP32_FMA_TFLOPS
    out["fp32_frac_of_157_3"] = out["fp32_op_rate_tflops"] / PEAK_FP32_PACKED_TFLOPS
    out["valu_insts_per_launch"] = valu
    out["int32_share_of_valu"] = c["SQ_INSTS_VALU_INT32"] / valu
    out["salu_per_valu"] = c["SQ_INSTS_SALU"] / valu
    out["lds_conflict_cycles_per_lds_inst"] = c["SQ_LDS_BANK_CONFLICT"] / max(1.0, c["SQ_INSTS_LDS"])
    out["traffic"] = entry.get("hbm_bytes")
    out["kernel_us_rocprof"] = entry.get("avg_duration_us")
    return out


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


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(prob, prob5, budget, k, n_sample: int, n_snapshots: int) -> dict:
    """The oracle as it stands on this host: the calls the GPU is timed on (the 64 best plans,
    the best plan and every candidate's outputs over the whole space; re-plans of an
    availability stream), sharded over the host's cores by index range, and its
    single-thread rate on a sample."""
    import numpy as np
    from oracle.oracle import MAX_THROUGHPUT, Oracle
    from paper_2504_17096_amd import workloads
    cores = os.cpu_count() or 1
    threads = min(cores, 16)
    orc = Oracle(prob)
    n = orc.num_candidates
    t0 = time.perf_counter()
    top = orc.topk(k, MAX_THROUGHPUT, budget, n_threads=threads)
    t_top = time.perf_counter() - t0
    t0 = time.perf_counter()
    best = orc.best(MAX_THROUGHPUT, budget, n_threads=threads)
    t_best = time.perf_counter() - t0
    t0 = time.perf_counter()
    outs = orc.eval_batch(objective=MAX_THROUGHPUT, bound=budget, n_threads=threads)
    t_eval = time.perf_counter() - t0
    del outs
    lat = []
    for snap in workloads.config5_snapshots(prob5)[:n_snapshots]:
        t0 = time.perf_counter()
        Oracle(prob5.with_avail(snap)).best(MAX_THROUGHPUT, n_threads=threads)
        lat.append(time.perf_counter() - t0)
    idx = np.random.default_rng(12345).integers(0, n, n_sample).astype(np.uint64)
    t0 = time.perf_counter()
    orc.eval_batch(indices=idx, n_threads=1)
    t_one = time.perf_counter() - t0
    return {"value": n / t_top, "unit": "candidates/s", "cores": threads, "kind": "oracle",
            "sample": f"the benchmark's own query (the {k} best plans, max throughput under the "
                      f"budget) over all {n} candidates, fp64 C -O2, {threads} threads by index "
                      f"range: {t_top:.2f} s",
            "cpu_model": cpu_model(), "host_cores": cores,
            "top64_s": t_top, "best_plan_s": t_best, "eval_batch_s": t_eval,
            "top1_index": top[0].index if top else None,
            "best_index": best.index if best else None,
            "replan_stream": {"snapshots": len(lat), "candidates": Oracle(prob5).num_candidates,
                              "p50_s": float(np.percentile(lat, 50)),
                              "p99_s": float(np.percentile(lat, 99))},
            "single_thread": {"candidates_per_s": n_sample / t_one,
                              "sample": f"{n_sample} uniformly drawn candidates, evaluation only "
                                        f"({t_one:.1f} s)"}}


def sweep(torch, workloads, Plan, MAX_THROUGHPUT, MIN_COST) -> int:
    """Time to the 64 best plans (max throughput under 1.2 x the cheapest plan's cost) and to
    the best plan, per workload; inputs resident, every call evaluates the whole space; 32
    (top-64) and 30 (best plan) repetitions after 5 warm-up calls."""
    from paper_2504_17096_amd.binding import sailor_result
    stream = torch.cuda.current_stream().cuda_stream
    base = {"cfg1": workloads.config1(), "cfg2": workloads.config2(), "cfg3": workloads.config3(),
            "cfg4": workloads.config4()}
    cases = []
    for name, p in base.items():
        cases += [(name, p), (name + "+segment_tp", p.with_per_segment_tp()),
                  (name + "+mixed_types", p.with_mixed_types())]
    cases.append(("cfg3+link_profiles", base["cfg3"].with_bw_poly(workloads.bandwidth_poly(base["cfg3"]))))
    cases.append(("cfg4_dense", workloads.config4_dense()))
    cases.append(("cfg4+segment_tp+mixed_types", base["cfg4"].with_per_segment_tp().with_mixed_types()))
    buf = (sailor_result * 64)()
    for name, p in cases:
        t0 = time.perf_counter()
        plan = Plan(p)
        create_ms = (time.perf_counter() - t0) * 1e3
        plan.set_incremental(False)
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


def replan_stream(np, Plan, prob, snapshots, stream, incremental):
    """Latency of set_avail + best_plan over an availability stream, and how many pieces of the
    space each re-plan evaluated again."""
    plan = Plan(prob)
    plan.set_incremental(incremental)
    plan.best_plan(stream=stream)  # the plan in force before the stream starts
    lat, evaluated = [], []
    for snap in snapshots:
        t0 = time.perf_counter()
        plan.set_avail(snap)
        plan.best_plan(stream=stream)
        lat.append((time.perf_counter() - t0) * 1e3)
        evaluated.append(plan.last_scan()[0])
    total = plan.last_scan()[1]
    plan.destroy()
    return {"p50_ms": float(np.percentile(lat, 50)), "p99_ms": float(np.percentile(lat, 99)),
            "units_total": total, "units_evaluated_mean": float(np.mean(evaluated)),
            "units_evaluated_per_snapshot": evaluated}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (a step takes about 0.04 ms; the first fifty-odd calls of a process run a quarter slower
    # while the HIP runtime grows its pools, hence the long default warm-up)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--cpu-sample", type=int, default=16_000_000)
    ap.add_argument("--cpu-snapshots", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: the top-64 query on every synthetic "
                         "workload and its widened variants, one JSON object per line")
    ap.add_argument("--only-kernels", action="store_true",
                    help="profiling runs: only the timed query, the whole-space evaluation and the "
                         "dense variant (the three kernels the counter summary covers)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy (calibrates FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be at least 1 and --warmup at least 0", file=sys.stderr)
        return 2
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no sharding across GPUs); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2504_17096_amd import microbench, workloads
    from paper_2504_17096_amd.binding import MAX_THROUGHPUT, MIN_COST, Plan, sailor_result

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    if args.sweep:
        return sweep(torch, workloads, Plan, MAX_THROUGHPUT, MIN_COST)
    prob = workloads.config4()
    t0 = time.perf_counter()
    plan = Plan(prob)
    create_ms = (time.perf_counter() - t0) * 1e3      # includes the start of the HIP runtime
    t0 = time.perf_counter()
    Plan(prob).destroy()
    create_warm_ms = (time.perf_counter() - t0) * 1e3  # the same problem once more
    plan.set_incremental(False)  # every timed call evaluates the whole space
    n = plan.num_candidates()
    stream = torch.cuda.current_stream().cuda_stream
    K = 64

    # the budget of the timed query comes from a first pass on the device
    cheapest = plan.best_plan(objective=MIN_COST, stream=stream)
    budget = 1.2 * cheapest.cost_per_iter
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
    units_evaluated, units_total = plan.last_scan()  # the rest fell to their cost bounds

    # the selected plans' 1F1B schedules event by event, against the closed form the
    # evaluator uses for T_pp (outside the timed region)
    top_idx = np.array([int(buf[j].index) for j in range(K)], dtype=np.uint64)
    d_idx = torch.from_numpy(top_idx.view(np.int64)).to("cuda:0")
    d_ev = torch.empty(K, dtype=torch.float64, device="cuda:0")
    d_cl = torch.empty(K, dtype=torch.float64, device="cuda:0")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(1 if args.only_kernels else 3):
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
    # (not in a counter run: its scan shares kernel and grid with the query below, whose
    # counters must stay apart)
    reps = 0 if args.only_kernels else 20
    best = None
    for _ in range(reps):
        best = plan.best_plan(objective=MAX_THROUGHPUT, bound=budget, stream=stream)
    best_ms = (time.perf_counter() - t0) / max(1, reps) * 1e3

    # the timed query once more with a budget that no plan exceeds: nothing falls to a cost
    # bound, only invalid plans are discarded (outside the timed region)
    unbound = None
    if True:
        for _ in range(3):
            plan.topk_raw(K, MAX_THROUGHPUT, 1e30, buf, stream)
        u_ms, u_scan_ms, u_found = timed_steps(
            plan, lambda: plan.topk_raw(K, MAX_THROUGHPUT, 1e30, buf, stream), 16, torch.cuda.synchronize)
        unbound = {"time_to_top64_ms": u_ms, "scan_kernel_ms": u_scan_ms, "found": u_found,
                   "units_evaluated": plan.last_scan()[0]}
        step()  # (the last query of the plan is the timed one again)

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
    del tt, cc, mm, kk

    # the same kind of query where nothing can be discarded: resources never bind, nearly every
    # candidate is a valid plan, and the budget is one that no plan exceeds (so no piece of the
    # space is ruled out by its cost bound either): every candidate's arithmetic is done
    dense_prob = workloads.config4_dense()
    pd = Plan(dense_prob)
    pd.set_incremental(False)
    budget_never = 1e30
    pd.set_timing(1)
    for _ in range(3):
        pd.topk_raw(K, MAX_THROUGHPUT, budget_never, buf, stream)
    dense_ms, dense_scan_ms, dense_found = timed_steps(
        pd, lambda: pd.topk_raw(K, MAX_THROUGHPUT, budget_never, buf, stream), 16, torch.cuda.synchronize)
    dense_counts = pd.last_counts()
    dense_evaluated, dense_units = pd.last_scan()
    assert dense_evaluated == dense_units, (dense_evaluated, dense_units)
    dense_budget = None
    if not args.only_kernels:
        # ... and under the timed query's kind of budget, where whole pieces fall to their bound
        budget_d = 1.2 * pd.best_plan(objective=MIN_COST, stream=stream).cost_per_iter
        for _ in range(3):
            pd.topk_raw(K, MAX_THROUGHPUT, budget_d, buf, stream)
        b_ms, b_scan_ms, b_found = timed_steps(
            pd, lambda: pd.topk_raw(K, MAX_THROUGHPUT, budget_d, buf, stream), 16, torch.cuda.synchronize)
        dense_budget = {"time_to_top64_ms": b_ms, "scan_kernel_ms": b_scan_ms, "found": b_found,
                        "units_evaluated": pd.last_scan()[0], "units": dense_units}
    pd.destroy()

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.only_kernels:
        print(json.dumps({"only_kernels": True, "candidates": n, "ms_per_step": ms_per_step,
                          "scan_kernel_ms": scan_ms, "eval_batch_ms": eval_ms,
                          "dense_time_to_top64_ms": dense_ms, "dense_scan_kernel_ms": dense_scan_ms,
                          "units_cfg4": units_total, "units_cfg4_evaluated": units_evaluated,
                          "scan_no_binding_budget_ms": unbound["scan_kernel_ms"],
                          "units_dense": dense_units,
                          "source_sha256": source_hash()}))
        plan.destroy()
        return 0

    # availability streams on the 4-zone x 3-type cluster (6 791 040 candidates): latency of
    # set_avail + best_plan per snapshot, with the per-unit minima kept between snapshots and
    # with a full evaluation at each
    prob5 = workloads.config3()
    walk, events = workloads.config5_snapshots(prob5), workloads.node_events(prob5)
    replan = {"snapshots": len(walk),
              "random_walk_full": replan_stream(np, Plan, prob5, walk, stream, False),
              "random_walk_incremental": replan_stream(np, Plan, prob5, walk, stream, True),
              "node_events_full": replan_stream(np, Plan, prob5, events, stream, False),
              "node_events_incremental": replan_stream(np, Plan, prob5, events, stream, True)}
    # the same kind of stream on the large workload, where the scan is half of a re-plan
    events4 = workloads.node_events(prob)
    replan["cfg4_node_events_full"] = replan_stream(np, Plan, prob, events4, stream, False)
    replan["cfg4_node_events_incremental"] = replan_stream(np, Plan, prob, events4, stream, True)
    # ... and on its space with a TP degree per segment (915 206 400 candidates), where a pass
    # over the space is most of a re-plan and kept minima shorten it
    prob4s = prob.with_per_segment_tp()
    replan["cfg4_segment_tp_node_events_full"] = replan_stream(np, Plan, prob4s, events4, stream, False)
    replan["cfg4_segment_tp_node_events_incremental"] = replan_stream(np, Plan, prob4s, events4, stream, True)
    for v in replan.values():
        if isinstance(v, dict) and not args.copy_probe:
            per = v.pop("units_evaluated_per_snapshot")
            v["units_evaluated_min_max"] = [int(min(per)), int(max(per))]

    # the same query on the widened spaces: a TP digit per segment (915 206 400 candidates),
    # replicas of a stage split over two GPU types (5 zones x 10 extended types)
    def widened(problem, reps):
        p = Plan(problem)
        p.set_incremental(False)
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

    # search over per-stage placements (spaces that cannot be enumerated: 12^32 and 20^48
    # placements per sub-problem), incumbent = the flat space's best plan through the evaluator
    def searched(problem, width, split, stage_tp=False):
        p = Plan(problem)
        p.set_incremental(False)
        flat = p.best_plan(objective=MAX_THROUGHPUT, stream=stream)
        kw = dict(incumbent="flat", allow_split=split, stage_tp=stage_tp, stream=stream)
        p.search(width, MAX_THROUGHPUT, **kw)  # (allocates its scratch)
        t0 = time.perf_counter()
        r = p.search(width, MAX_THROUGHPUT, **kw)
        ms = (time.perf_counter() - t0) * 1e3
        out = {"beam_width": width, "split_stages": split, "tp_per_stage": stage_tp,
               "tp_degrees_used": sorted({int(problem.tp_values[t]) for t in r.tps}),
               "ms_incl_flat_best_plan": ms,
               "placements_generated": r.expanded, "exact": r.exact, "flat_iter_time_s": flat.iter_time_s,
               "search_iter_time_s": r.iter_time_s, "pp": r.pp,
               "runs_of_pools": 1 + sum(a != b for a, b in zip(zip(r.pools, r.pools_b), zip(r.pools[1:], r.pools_b[1:]))),
               "stages_split": sum(a != b for a, b in zip(r.pools, r.pools_b))}
        p.destroy()
        return out

    # independent queries in flight: one plan, one stream and one host thread each (a serving
    # loop); the small kernels behind one query's scan then overlap the other queries' scans
    def in_flight(k, n=200):
        import threading
        plans = [Plan(prob) for _ in range(k)]
        streams = [torch.cuda.Stream() for _ in range(k)]
        for p in plans:
            p.set_incremental(False)
        took = [0.0] * k
        gate = threading.Barrier(k)

        def run(i):
            out = (sailor_result * K)()
            for _ in range(10):
                plans[i].topk_raw(K, MAX_THROUGHPUT, budget, out, streams[i].cuda_stream)
            gate.wait()
            t0 = time.perf_counter()
            for _ in range(n):
                plans[i].topk_raw(K, MAX_THROUGHPUT, budget, out, streams[i].cuda_stream)
            took[i] = time.perf_counter() - t0

        threads = [threading.Thread(target=run, args=(i,)) for i in range(k)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        for p in plans:
            p.destroy()
        return {"queries_in_flight": k, "ms_per_query_per_thread": max(took) / n * 1e3,
                "candidates_per_s_in_all": k * n * prob_n / max(took)}

    prob_n = n
    serving = [in_flight(2), in_flight(4)]

    search = {"cfg3": searched(prob5, 64, False), "cfg4": searched(prob, 64, False),
              "cfg3_split": searched(prob5, 32, True), "cfg4_split": searched(prob, 16, True),
              "cfg3_stage_tp": searched(prob5, 64, False, True), "cfg4_stage_tp": searched(prob, 32, False, True),
              # two pools and a TP degree per stage: 12 x 12 x 4 and 20 x 20 x 4 choices per stage
              "cfg3_split_stage_tp": searched(prob5, 16, True, True),
              "cfg4_split_stage_tp": searched(prob, 8, True, True)}

    # measured ceilings: scalar-per-lane FMA chain, streaming 16-byte stores, and the four
    # output arrays of the per-candidate evaluation written by a kernel that does nothing else
    fma_tflops, _ = microbench.fma(stream=stream)
    write_gbps, _ = microbench.write(stream=stream)
    records_gbps, _ = microbench.write_records(n, stream=stream)

    pbar = mean_pipeline_depth(prob)
    flops_per_cand = FLOPS_PER_STAGE * pbar + FLOPS_EPILOGUE
    counters, counters_note = load_counters()
    # The timed query's pass over the space.  Its budget leaves units_evaluated of units_total
    # pieces alive (the others fall to their cost bounds without being touched), so the pass is a
    # short, latency-bound launch; what the evaluation kernel sustains when the arithmetic has to
    # be done is in roofline_scan_no_binding_budget (validity pruning only) and roofline_dense
    # (nothing to prune).
    roof = alu_roofline(counters.get("pass_cfg4"), scan_ms, flops_per_cand * n)
    roof.update({"kernel": "k_units<COLLECT>, one pass over the pieces the budget leaves alive",
                 "pieces_evaluated": units_evaluated, "pieces_total": units_total,
                 "regime": "latency-bound: nearly all of the space falls to per-piece cost bounds; "
                           "see roofline_scan_no_binding_budget and roofline_dense for the kernel "
                           "at work",
                 "counters": counters_note,
                 "peak_note": "256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: one vector instruction per "
                              "lane and cycle; an FMA is one such instruction (78.6 TFLOP/s), "
                              "157.3 TFLOP/s needs packed FP32, which the library is compiled without",
                 "measured_fma_chain_tflops": fma_tflops,
                 "measured_clock_ghz": fma_tflops * 1e12 / (2 * CUS * SIMDS_PER_CU * LANES_PER_SIMD) / 1e9,
                 "flops_per_candidate_nominal": flops_per_cand})
    roof_unbound = alu_roofline(counters.get("scan_cfg4"), unbound["scan_kernel_ms"], flops_per_cand * n)
    roof_unbound.update({"kernel": "k_units<SCAN>",
                         "workload": "cfg4, the timed query under a budget that never binds"})
    roof_dense = alu_roofline(counters.get("scan_cfg4_dense"), dense_scan_ms, flops_per_cand * n)
    roof_dense.update({"kernel": "k_units<SCAN>", "workload": "cfg4_dense"})
    eval_entry = counters.get("eval_rows_cfg4")
    roof_eval = {"bound": "hbm", "kernel": "k_eval_rows", "unit": "GB/s",
                 "achieved": 20.0 * n / (eval_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS,
                 "frac": 20.0 * n / (eval_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                 "traffic": eval_entry.get("hbm_bytes") if eval_entry else None,
                 "kernel_ms": eval_ms, "measured_stream_write_GBps": write_gbps,
                 "frac_of_measured_write": 20.0 * n / (eval_ms * 1e-3) / 1e9 / write_gbps,
                 "measured_output_write_GBps": records_gbps,
                 "frac_of_measured_output_write": 20.0 * n / (eval_ms * 1e-3) / 1e9 / records_gbps,
                 "valu_insts_per_candidate": (eval_entry["counters"]["SQ_INSTS_VALU"] * 64 / n
                                              if eval_entry else None)}
    out = {
        "metric": "candidate plans evaluated/sec (whole space decided per step, top-64 selection "
                  "included) and time-to-best-plan",
        "value": n / (ms_per_step * 1e-3), "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg4: OPT-30B-like, 5 zones x 4 GPU types, 48 layers, "
                               "8 layer splits per pp, <=3 segments",
                   "candidates": n, "objective": "max throughput s.t. cost <= 1.2 x cheapest",
                   "top_k": K, "mean_pipeline_depth": pbar},
        "roofline": dict(roof, frac_scan_no_binding_budget=roof_unbound["frac"],
                         frac_scan_dense=roof_dense["frac"]),
        "roofline_scan_no_binding_budget": roof_unbound,
        "roofline_dense": roof_dense,
        "roofline_eval_batch": roof_eval,
        "extra": {"time_to_top64_ms": ms_per_step, "time_to_best_plan_ms": best_ms,
                  "scan_kernel_ms": scan_ms,
                  # (pieces hold equally many candidates before empty ones are dropped and long ones
                  # cut, so the share of pieces is about the share of candidates)
                  "pieces_of_the_space": {"evaluated": units_evaluated, "total": units_total,
                                          "share_evaluated_candidate_by_candidate": units_evaluated / units_total,
                                          "rest": "ruled out by the cost bound of their piece (one comparison "
                                                  "each); results equal the oracle's over all candidates"},
                  "same_query_with_a_budget_that_never_binds": unbound,
                  "every_candidate_evaluated": {
                      "eval_batch_ms": eval_ms,
                      "eval_batch_candidates_per_s": n / (eval_ms * 1e-3),
                      "dense_time_to_top64_ms": dense_ms, "dense_scan_kernel_ms": dense_scan_ms,
                      "dense_candidates_per_s": n / (dense_ms * 1e-3),
                      "dense_found": dense_found,
                      "dense_under_budget_of_1p2x_cheapest": dense_budget,
                      "dense_survivors_refined_valid": list(dense_counts)},
                  "plan_create_ms": create_ms, "plan_create_warm_ms": create_warm_ms,
                  "replan_stream": replan,
                  "per_segment_tp": segtp, "mixed_types": mixed, "placement_search": search,
                  "independent_queries_in_flight": serving,
                  "event_schedule_top64": event_sched,
                  "survivors_refined_valid": list(counts), "best_index": best.index,
                  "top1_index": top1_index},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(prob, prob5, budget, K, args.cpu_sample, args.cpu_snapshots)
    plan.destroy()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
