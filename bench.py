#!/usr/bin/env python3
"""Benchmark of the plan-evaluation path on one MI355X.

A step is one pass of the whole path over one synthetic scheduling problem:
enumerate plans -> (per job chunk) evaluate candidates into the candidate
tensor and take the best plan per segment, in one kernel -> curves -> greedy
allocation.  Inputs are resident in HBM before the timed
region.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on the stress workload with 3 job
# chunks (profiles/hbm_traffic_stress.txt), already scaled by the plain-copy calibration (fetch x2.0, write x1.0).
# Valid only for the kernel sources they were taken with: keyed by the digest of those sources.
KERNEL_SOURCES = ("paper_2408_08586_amd/csrc/rk_eval.hip", "paper_2408_08586_amd/csrc/rk_model.h")
MEASURED_TRAFFIC = {
    # digest: {kernel: bytes per launch}
    "7270069ae4037b51": {"k_eval_best": 946942623, "k_eval": 918506644, "k_best_plan": 932046735},
}


# Vector-ALU instructions per launch of the fused kernel on the stress workload (rocprofv3 --pmc SQ_INSTS_VALU,
# profiles/valu_stress.txt: wavefront instructions, 64 lanes each), keyed by the digest of its sources.
FUSED_SOURCES = ("paper_2408_08586_amd/csrc/rk_fused.hip", "paper_2408_08586_amd/csrc/rk_model.h")
MEASURED_FUSED_VALU = {"3debe60fc20d6551": 47806051}
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz: vector instructions per lane and second (an FMA is one of them,
# so this is half of the 78.6 TFLOP/s of unpacked FP32 and a quarter of the 157.3 TFLOP/s with packed FP32)
VALU_PEAK_LANE_INSTR = 256 * 4 * 16 * 2.4e9
# log2 / exp2 / reciprocal issue at a quarter of that rate
TRANS_PEAK_LANE_INSTR = VALU_PEAK_LANE_INSTR / 4
# Arithmetic the model needs once everything shared is computed once (counted from the formulas of Sec. 4 as the fused
# kernel factors them; float32 operations / quarter-rate operations, a correctly rounded division = 10 + 1):
#   per triple:                      terms shared by its 16 options (times, volumes, two overlaps, activations)
#   per plan without offload:        memory verdict + optimizer term + throughput
#   per triple with offload allowed: PCIe term, one overlap, host bytes, four memory verdicts
#   per (CPU level, such a triple):  swap overlap, two throughputs, keys, tier tests
ALGO_OPS = {"triple": (120, 18), "plain_plan": (20, 2.25), "offload_triple": (90, 14), "offload_level": (34, 8)}


def source_digest(sources):
    import hashlib
    h = hashlib.sha256()
    for rel in sources:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def kernel_digest():
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def build_workload(name):
    import workloads
    if name == "stress":
        return workloads.stress(), ("stress: 10,000 jobs, G=4096 (512 nodes x 8 GPUs), CPU ratios {1,2,4,8,16} per GPU, "
                                    "host-memory tiers {0,64,256,1024} GiB")
    if name == "large":
        return workloads.large(), "large: 1,000 jobs, G=1024, CPU ratios {1,2,4,8,16} per GPU, one 2048 GiB tier"
    if name == "paper_scale":
        return workloads.paper_scale(), "paper_scale: 64 jobs, G=64, 1..32 CPUs, one 64 GiB tier"
    if name == "tiny":
        return workloads.tiny(), "tiny: 8 jobs, G=8"
    raise SystemExit(f"unknown workload {name}")


def oracle_round(oracle, wl, threads):
    """One whole round of the oracle, as it stands, on `threads` host threads (enumeration, evaluation and best-plan
    search share the jobs among them; curves and greedy are plain loops on one).  Returns (candidates, seconds per stage)."""
    t0 = time.perf_counter()
    tb = oracle.enumerate_plans(wl.ints, wl.bounds, n_threads=threads)
    t1 = time.perf_counter()
    thr, _ = oracle.eval_jobs(wl.coef, wl.ints, wl.bounds, tb, wl.grid, wl.env, want_reason=False, n_threads=threads)
    t2 = time.perf_counter()
    bt64, bp = oracle.best_plan(tb, wl.grid, thr, n_threads=threads)
    bt = bt64.astype(np.float32)
    ct, cp, cg = oracle.curves(tb, wl.grid, bt, bp)
    t3 = time.perf_counter()
    oracle.greedy(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct)
    t4 = time.perf_counter()
    return thr.size, {"enumerate": t1 - t0, "evaluate": t2 - t1, "best_plan+curves": t3 - t2, "greedy": t4 - t3,
                      "round": t4 - t0}


def cpu_baseline(wl, sample_jobs):
    """The oracle, as it stands, timed on this machine's host cores: the benchmark's workload (a stated sample of its
    jobs) and the other configurations, each on all the cores this process may use and on one."""
    import oracle
    import workloads
    host_cores = oracle.host_cores()
    # the box gives one GPU's share of its cores to a job: 16 threads (OMP_NUM_THREADS), whatever the machine has
    threads = max(1, min(host_cores, int(os.environ.get("OMP_NUM_THREADS", "16"))))

    def sample(w, n):
        sub = w.subset(np.arange(min(n, w.n_jobs)))
        frac = sub.n_jobs / w.n_jobs
        sub.cluster = workloads.Cluster(max(1, int(w.cluster.G * frac)), max(1, int(w.cluster.C * frac)),
                                        w.cluster.host_mem_gb * frac)
        return sub

    def both(w, n_all, n_one):
        a, b = sample(w, n_all), sample(w, n_one)
        n_a, s_a = oracle_round(oracle, a, threads)
        n_b, s_b = oracle_round(oracle, b, 1)
        return {"all_cores": {"jobs": a.n_jobs, "candidates": n_a, "candidates_per_s": n_a / s_a["round"],
                              "round_ms": s_a["round"] * 1e3, "eval_only_candidates_per_s": n_a / s_a["evaluate"],
                              "seconds": s_a},
                "one_thread": {"jobs": b.n_jobs, "candidates": n_b, "candidates_per_s": n_b / s_b["round"],
                               "round_ms": s_b["round"] * 1e3, "eval_only_candidates_per_s": n_b / s_b["evaluate"],
                               "seconds": s_b}}

    main = both(wl, sample_jobs, max(1, sample_jobs // 8))
    others = {}
    for name, w, n_all, n_one in (("tiny", workloads.tiny(), 8, 8), ("paper_scale", workloads.paper_scale(), 64, 64),
                                  ("large", workloads.large(), 1000, 250), ("what_if[0]", workloads.what_if(0), 500, 250)):
        if w.name != wl.name:
            others[name] = both(w, n_all, n_one)
    a = main["all_cores"]
    return {"value": a["candidates_per_s"], "unit": "candidates/s", "cores": threads, "host_cores": host_cores,
            "kind": "oracle", "round_ms": a["round_ms"],
            "sample": f"first {a['jobs']} of the workload's {wl.n_jobs} jobs ({a['candidates']} candidates), capacities "
                      f"scaled to the sample; whole path (enumerate, evaluate, best plan, curves, greedy); enumeration, "
                      f"evaluation and best-plan search on {threads} threads, curves and greedy on 1; one-thread figures "
                      f"on the first {main['one_thread']['jobs']} jobs",
            "seconds": a["seconds"], "eval_only_candidates_per_s": a["eval_only_candidates_per_s"],
            "one_thread": main["one_thread"], "other_configurations": others}


def other_rounds(rk, ctx, dev, skip, reps):
    """rk_schedule_round on the small configurations (the oracle's times for the same rounds are in cpu_baseline):
    latency of the whole round, host-synchronous, inputs resident."""
    import torch
    import workloads
    out = {}
    for name, make in (("tiny", workloads.tiny), ("paper_scale", workloads.paper_scale), ("large", workloads.large)):
        if name == skip:
            continue
        w = make()
        jobs = rk.Jobs(w.coef, w.ints, dev)
        bounds, grid, env, cluster = rk.make_bounds(w.bounds), rk.make_grid(w.grid), rk.make_env(w.env), rk.make_cluster(w.cluster)
        table = rk.enumerate_to_table(ctx, jobs, bounds, dev)
        n_rows = len(w.grid.cpu_levels) * len(w.grid.mem_levels_gb)
        assign, total = rk.new_assign(w.n_jobs, dev), torch.zeros(1, dtype=torch.float32, device=dev)
        lat = []
        for i in range(reps + 3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rk.rk_schedule_round(ctx, jobs, bounds, grid, env, cluster, assign, total)
            torch.cuda.synchronize()
            if i >= 3:
                lat.append((time.perf_counter() - t0) * 1e3)
        n = table.n_candidates(n_rows)
        out[name] = {"jobs": w.n_jobs, "candidates": n, "round_ms": {"min": float(np.min(lat)), "median": float(np.median(lat)),
                                                                     "max": float(np.max(lat))},
                     "nominal_candidates_per_s": n / (float(np.median(lat)) * 1e-3)}
    return out


def what_if_batch(rk, ctx, dev, n_rounds):
    """What-if configuration: independent rounds of 500 jobs on about 512 GPUs.  Latency of each round run on
    its own (rk_schedule_round, host-synchronous) and time of all rounds as one rk_schedule_rounds batch."""
    import torch
    import workloads
    rounds = [workloads.what_if(r) for r in range(n_rounds)]
    coef = np.concatenate([w.coef for w in rounds])
    ints = np.concatenate([w.ints for w in rounds])
    base = rounds[0]
    bounds, grid, env = rk.make_bounds(base.bounds), rk.make_grid(base.grid), rk.make_env(base.env)
    clusters = [rk.make_cluster(w.cluster) for w in rounds]
    jobs_all = rk.Jobs(coef, ints, dev)
    round_off = np.concatenate([[0], np.cumsum([w.n_jobs for w in rounds])]).astype(np.uint32)
    assign = rk.new_assign(len(coef), dev)
    totals = torch.zeros(n_rounds, dtype=torch.float32, device=dev)
    batch_ms = []
    for it in range(4):
        torch.cuda.synchronize()
        a = time.perf_counter()
        rk.rk_schedule_rounds(ctx, jobs_all, bounds, grid, env, round_off, clusters, assign, totals)
        torch.cuda.synchronize()
        if it:
            batch_ms.append((time.perf_counter() - a) * 1e3)
    single = rk.Jobs(rounds[0].coef, rounds[0].ints, dev)
    a1, t1 = rk.new_assign(rounds[0].n_jobs, dev), torch.zeros(1, dtype=torch.float32, device=dev)
    lat = []
    for r, w in enumerate(rounds):
        single = rk.Jobs(w.coef, w.ints, dev)
        torch.cuda.synchronize()
        a = time.perf_counter()
        rk.rk_schedule_round(ctx, single, bounds, grid, env, clusters[r], a1, t1)
        torch.cuda.synchronize()
        lat.append((time.perf_counter() - a) * 1e3)
    lat = np.array(lat[1:])                                     # the first call sizes the scratch buffers
    q = lambda p: float(np.percentile(lat, p))
    # the same rounds with every distinct job listed once (nine jobs in ten are shared by all rounds)
    swl, s_off, s_jobs, s_clusters = workloads.what_if_shared(n_rounds)
    jobs_distinct = rk.Jobs(swl.coef, swl.ints, dev)
    assign_s = rk.new_assign(len(s_jobs), dev)
    totals_s = torch.zeros(n_rounds, dtype=torch.float32, device=dev)
    shared_ms = []
    for it in range(4):
        torch.cuda.synchronize()
        a = time.perf_counter()
        rk.rk_schedule_rounds_shared(ctx, jobs_distinct, bounds, grid, env, s_off, s_jobs, clusters, assign_s, totals_s)
        torch.cuda.synchronize()
        if it:
            shared_ms.append((time.perf_counter() - a) * 1e3)
    same = bool(torch.equal(totals, totals_s)) and bool(torch.equal(assign, assign_s))
    return {"rounds": n_rounds, "jobs_per_round": rounds[0].n_jobs,
            "single_round_latency_ms": {"min": float(lat.min()), "median": q(50), "p95": q(95), "p99": q(99),
                                        "max": float(lat.max())},
            "batch_ms": float(np.median(batch_ms)), "batch_rounds_per_s": n_rounds / (float(np.median(batch_ms)) * 1e-3),
            "shared_jobs_batch": {"entry": "rk_schedule_rounds_shared", "distinct_jobs": swl.n_jobs,
                                  "ms": float(np.median(shared_ms)),
                                  "rounds_per_s": n_rounds / (float(np.median(shared_ms)) * 1e-3),
                                  "identical_to_batch": same}}


def placement(rk, ctx, dev, wl, assign, reps):
    """Node-level placement (rk_place) of the round's assignment on nodes of the
    workload's shape (the cluster's GPUs, CPUs and memory spread evenly over nodes
    of 8 GPUs), and on nodes with only 6 CPUs (less than the one CPU per GPU the
    round's jobs hold), where the job-by-job stage has to run and some jobs find
    no place.  Host-synchronous latency of the call."""
    import torch
    J = wl.n_jobs
    gpn = 8
    n_nodes = max(1, wl.cluster.G // gpn)
    cap = n_nodes * gpn
    off = torch.zeros(J + 1, dtype=torch.int32, device=dev)
    status = torch.zeros(J, dtype=torch.int32, device=dev)
    ent = rk.new_place_entries(cap, dev)
    out = {"entry": "rk_place (host-synchronous)", "nodes": n_nodes, "gpus_per_node": gpn}
    for name, cpn in (("roomy", wl.cluster.C // n_nodes), ("tight_cpus", 6)):
        nodes = rk.rk_nodes(n_nodes, gpn, min(int(cpn), 65535), float(wl.cluster.host_mem_gb) / n_nodes)
        lat = []
        for i in range(reps + 2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            res = rk.rk_place(ctx, nodes, J, assign, off, ent, cap, status)
            if i >= 2:
                lat.append((time.perf_counter() - t0) * 1e3)
        out[name] = {"cpus_per_node": int(nodes.cpus_per_node), "ms": float(np.median(lat)), "placed": res.n_placed,
                     "not_placed": res.n_failed, "parts": res.n_entries, "job_by_job_stage": bool(res.in_order)}
    return out


def algorithm1_bench(rk, ctx, dev, wl, jobs, table, grid, env, best_thr, best_plan, curve_thr, assign, reps):
    """Algorithm 1 as a loop and on nodes, on the same workload: the state the from-scratch round leaves, then a tenth
    of the jobs leave (their slots are new arrivals) and the cluster loses a tenth of its GPUs and CPUs:
    rk_reschedule from that state; then rk_place_plans of its result on nodes of 8 GPUs, roomy and with 6 CPUs each
    (fall-back to smaller GPU counts, plans chosen again on the actual node split), with the placement of the state
    before as the earlier placement: jobs whose amounts the loop left alone stay on their nodes."""
    import torch
    J = wl.n_jobs
    a0 = rk.assign_to_numpy(assign)
    seg_off = np.asarray(table.h_seg_off[:J + 1], dtype=np.int64)
    seg_g = rk.u32(table.seg_g)
    levels = np.asarray(wl.grid.cpu_levels)
    cur_seg, cur_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    for j in np.flatnonzero(a0["g"] > 0).tolist():
        cur_seg[j] = int(np.flatnonzero(seg_g[seg_off[j]:seg_off[j + 1]] == a0["g"][j])[0])
        per = a0["c"][j] // a0["g"][j] if wl.grid.cpu_mode else a0["c"][j]
        cur_c[j] = int(np.flatnonzero(levels == per)[0])
    rng = np.random.default_rng(J)
    cur_seg[rng.uniform(size=J) < 0.1] = -1
    held = int(sum(int(seg_g[seg_off[j] + cur_seg[j]]) for j in np.flatnonzero(cur_seg >= 0)))
    small = rk.make_cluster(type(wl.cluster)(max(held, int(wl.cluster.G * 0.9)), int(wl.cluster.C * 0.9), wl.cluster.host_mem_gb))
    d_seg = torch.from_numpy(cur_seg).to(dev)
    d_c = torch.from_numpy(cur_c.view(np.int32)).to(dev)
    out, total = rk.new_assign(J, dev), torch.zeros(1, dtype=torch.float32, device=dev)
    moves = torch.zeros(4, dtype=torch.int32, device=dev)
    ms = []
    for i in range(reps + 2):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        rk.rk_reschedule(ctx, jobs.ref_thr, table.c, grid, small, best_thr, best_plan, curve_thr, d_seg, d_c, out, total,
                         n_moves=moves)
        b.record()
        torch.cuda.synchronize()
        if i >= 2:
            ms.append(a.elapsed_time(b))
    res = rk.assign_to_numpy(out)
    info = {"entry": "rk_reschedule (one workgroup; sequential by definition)", "jobs": J,
            "jobs_running_before": int((cur_seg >= 0).sum()), "steps_committed": int(moves[0].item()), "jobs_on_the_full_path": int(moves[1].item()),
            "shrinks_applied": int(moves[2].item()), "steps_taken_back": int(moves[3].item()),
            "jobs_running_after": int((res["g"] > 0).sum()), "ms": float(np.median(ms))}
    # what-if: the same state under 64 other capacities (0.75 to 1.25 of the cluster), all rounds in one call
    n_what = 64
    what = [rk.make_cluster(type(wl.cluster)(max(held, int(wl.cluster.G * u)), int(wl.cluster.C * u), wl.cluster.host_mem_gb))
            for u in np.linspace(0.75, 1.25, n_what)]
    outs, totals = rk.new_assign(J * n_what, dev), torch.zeros(n_what, dtype=torch.float32, device=dev)
    st64 = torch.zeros(4 * n_what, dtype=torch.int32, device=dev)
    ms64 = []
    for i in range(reps + 2):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        rk.rk_reschedule_rounds(ctx, jobs.ref_thr, table.c, grid, what, best_thr, best_plan, curve_thr, d_seg, d_c, outs, totals,
                                stats=st64)
        b.record()
        torch.cuda.synchronize()
        if i >= 2:
            ms64.append(a.elapsed_time(b))
    info["what_if_rounds"] = {"entry": "rk_reschedule_rounds (a workgroup per round)", "rounds": n_what, "jobs": J,
                              "capacities": "0.75 to 1.25 of the cluster's GPUs and CPUs, from the same state",
                              "steps_committed_min_max": [int(st64.cpu().numpy()[0::4].min()), int(st64.cpu().numpy()[0::4].max())],
                              "ms": float(np.median(ms64)), "ms_per_round": float(np.median(ms64)) / n_what,
                              "rounds_per_s": n_what / (float(np.median(ms64)) * 1e-3)}
    del outs
    # service levels through the loop: 30 % guaranteed jobs of 6 tenants (quotas: half the cluster), minimum demands at
    # half the drawn request; rk_privileged turns them into floors and states, the loop runs from these
    import workloads
    sl = workloads.sla_draws(wl, quota_share=0.5)
    ns = (seg_off[1:] - seg_off[:-1])
    min_seg = np.where(ns > 0, np.minimum((sl.u_seg * ns * 0.5).astype(np.int64), np.maximum(ns - 1, 0)), -1).astype(np.int32)
    sla = rk.Sla(sl.guaranteed, sl.tenant, sl.quota_g, sl.quota_c, device=dev)
    d_min = torch.from_numpy(min_seg).to(dev)
    d_minc = torch.zeros(J, dtype=torch.int32, device=dev)
    fl_s, fl_c = torch.zeros(J, dtype=torch.int32, device=dev), torch.zeros(J, dtype=torch.int32, device=dev)
    st_o = torch.zeros(J, dtype=torch.uint8, device=dev)
    ms_p, ms_l = [], []
    for i in range(reps + 2):
        a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        a.record()
        rk.rk_privileged(ctx, table.c, grid, sla, d_min, d_minc, d_seg, d_c, fl_s, fl_c, st_o)
        b.record()
        rk.rk_reschedule(ctx, jobs.ref_thr, table.c, grid, small, best_thr, best_plan, curve_thr, d_seg, d_c, out, total,
                         state=st_o, floor_seg=fl_s, floor_c=fl_c, n_moves=moves)
        c.record()
        torch.cuda.synchronize()
        if i >= 2:
            ms_p.append(a.elapsed_time(b)); ms_l.append(b.elapsed_time(c))
    res_s = rk.assign_to_numpy(out)
    gu = sl.guaranteed != 0
    info["with_service_levels"] = {"entry": "rk_privileged, then rk_reschedule from its floors and states",
                                   "guaranteed_jobs": int(gu.sum()), "floors_granted": int((fl_s.cpu().numpy() >= 0).sum()),
                                   "jobs_that_wait": int((st_o.cpu().numpy() == 1).sum()),
                                   "guaranteed_jobs_running_after": int((gu & (res_s["g"] > 0)).sum()),
                                   "steps_committed": int(moves[0].item()), "privileged_ms": float(np.median(ms_p)),
                                   "loop_ms": float(np.median(ms_l))}
    gpn, n_nodes = 8, max(1, wl.cluster.G // 8)
    cap = n_nodes * gpn
    placed = rk.new_assign(J, dev)
    off = torch.zeros(J + 1, dtype=torch.int32, device=dev)
    status = torch.zeros(J, dtype=torch.int32, device=dev)
    ent = rk.new_place_entries(cap, dev)
    info["place_plans"] = {"entry": "rk_place_plans (host-synchronous)", "nodes": n_nodes, "gpus_per_node": gpn}
    # where the jobs sat before the loop: the from-scratch round's amounts on the same nodes (the earlier placement)
    before = rk.new_assign(J, dev)
    off0 = torch.zeros(J + 1, dtype=torch.int32, device=dev)
    ent0 = rk.new_place_entries(cap, dev)
    for name, cpn in (("roomy", wl.cluster.C // n_nodes), ("tight_cpus", 6)):
        nodes = rk.rk_nodes(n_nodes, gpn, min(int(cpn), 65535), float(wl.cluster.host_mem_gb) / n_nodes)
        rk.rk_place_plans(ctx, jobs, table.c, grid, env, nodes, best_thr, assign, None, before, off0, ent0, cap, status, total)
        lat = []
        for i in range(reps + 2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            r = rk.rk_place_plans(ctx, jobs, table.c, grid, env, nodes, best_thr, out, None, placed, off, ent, cap, status, total,
                                  prev_off=off0, prev_entries=ent0)
            if i >= 2:
                lat.append((time.perf_counter() - t0) * 1e3)
        o0, o1 = rk.u32(off0)[:J + 1].astype(np.int64), rk.u32(off)[:J + 1].astype(np.int64)
        e0, e1 = rk.place_entries_to_numpy(ent0, int(o0[J])), rk.place_entries_to_numpy(ent, r.n_entries)
        stayed = sum(1 for j in np.flatnonzero((np.diff(o0) > 0) & (np.diff(o1) > 0)).tolist()
                     if np.array_equal(e0[o0[j]:o0[j + 1]], e1[o1[j]:o1[j + 1]]))
        st = rk.u32(status)[:J]
        p = rk.assign_to_numpy(placed)
        info["place_plans"][name] = {"cpus_per_node": int(nodes.cpus_per_node), "ms": float(np.median(lat)),
                                     "placed_as_asked": int((st == 1).sum()), "placed_with_fewer_gpus": int((st == 2).sum()),
                                     "not_placed": int((st == 3).sum()), "parts": r.n_entries,
                                     "plans_changed_by_the_split": int(((p["plan"] != res["plan"]) & (st == 1)).sum()),
                                     "jobs_that_stayed_on_their_nodes": int(stayed),
                                     "job_by_job_stage": bool(r.in_order)}
    if wl.grid.cpu_mode == 1:
        # the same loop with ScheduleJob searching node by node: the jobs start where the from-scratch round's amounts
        # were placed (roomy nodes), those of the departed slots hold nothing
        nodes = rk.rk_nodes(n_nodes, gpn, min(int(wl.cluster.C // n_nodes), 65535), float(wl.cluster.host_mem_gb) / n_nodes)
        r0 = rk.rk_place_plans(ctx, jobs, table.c, grid, env, nodes, best_thr, assign, None, before, off0, ent0, cap, status, total)
        seg_n = cur_seg.copy()
        seg_n[rk.u32(status)[:J] != 1] = -1
        d_seg_n = torch.from_numpy(seg_n).to(dev)
        stats = torch.zeros(5, dtype=torch.int32, device=dev)
        ms = []
        for i in range(reps + 2):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rk.rk_reschedule_nodes(ctx, jobs.ref_thr, table.c, grid, nodes, best_thr, best_plan, curve_thr, d_seg_n, d_c, out, off,
                                   ent, cap, total, prev_off=off0, prev_entries=ent0, n_prev_entries=r0.n_entries, stats=stats)
            b.record()
            torch.cuda.synchronize()
            if i >= 2:
                ms.append(a.elapsed_time(b))
        res_n = rk.assign_to_numpy(out)
        o1 = rk.u32(off)[:J + 1].astype(np.int64)
        # GetBestPlan(j, placement) on what the loop left: the plans under the bandwidths of the actual node splits
        ms_plan = []
        for i in range(reps + 2):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rk.rk_best_plan_placed(ctx, jobs, table.c, grid, env, out, off, ent, placed, total)
            b.record()
            torch.cuda.synchronize()
            if i >= 2:
                ms_plan.append(a.elapsed_time(b))
        p_n = rk.assign_to_numpy(placed)
        # the whole round in one call from the job descriptors (enumeration, curves, the loop, the plans); host time
        lat = []
        for i in range(reps + 2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rk.rk_schedule_round_nodes(ctx, jobs, rk.make_bounds(wl.bounds), grid, env, nodes, d_seg_n, d_c, out, placed, off, ent,
                                       cap, total, prev_off=off0, prev_entries=ent0, n_prev_entries=r0.n_entries)
            torch.cuda.synchronize()
            if i >= 2:
                lat.append((time.perf_counter() - t0) * 1e3)
        st5 = stats.cpu().numpy()
        info["over_nodes"] = {"entry": "rk_reschedule_nodes (one workgroup; the job to shrink is one of the node under search)",
                              "nodes": n_nodes, "gpus_per_node": gpn, "cpus_per_node": int(nodes.cpus_per_node),
                              "jobs_running_before": int((seg_n >= 0).sum()), "steps_committed": int(st5[0]),
                              "jobs_on_the_full_path": int(st5[1]), "shrinks_applied": int(st5[2]),
                              "steps_taken_back": int(st5[3]), "jobs_running_after": int((res_n["g"] > 0).sum()),
                              "jobs_on_several_nodes": int((np.diff(o1) > 1).sum()), "parts": int(o1[J]),
                              "ms": float(np.median(ms)),
                              "best_plan_placed": {"entry": "rk_best_plan_placed (k_replan + k_place_total)",
                                                   "plans_changed_by_the_split": int(((p_n["plan"] != res_n["plan"]) & (res_n["g"] > 0)).sum()),
                                                   "total": float(total[0].item()), "ms": float(np.median(ms_plan))},
                              "round_from_descriptors": {"entry": "rk_schedule_round_nodes (host-synchronous)",
                                                         "ms": float(np.median(lat))}}
    return info


def sla_round(rk, ctx, dev, wl, jobs, table, bounds, grid, env, cluster, best_plan, n_rows, reps):
    """Service-level variant of the round on the same workload: 30 % guaranteed
    jobs of 6 tenants whose quotas sum to half the cluster.  A job's original
    plan is the best plan of its requested GPU count at the lowest CPU level and
    memory tier (taken from the library's own output), evaluated at the
    requested resources by rk_eval_points.  Times of the added calls (HIP
    events) and the latency of the single-call round."""
    import torch
    import workloads
    J = wl.n_jobs
    d = workloads.sla_draws(wl, quota_share=0.5)
    seg_off = np.asarray(table.h_seg_off[:J + 1], dtype=np.int64)
    seg_g = rk.u32(table.seg_g)
    ns = seg_off[1:] - seg_off[:-1]
    s_req = np.minimum((d.u_seg * ns).astype(np.int64), np.maximum(ns - 1, 0))
    req_g = np.where(ns > 0, seg_g[np.minimum(seg_off[:-1] + s_req, len(seg_g) - 1)], 0).astype(np.uint32)
    bp = rk.u32(best_plan)
    plan = bp[np.minimum(n_rows * seg_off[:-1] + s_req, len(bp) - 1)]      # row 0: lowest CPU level and memory tier
    seg_first = rk.u32(table.seg_first)
    fallback = (seg_first[np.minimum(seg_off[:-1] + s_req, len(seg_first) - 1)] * 16).astype(np.uint32)
    plan = np.where((plan == rk.RK_NO_PLAN) | (ns == 0), fallback, plan).astype(np.uint32)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).to(dev)
    base = torch.zeros(J + 4, dtype=torch.float32, device=dev)
    pj, pp, pc, pm = to_dev(np.arange(J)), to_dev(plan), to_dev(d.req_c), to_dev(d.req_m)
    sla = rk.Sla(d.guaranteed, d.tenant, d.quota_g, d.quota_c, req_g, d.req_c, d.req_m, base[:J], device=dev)
    assign = rk.new_assign(J, dev)
    total = torch.zeros(1, dtype=torch.float32, device=dev)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    t_points, lat = [], []
    for i in range(reps + 2):
        a, b = ev(), ev()
        a.record()
        rk.rk_eval_points(ctx, jobs, table.c, grid, env, pj, pp, pc, pm, base[:J])
        b.record()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rk.rk_schedule_round_sla(ctx, jobs, bounds, grid, env, cluster, sla, assign, total)
        torch.cuda.synchronize()
        if i >= 2:
            t_points.append(a.elapsed_time(b))
            lat.append((time.perf_counter() - t0) * 1e3)
    res = rk.assign_to_numpy(assign)
    gu = d.guaranteed != 0
    return {"entry": "rk_eval_points (baselines) + rk_schedule_round_sla (host-synchronous)",
            "guaranteed_jobs": int(gu.sum()), "guaranteed_served": int((gu & (res["g"] > 0)).sum()),
            "jobs_served": int((res["g"] > 0).sum()), "gpus_granted": int(res["g"].sum()),
            "eval_points_ms": float(np.mean(t_points)),
            "round_ms": {"min": float(np.min(lat)), "median": float(np.median(lat)), "max": float(np.max(lat))}}


def fit_bench(rk, ctx, dev, wl, env, reps):
    """Model fitting on the same 10,000 job descriptors, each taken as a model
    type with 16 measured runs (5 of them offloaded) on at most 64 GPUs.  The
    "measurements" are the library's own float32 predictions under the true
    parameters times 5 % log-normal noise; the fit starts from parameters that
    are off by up to a factor of two, plus 4 perturbed starting points."""
    import torch
    import workloads
    J, S = wl.n_jobs, 16
    dr = workloads.fit_draws(J, S)
    jobs_true = rk.Jobs(wl.coef, wl.ints, dev)
    b64 = rk.make_bounds(workloads.Bounds(g_max=64))
    table = rk.enumerate_to_table(ctx, jobs_true, b64, dev)
    triples = table.unpack_triples()
    d, t, p = workloads.fit_sample_triples(dr, table.h_triple_off, triples)
    levels = np.array([1, 2, 4, 8, 16, 32], np.uint32)
    grid = rk.make_grid(workloads.Grid(levels, 0, np.array([1.0e9], np.float32), 0))
    t0 = np.asarray(table.h_triple_off[:J], np.int64)[:, None]
    nt = (np.asarray(table.h_triple_off[1:J + 1], np.int64) - t0[:, 0])[:, None]
    local = np.minimum((dr.u_triple * nt).astype(np.int64), np.maximum(nt - 1, 0))
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).reshape(-1).view(np.int32)).to(dev)
    clean = torch.zeros(J * S + 4, dtype=torch.float32, device=dev)
    rk.rk_eval_points(ctx, jobs_true, table.c, grid, env, to_dev(np.repeat(np.arange(J), S)),
                      to_dev(local * 16 + dr.option), to_dev(np.searchsorted(levels, dr.cpus)),
                      to_dev(np.zeros((J, S))), clean[:J * S])
    rk.rk_sync(ctx)
    y = clean[:J * S].cpu().numpy().reshape(J, S) * np.exp(0.05 * dr.noise_z)
    coef0 = wl.coef.copy()
    cols = [5, 6, 7, 8, 9, 10, 11]
    start = coef0[:, cols].astype(np.float64) * dr.start_factor
    start[:, [1, 4, 5]] = np.clip(start[:, [1, 4, 5]], 1.0, rk.RK_FIT_K_MAX)
    coef0[:, cols] = start.astype(np.float32)
    jobs0 = rk.Jobs(coef0, wl.ints, dev)
    smp = rk.Samples(np.arange(J + 1) * S, rk.pack_triples(d, t, p).reshape(-1), dr.option.reshape(-1),
                     dr.cpus.reshape(-1), y.reshape(-1), device=dev)
    res = rk.FitResult(J, dev)
    ms = []
    for i in range(reps + 1):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        rk.rk_fit_models(ctx, jobs0, env, smp, res, max_iter=100, start_offsets=dr.start_offsets)
        b.record()
        torch.cuda.synchronize()
        if i:
            ms.append(a.elapsed_time(b))
    before, after = res.rmsle_before.cpu().numpy()[:J], res.rmsle_after.cpu().numpy()[:J]
    iters = res.iters.cpu().numpy()[:J].astype(np.int64)
    return {"entry": "rk_fit_models", "models": J, "runs_per_model": S, "starting_points": 1 + len(dr.start_offsets),
            "dtype": "f64", "ms": float(np.median(ms)), "models_per_s": J / (float(np.median(ms)) * 1e-3),
            "iterations_per_model": float(iters.mean()), "model_evaluations_per_s": float(iters.sum()) * S / (float(np.median(ms)) * 1e-3),
            "rmsle_before_median": float(np.median(before)), "rmsle_after_median": float(np.median(after)),
            "noise_sigma": 0.05}


def sim_bench(rk, ctx, dev, reps):
    """Discrete-time simulation in the shape of the paper's trace experiment:
    406 jobs arriving over 12 hours on 64 GPUs, one-minute ticks (720 rounds with
    the reconfiguration-penalty gate), curves computed once by the library."""
    import torch
    import workloads
    wl = workloads.trace_scale()
    J = wl.n_jobs
    jobs = rk.Jobs(wl.coef, wl.ints, dev)
    bounds, grid, env = rk.make_bounds(wl.bounds), rk.make_grid(wl.grid), rk.make_env(wl.env)
    cluster = rk.make_cluster(wl.cluster)
    table = rk.enumerate_to_table(ctx, jobs, bounds, dev)
    n_rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
    n = table.n_segments(n_rows)
    f32 = lambda: torch.empty(n + 4, dtype=torch.float32, device=dev)
    i32 = lambda: torch.empty(n + 4, dtype=torch.int32, device=dev)
    bt, bp, ct, cp, cg = f32(), i32(), f32(), i32(), i32()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    rk.rk_job_curves(ctx, jobs, table.c, grid, env, 0, J, bt, bp, ct, cp, cg)
    b.record()
    tr = workloads.trace(J, horizon_s=12 * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * 4.0
    f64 = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.float64)).to(dev)
    arrival, work_d, delta = f64(tr.arrival), f64(work), f64(tr.delta)
    n_ticks = 720
    res = rk.SimResult(J, n_ticks, dev)
    wall = []
    for i in range(reps + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rk.rk_simulate(ctx, jobs.ref_thr, table.c, grid, cluster, bt, bp, ct, arrival, work_d, delta, 60.0, n_ticks, 0.97, res)
        torch.cuda.synchronize()
        if i:
            wall.append((time.perf_counter() - t0) * 1e3)
    def summary(ms):
        fin = res.finish.cpu().numpy()[:J]
        done = fin >= 0
        return {"simulate_ms": ms, "ms_per_tick": ms / n_ticks, "ticks_per_s": n_ticks / (ms * 1e-3),
                "jobs_finished": int(done.sum()),
                "mean_jct_s": float(np.mean((fin - tr.arrival)[done])) if done.any() else None,
                "reconfigurations": int(res.n_reconf.cpu().numpy()[:J].sum()),
                "mean_gpus_in_use": float(res.gpus_in_use.cpu().numpy()[:n_ticks].mean())}
    out = {"entry": "rk_job_curves once + rk_simulate", "jobs": J, "gpus": int(wl.cluster.G), "ticks": n_ticks,
           "tick_s": 60.0, "gate": 0.97, "curves_ms": a.elapsed_time(b), **summary(float(np.median(wall)))}
    # the same trace with Algorithm 1's Schedule loop as the round of every tick (running jobs keep what they hold)
    wall = []
    for i in range(reps + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rk.rk_simulate(ctx, jobs.ref_thr, table.c, grid, cluster, bt, bp, ct, arrival, work_d, delta, 60.0, n_ticks, 0.97, res,
                       policy=1)
        torch.cuda.synchronize()
        if i:
            wall.append((time.perf_counter() - t0) * 1e3)
    out["schedule_loop_policy"] = summary(float(np.median(wall)))
    # the loop searching node by node needs CPU levels per GPU: the same jobs and trace on 8 nodes of 8 GPUs, 128 CPUs
    # and 512 GiB with CPU ratios {1, 2, 4, 8, 16} per GPU, under the loop over totals and under the loop over nodes
    wl2 = workloads.Workload("trace_scale_per_gpu", wl.coef, wl.ints, wl.bounds,
                             workloads.Grid(np.array([1, 2, 4, 8, 16], np.uint32), 1, np.array([64.0], np.float32), 0),
                             wl.env, workloads.Cluster(64, 8 * 128, 8 * 512.0))
    grid2, cluster2 = rk.make_grid(wl2.grid), rk.make_cluster(wl2.cluster)
    n2 = table.n_segments(len(wl2.grid.cpu_levels) * len(wl2.grid.mem_levels_gb))
    f32 = lambda: torch.empty(n2 + 4, dtype=torch.float32, device=dev)
    i32 = lambda: torch.empty(n2 + 4, dtype=torch.int32, device=dev)
    bt, bp, ct, cp, cg = f32(), i32(), f32(), i32(), i32()
    rk.rk_job_curves(ctx, jobs, table.c, grid2, env, 0, J, bt, bp, ct, cp, cg)
    nodes = rk.rk_nodes(8, 8, 128, 512.0)
    out["per_gpu_cpu_levels"] = {"nodes": 8, "gpus_per_node": 8, "cpus_per_node": 128, "mem_per_node_gb": 512.0}
    for key, policy in (("schedule_loop_policy", 1), ("schedule_loop_over_nodes_policy", 2)):
        wall = []
        for i in range(reps + 1):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rk.rk_simulate(ctx, jobs.ref_thr, table.c, grid2, cluster2, bt, bp, ct, arrival, work_d, delta, 60.0, n_ticks, 0.97,
                           res, policy=policy, nodes=nodes if policy == 2 else None)
            torch.cuda.synchronize()
            if i:
                wall.append((time.perf_counter() - t0) * 1e3)
        out["per_gpu_cpu_levels"][key] = summary(float(np.median(wall)))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="stress")
    ap.add_argument("--chunks", type=int, default=3, help="job chunks streamed through one candidate buffer")
    ap.add_argument("--cpu-sample-jobs", type=int, default=4000,
                    help="jobs of the workload the oracle is timed on (4,000 jobs of the stress workload: about 2.7e8 "
                         "candidates, 2.2 GB of float64 throughputs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-what-if", action="store_true")
    ap.add_argument("--no-place", action="store_true", help="skip the node-level placement")
    ap.add_argument("--no-sla", action="store_true")
    ap.add_argument("--no-fit", action="store_true")
    ap.add_argument("--no-sim", action="store_true")
    ap.add_argument("--what-if-rounds", type=int, default=256)
    ap.add_argument("--stream-calibration", action="store_true",
                    help="also run, five times each, a strided read of a chunk's candidate buffer and the evaluation with "
                         "the feasibility output (for profiles)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB elementwise copy (reads 1 GiB, writes 1 GiB) three times, "
                         "to scale the profiler's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("this benchmark measures one GPU; the path runs on a single device (use --gpus 1)")

    import torch
    import paper_2408_08586_amd as rk

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    rk.load_library()
    wl, desc = build_workload(args.workload)
    dev = "cuda:0"
    ctx = rk.rk_create(0)
    jobs = rk.Jobs(wl.coef, wl.ints, dev)
    bounds, grid, env = rk.make_bounds(wl.bounds), rk.make_grid(wl.grid), rk.make_env(wl.env)
    cluster = rk.make_cluster(wl.cluster)
    n_rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)

    # host <-> device copies of a round's inputs and outputs, apart from the kernels (inputs stay resident afterwards)
    torch.cuda.synchronize()
    h2d = []
    for _ in range(5):
        a = time.perf_counter()
        jobs = rk.Jobs(wl.coef, wl.ints, dev)
        torch.cuda.synchronize()
        h2d.append((time.perf_counter() - a) * 1e3)
    table = rk.enumerate_to_table(ctx, jobs, bounds, dev)      # sizes the buffers; enumeration is re-run per step
    J = wl.n_jobs
    n_chunks = max(1, min(args.chunks, J))
    edges = np.linspace(0, J, n_chunks + 1).astype(int)
    chunk_cands = [table.n_candidates(n_rows, int(a), int(b)) for a, b in zip(edges[:-1], edges[1:])]
    n_cand = table.n_candidates(n_rows)
    n_seg = table.n_segments(n_rows)
    thr = torch.empty(max(chunk_cands) + 4, dtype=torch.float32, device=dev)
    f32 = lambda n: torch.empty(n + 4, dtype=torch.float32, device=dev)
    i32 = lambda n: torch.empty(n + 4, dtype=torch.int32, device=dev)
    best_thr, best_plan = f32(n_seg), i32(n_seg)
    curve_thr, curve_plan, curve_g = f32(n_seg), i32(n_seg), i32(n_seg)
    assign = rk.new_assign(J, dev)
    total = torch.zeros(1, dtype=torch.float32, device=dev)
    seg_start = [n_rows * int(table.h_seg_off[a]) for a in edges[:-1]]
    seg_count = [table.n_segments(n_rows, int(a), int(b)) for a, b in zip(edges[:-1], edges[1:])]

    # Event records cost the stream a few microseconds each, so the timed steps carry only those that the roofline
    # needs (one before the first chunk's kernel, then one after every chunk's: 4 per step of 3 chunks); the duration
    # of every stage is measured in a pass of its own after the timed region, with events around every call, and so
    # is the same path with the evaluation and the best plan as two kernels (rk_eval_candidates, rk_best_plan).
    hot_ms = {"eval_best": []}
    stage_ms = {"enumerate": [], "eval_best": [], "curves": [], "allocate": []}
    pair_ms = {"eval": [], "best_plan": []}

    def mark():
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    def step(mode):
        """mode: None = no events, "hot" = events around the HBM-bound kernel, "all" = around every call, "pair" = the
        evaluation and the best plan as two kernels, events around both."""
        every = mode == "all"
        e0 = mark() if every else None
        rk.rk_enumerate_plans(ctx, jobs, bounds, table.c)
        if every:
            e1 = mark()
            stage_ms["enumerate"].append((e0, e1))
        c = None
        for k in range(n_chunks):
            jb, je = int(edges[k]), int(edges[k + 1])
            s0 = seg_start[k]
            a = (mark() if c is None else c) if mode else None   # the event after a chunk's kernel also opens the next
            if mode == "pair":
                rk.rk_eval_candidates(ctx, jobs, table.c, grid, env, jb, je, thr, None)
                b = mark()
                rk.rk_best_plan(ctx, table.c, grid, jb, je, thr, best_thr[s0:], best_plan[s0:])
                c = mark()
                pair_ms["eval"].append((a, b))
                pair_ms["best_plan"].append((b, c))
                continue
            # candidates of the chunk to thr, their per-segment maxima and plans to best_thr / best_plan, in one pass
            rk.rk_eval_best_plan(ctx, jobs, table.c, grid, env, jb, je, thr, best_thr[s0:], best_plan[s0:])
            if mode:
                c = mark()
                (stage_ms if every else hot_ms)["eval_best"].append((a, c))
        # the curves need only the per-segment maxima, which are small: one launch for all jobs
        e15 = mark() if every else None
        rk.rk_curves(ctx, table.c, grid, 0, J, best_thr, best_plan, curve_thr, curve_plan, curve_g)
        e2 = mark() if every else None
        if every:
            stage_ms["curves"].append((e15, e2))
        rk.rk_allocate(ctx, jobs.ref_thr, table.c, grid, cluster, 0, J, best_thr, best_plan, curve_thr, assign, total)
        if every:
            stage_ms["allocate"].append((e2, mark()))

    # What the chip gives kernels that do nothing but fill, then read, the candidate buffer of one chunk: the measured
    # ceiling of the one-pass kernel, whose launches follow each other (a fill that follows a fill), and of the k_eval +
    # k_best_plan pair (fill, then read).  A read that follows a write of the same buffer is slower than the same
    # read after another read (the written lines are still on their way to HBM), so both positions are timed.
    n_probe = (max(chunk_cands) // 4) * 4
    probe = {"fill": [], "fill_after_fill": [], "read_after_fill": [], "read_after_read": []}
    for i in range(7):
        e = [mark()]
        rk.rk_probe_stream(ctx, thr, n_probe, 1, 1.0)
        e.append(mark())
        rk.rk_probe_stream(ctx, thr, n_probe, 4, 2.0)
        e.append(mark())
        rk.rk_probe_stream(ctx, thr, n_probe, 0, out=total)
        e.append(mark())
        rk.rk_probe_stream(ctx, thr, n_probe, 3, out=total)
        e.append(mark())
        if i >= 2:
            for k, (x, y) in zip(probe, zip(e[:-1], e[1:])):
                probe[k].append((x, y))
    torch.cuda.synchronize()
    probe_ms = {k: sum(x.elapsed_time(y) for x, y in v) / len(v) for k, v in probe.items()}
    # the slope table of the curves (not part of the timed step: the allocation computes its steps itself)
    n_sl = table.n_segments(n_rows)
    sl_f = [torch.empty(n_sl + 4, dtype=torch.float32, device=dev) for _ in range(2)]
    sl_i = [torch.empty(n_sl + 4, dtype=torch.int32, device=dev) for _ in range(2)]
    sl_0 = (torch.empty(n_rows * J + 4, dtype=torch.float32, device=dev), torch.empty(n_rows * J + 4, dtype=torch.int32, device=dev))
    slopes = []
    for i in range(7):
        x = mark()
        rk.rk_curve_slopes(ctx, jobs.ref_thr, table.c, grid, 0, J, best_thr, curve_thr, sl_f[0][:n_sl], sl_i[0], sl_0[0], sl_0[1],
                           sl_f[1], sl_i[1])
        y = mark()
        if i >= 2:
            slopes.append((x, y))
    torch.cuda.synchronize()
    slopes_ms = sum(x.elapsed_time(y) for x, y in slopes) / len(slopes)
    del sl_f, sl_i, sl_0
    if args.stream_calibration:
        # for profiles: the strided read, and k_eval with the feasibility output, which the timed steps do not ask for
        feas = torch.empty(max(chunk_cands) + 16, dtype=torch.uint8, device=dev)
        for _ in range(5):
            rk.rk_probe_stream(ctx, thr, n_probe, 2, out=total)
            rk.rk_eval_candidates(ctx, jobs, table.c, grid, env, 0, int(edges[1]), thr, feas)
        torch.cuda.synchronize()
        del feas
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step("hot")
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    stage_steps = min(args.steps, 5)
    for _ in range(stage_steps):
        step("all")
    for _ in range(stage_steps):
        step("pair")
    torch.cuda.synchronize()
    mean_ms = lambda v: sum(a.elapsed_time(b) for a, b in v) / len(v) if v else 0.0
    avg_ms = {k: mean_ms(v) for k, v in stage_ms.items()}
    per_step_ms = {k: avg_ms[k] * (len(v) / stage_steps) for k, v in stage_ms.items()}
    hot_avg_ms = {k: mean_ms(v) for k, v in hot_ms.items()}
    pair_avg_ms = {k: mean_ms(v) for k, v in pair_ms.items()}

    # fused round (the path a scheduler would call): latency of rk_schedule_round
    for _ in range(2):
        rk.rk_schedule_round(ctx, jobs, bounds, grid, env, cluster, assign, total)
    torch.cuda.synchronize()
    lat = []
    for _ in range(max(5, args.steps)):
        a = time.perf_counter()
        rk.rk_schedule_round(ctx, jobs, bounds, grid, env, cluster, assign, total)
        torch.cuda.synchronize()
        lat.append((time.perf_counter() - a) * 1e3)
    lat = np.array(lat)
    # the same round when the curves are kept from an earlier round (Sec. 5.2: they do not depend on the cluster's
    # state and can be cached): only the allocation runs
    rk.rk_job_curves(ctx, jobs, table.c, grid, env, 0, J, best_thr, best_plan, curve_thr, curve_plan, curve_g)
    torch.cuda.synchronize()
    lat_cached = []
    for i in range(max(5, args.steps) + 2):
        a = time.perf_counter()
        rk.rk_allocate(ctx, jobs.ref_thr, table.c, grid, cluster, 0, J, best_thr, best_plan, curve_thr, assign, total)
        torch.cuda.synchronize()
        if i >= 2:
            lat_cached.append((time.perf_counter() - a) * 1e3)
    lat_cached = np.array(lat_cached)

    d2h = []
    for _ in range(5):
        a = time.perf_counter()
        rk.assign_to_numpy(assign)
        d2h.append((time.perf_counter() - a) * 1e3)

    # roofline of the dominant kernel (algorithmic bytes per launch / average launch duration)
    cand_per_launch = n_cand / n_chunks
    seg_per_launch = n_seg / n_chunks
    bytes_eval = 4.0 * cand_per_launch + 4.0 * table.n_triples / n_chunks
    bytes_best = 4.0 * cand_per_launch + 8.0 * seg_per_launch
    # the one-pass kernel writes every candidate once (4 B), reads the plan table (4 B per triple) and writes the
    # per-segment results (8 B per entry); it does not read the candidates back
    bytes_one = 4.0 * cand_per_launch + 4.0 * table.n_triples / n_chunks + 8.0 * seg_per_launch
    achieved = bytes_one / (hot_avg_ms["eval_best"] * 1e-3) / 1e9         # over the launches of the timed region
    gbs_eval = bytes_eval / (pair_avg_ms["eval"] * 1e-3) / 1e9
    gbs_best = bytes_best / (pair_avg_ms["best_plan"] * 1e-3) / 1e9
    pair_gbs = (bytes_eval + bytes_best) / ((pair_avg_ms["eval"] + pair_avg_ms["best_plan"]) * 1e-3) / 1e9

    digest = kernel_digest()
    traffic = None
    if args.workload == "stress" and n_chunks == 3:
        traffic = MEASURED_TRAFFIC.get(digest, {}).get("k_eval_best")
        if traffic is None:
            print(f"bench.py: the evaluation kernels' sources (digest {digest}) have changed since the HBM counters of "
                  f"profiles/hbm_traffic_stress.txt were taken: roofline.traffic is null until they are taken again",
                  file=sys.stderr)

    out = {
        "metric": "candidate plan evaluations/sec (whole path: enumerate + evaluate + best plan + curves + greedy), 1 GPU",
        "value": n_cand / (ms_per_step * 1e-3),
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": desc, "n_jobs": J, "n_candidates": n_cand, "n_segment_rows": n_seg,
                   "n_triples": table.n_triples, "job_chunks": n_chunks},
        "roofline": {"bound": "hbm", "kernel": "k_eval_best",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "duration_covers": "one rk_eval_best_plan call between two events: k_eval_best and the small "
                                        "k_merge_spanning that finishes the segments spanning tiles (rocprofv3 per kernel: "
                                        "profiles/whole_path_stress.txt)",
                     "algorithmic_bytes_per_launch": bytes_one,
                     "traffic": traffic, "traffic_source": "profiles/hbm_traffic_stress.txt (rocprofv3 --pmc FETCH_SIZE / "
                                                            "WRITE_SIZE, scaled by a plain copy's counters)",
                     "kernel_source_digest": digest,
                     # the same result with the candidates read back (rk_eval_candidates + rk_best_plan): twice the
                     # bytes at a higher rate, and a slower step; measured in a pass of its own (kernels.two_kernels)
                     "eval_then_best_plan": {"achieved": pair_gbs, "frac": pair_gbs / HBM_PEAK_GBS,
                                             "ms_per_chunk": pair_avg_ms["eval"] + pair_avg_ms["best_plan"],
                                             "one_pass_ms_per_chunk": hot_avg_ms["eval_best"]}},
        "kernels": {"timed_region_avg_launch_ms": hot_avg_ms,
                    "stage_pass": "separate pass after the timed region, events around every call",
                    "avg_launch_ms": avg_ms, "per_step_ms": per_step_ms,
                    "curve_slopes_ms": slopes_ms,
                    "eval_best_candidates_per_s": n_cand / (hot_avg_ms["eval_best"] * n_chunks * 1e-3),
                    # kernels that only fill and only read the same buffer (4 bytes per candidate each way)
                    "plain_stream_ms": probe_ms,
                    "eval_best_over_plain_fill_after_fill": hot_avg_ms["eval_best"] / probe_ms["fill_after_fill"],
                    # the same path with the candidates read back: rk_eval_candidates, then rk_best_plan
                    "two_kernels": {"pass": "separate pass after the timed region, events around both kernels",
                                    "avg_launch_ms": pair_avg_ms, "eval_GBps": gbs_eval, "best_plan_GBps": gbs_best,
                                    "eval_plus_best_plan_GBps": pair_gbs,
                                    "eval_plus_best_plan_frac_of_hbm": pair_gbs / HBM_PEAK_GBS,
                                    "eval_plus_best_plan_over_plain_fill_plus_read":
                                        (pair_avg_ms["eval"] + pair_avg_ms["best_plan"]) /
                                        (probe_ms["fill"] + probe_ms["read_after_fill"]),
                                    "eval_plus_best_plan_candidates_per_s":
                                        n_cand / ((pair_avg_ms["eval"] + pair_avg_ms["best_plan"]) * n_chunks * 1e-3)}},
        "round_latency_ms": {"entry": "rk_schedule_round (fused evaluation, host-synchronous)",
                             "min": float(lat.min()), "median": float(np.median(lat)), "max": float(lat.max()),
                             "with_cached_curves": {"entry": "rk_allocate on curves kept from an earlier round",
                                                    "min": float(lat_cached.min()), "median": float(np.median(lat_cached)),
                                                    "max": float(lat_cached.max())}},
    }
    out["transfers_ms"] = {"h2d_job_descriptors": float(np.median(h2d)), "h2d_bytes": int(wl.coef.nbytes + wl.ints.nbytes),
                           "d2h_assignment": float(np.median(d2h)), "d2h_bytes": int(J * 20),
                           "note": "pageable host arrays through torch; not part of any timed region"}
    # the fused kernel (evaluation + best plan + curves without the candidate tensor): bound by the vector ALUs
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(5, args.steps) + 2)]
    for a, b in ev:
        a.record()
        rk.rk_job_curves(ctx, jobs, table.c, grid, env, 0, J, best_thr, best_plan, curve_thr, curve_plan, curve_g)
        b.record()
    torch.cuda.synchronize()
    fused_ms = float(np.median([a.elapsed_time(b) for a, b in ev[2:]]))
    n_cpu = len(wl.grid.cpu_levels)
    # plans without offload once (8 per triple), the 4 offload plans that ZeRO stage >= 2 allows once per CPU level;
    # memory tiers only mask
    nt_all = table.n_triples
    unique = nt_all * (8 + 4 * n_cpu)
    fd = source_digest(FUSED_SOURCES)
    valu = MEASURED_FUSED_VALU.get(fd) if args.workload == "stress" else None
    if args.workload == "stress" and valu is None:
        print(f"bench.py: no instruction count on record for the fused kernel's sources (digest {fd}); its issue-slot "
              f"figure is reported as null until profiles/valu_stress.txt is taken again", file=sys.stderr)
    ops = sum(ALGO_OPS[k][0] * n for k, n in (("triple", nt_all), ("plain_plan", 8 * nt_all), ("offload_triple", nt_all),
                                              ("offload_level", n_cpu * nt_all)))
    trans = sum(ALGO_OPS[k][1] * n for k, n in (("triple", nt_all), ("plain_plan", 8 * nt_all), ("offload_triple", nt_all),
                                                ("offload_level", n_cpu * nt_all)))
    sec = fused_ms * 1e-3
    out["fused"] = {"entry": "rk_job_curves (k_fused)", "ms": fused_ms,
                    "nominal_candidates_per_s": n_cand / sec,
                    "unique_evaluations": unique, "unique_evaluations_per_s": unique / sec,
                    # algorithmic arithmetic against the vector-ALU ceilings: issue slots the model's own operations
                    # need (a quarter-rate operation takes four) over the slots the chip has in that time
                    "roofline_algorithmic": {"bound": "alu", "unit": "lane-operations/s",
                                             "float_ops_per_launch": ops, "quarter_rate_ops_per_launch": trans,
                                             "float_ops_per_s": ops / sec, "quarter_rate_ops_per_s": trans / sec,
                                             "peak_float": VALU_PEAK_LANE_INSTR, "peak_quarter_rate": TRANS_PEAK_LANE_INSTR,
                                             "frac_quarter_rate": trans / sec / TRANS_PEAK_LANE_INSTR,
                                             "frac": (ops + 4 * trans) / sec / VALU_PEAK_LANE_INSTR},
                    # every vector instruction the kernel issues (address arithmetic, keys and LDS traffic included)
                    "roofline": {"bound": "alu", "unit": "lane-instructions/s", "peak": VALU_PEAK_LANE_INSTR,
                                 "achieved": None if valu is None else valu * 64 / sec,
                                 "frac": None if valu is None else valu * 64 / sec / VALU_PEAK_LANE_INSTR,
                                 "valu_wave_instructions_per_launch": valu, "kernel_source_digest": fd,
                                 "count_source": "profiles/valu_stress.txt"}}
    if not args.no_place:
        rk.rk_schedule_round(ctx, jobs, bounds, grid, env, cluster, assign, total)
        out["placement"] = placement(rk, ctx, dev, wl, assign, max(5, args.steps))
    if not args.no_place:
        rk.rk_job_curves(ctx, jobs, table.c, grid, env, 0, J, best_thr, best_plan, curve_thr, curve_plan, curve_g)
        rk.rk_allocate(ctx, jobs.ref_thr, table.c, grid, cluster, 0, J, best_thr, best_plan, curve_thr, assign, total)
        out["algorithm1"] = algorithm1_bench(rk, ctx, dev, wl, jobs, table, grid, env, best_thr, best_plan, curve_thr, assign,
                                             max(5, args.steps))
    if not args.no_sla:
        out["sla_round"] = sla_round(rk, ctx, dev, wl, jobs, table, bounds, grid, env, cluster, best_plan, n_rows,
                                     max(5, args.steps))
    if not args.no_fit:
        out["fit"] = fit_bench(rk, ctx, dev, wl, env, 3)
    if not args.no_sim:
        out["simulation"] = sim_bench(rk, ctx, dev, 3)
    if not args.no_what_if:
        out["other_configurations"] = {"entry": "rk_schedule_round (fused evaluation, host-synchronous)",
                                       **other_rounds(rk, ctx, dev, args.workload, 20)}
        out["what_if"] = what_if_batch(rk, ctx, dev, args.what_if_rounds)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_jobs)
    rk.rk_destroy(ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
