#!/usr/bin/env python3
"""Writes tests/golden/stress_round.json: the CPU oracle's result of one whole
scheduling round on the stress workload (10,000 jobs).  Calls only the oracle
and the workload generator; takes a few minutes.  Usage: python tests/golden/make_stress_round.py"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle      # noqa: E402
import workloads   # noqa: E402


def main():
    wl = workloads.stress()
    threads = min(16, os.cpu_count() or 1)
    table = oracle.enumerate_plans(wl.ints, wl.bounds)
    bts, bps = [], []
    for jb in range(0, wl.n_jobs, 1000):          # evaluation in job chunks keeps the float64 array small
        thr, _ = oracle.eval_jobs(wl.coef, wl.ints, wl.bounds, table, wl.grid, wl.env, jb, jb + 1000,
                                  want_reason=False, n_threads=threads)
        bt, bp = oracle.best_plan(table, wl.grid, thr, jb, jb + 1000)
        bts.append(bt.astype(np.float32))
        bps.append(bp)
    bt, bp = np.concatenate(bts), np.concatenate(bps)
    ct, _, _ = oracle.curves(table, wl.grid, bt, bp)
    assign, total, gap = oracle.greedy(wl.coef[:, 16], table, wl.grid, wl.cluster, bt, bp, ct)
    sched = np.flatnonzero(assign["g"] > 0)
    out = {
        "_about": "Oracle result of one scheduling round on workloads.stress() (seed 0x52554249): records of the "
                  "scheduled jobs (all others are unscheduled), total normalised throughput, smallest relative slope "
                  "gap met by the greedy.  Written by tests/golden/make_stress_round.py.",
        "n_jobs": int(wl.n_jobs), "n_triples": int(len(table.triples)), "n_segments": int(len(table.seg_g)),
        "total": total, "min_gap": gap,
        "scheduled": [[int(j), int(assign["g"][j]), int(assign["c"][j]), float(assign["mem_gb"][j]),
                       int(assign["plan"][j]), float(assign["thr"][j])] for j in sched],
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "stress_round.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=0)
    print("wrote", path, len(sched), "scheduled jobs, total", total, "min gap", gap)


if __name__ == "__main__":
    main()
