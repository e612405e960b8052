"""GPU parity at the full size of the two largest configurations.

Stress (10,000 jobs, 6.8e8 candidates): every job, 1,000 at a time - the plan
table bit for bit, every throughput within 1e-5 relative, every feasibility
mask bit for bit, every best plan equal to the oracle's or inside the 1e-5
band of its maximum, the best-plan and curve kernels bit for bit on the
oracle's own float32 values, the one-pass and the fused entry points bit for
bit what the separate calls give.

What-if batch (rounds of 500 jobs on about 512 GPUs): whole rounds through
rk_schedule_rounds and rk_schedule_rounds_shared against the oracle's rounds.
RK_WHAT_IF_ROUNDS sets how many of the 256 rounds are compared (default: all 256)."""
import os
import time

import numpy as np
import pytest

import workloads
from test_gpu_parity import check_best_in_band, check_thr, compare_rounds, oracle_table_equal, own_values

pytestmark = pytest.mark.gpu

THREADS = 16


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def test_stress_every_job(gpu, orc, capsys):
    import torch
    wl = workloads.stress()
    t0 = time.time()
    ot = orc.enumerate_plans(wl.ints, wl.bounds, n_threads=THREADS)
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    with capsys.disabled():
        print(f"\n  stress: plan table of {wl.n_jobs} jobs equal ({ot.triples.shape[0]} triples, {time.time() - t0:.0f} s)", flush=True)
    worst, n_mis, n_seg, n_cand = 0.0, 0, 0, 0
    step = 1000
    for jb in range(0, wl.n_jobs, step):
        je = min(jb + step, wl.n_jobs)
        o_thr, o_reason = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, jb, je, n_threads=THREADS)
        thr, feas, n = run.eval(jb, je)
        assert n == o_thr.size
        worst = max(worst, check_thr(run.host(thr, n), run.host(feas, n), o_thr, o_reason))
        # best plan from the library's own values: the oracle's float64 choice, or inside its band
        bt, bp, ns = run.best(thr, jb, je)
        o_bt, o_bp = orc.best_plan(ot, wl.grid, o_thr, jb, je, n_threads=THREADS)
        g_bt, g_bp = run.host(bt, ns), run.host(bp, ns).view(np.uint32)
        n_mis += check_best_in_band(ot, run.n_rows, jb, je, o_thr, o_bt, o_bp, g_bt, g_bp)
        # evaluation and best plan in one pass: the same bits as the two calls
        t1, f1, b1, p1, n1, ns1 = run.eval_best(jb, je)
        assert (n1, ns1) == (n, ns)
        assert torch.equal(t1[:n], thr[:n]) and torch.equal(f1[:n], feas[:n])
        assert torch.equal(b1[:ns].view(torch.int32), bt[:ns].view(torch.int32)) and torch.equal(p1[:ns], bp[:ns])
        del t1, f1, b1, p1
        # the fused entry point gives the same bits as evaluation -> best plan -> curves
        ct, cp, cg = run.curves(bt, bp, jb, je)
        fused = run.fused(jb, je)
        for a, b in zip(fused[:5], (bt, bp, ct, cp, cg)):
            assert np.array_equal(run.host(a, ns), run.host(b, ns))
        # best plan and curves on values both sides share (the oracle's, rounded to float32): bit for bit
        o32 = o_thr.astype(np.float32)
        e_bt, e_bp = orc.best_plan(ot, wl.grid, o32, jb, je, n_threads=THREADS)
        bt2, bp2, _ = run.best(run.dev_f32(o32), jb, je)
        assert np.array_equal(run.host(bt2, ns), e_bt) and np.array_equal(run.host(bp2, ns).view(np.uint32), e_bp)
        ct2, cp2, cg2 = run.curves(bt2, bp2, jb, je)
        for got, want in zip((ct2, cp2, cg2), orc.curves(ot, wl.grid, e_bt, e_bp, jb, je)):
            assert np.array_equal(run.host(got, ns).view(want.dtype), want)
        n_seg += ns
        n_cand += n
        with capsys.disabled():
            print(f"  stress: jobs [{jb}, {je}) equal; {n_cand} candidates so far, max rel err {worst:.2e}, "
                  f"{n_mis}/{n_seg} best plans differ inside the band ({time.time() - t0:.0f} s)", flush=True)
    assert n_cand == 16 * run.n_rows * ot.triples.shape[0]
    assert n_mis <= 0.01 * n_seg
    run.close()


def test_what_if_full_rounds(gpu, orc, capsys):
    import paper_2408_08586_amd as rk
    import torch
    n_rounds = int(os.environ.get("RK_WHAT_IF_ROUNDS", "256"))
    t0 = time.time()
    rounds = [workloads.what_if(r) for r in range(n_rounds)]
    assert all(w.n_jobs == 500 for w in rounds)
    base = rounds[0]
    cat = workloads.Workload("batch", np.concatenate([w.coef for w in rounds]), np.concatenate([w.ints for w in rounds]),
                             base.bounds, base.grid, base.env, base.cluster)
    run = gpu(cat)
    round_off = (np.arange(n_rounds + 1) * 500).astype(np.uint32)
    clusters = [rk.make_cluster(w.cluster) for w in rounds]
    assign = rk.new_assign(cat.n_jobs)
    totals = torch.zeros(n_rounds, dtype=torch.float32, device="cuda:0")
    rk.rk_schedule_rounds(run.ctx, run.jobs, run.bounds, run.grid, run.env, round_off, clusters, assign, totals)
    rk.rk_sync(run.ctx)
    a = rk.assign_to_numpy(assign)
    # the same rounds over their distinct jobs: record for record what the concatenated batch gives
    swl, s_off, s_jobs, s_clusters = workloads.what_if_shared(n_rounds)
    run_s = gpu(swl)
    assign_s = rk.new_assign(len(s_jobs))
    totals_s = torch.zeros(n_rounds, dtype=torch.float32, device="cuda:0")
    rk.rk_schedule_rounds_shared(run_s.ctx, run_s.jobs, run_s.bounds, run_s.grid, run_s.env, s_off, s_jobs,
                                 [rk.make_cluster(c) for c in s_clusters], assign_s, totals_s)
    rk.rk_sync(run_s.ctx)
    assert np.array_equal(a, rk.assign_to_numpy(assign_s)) and torch.equal(totals, totals_s)
    n_same, gaps = 0, []
    for i, w in enumerate(rounds):
        r = orc.schedule_round(w, n_threads=THREADS)
        one = gpu(w)
        same = compare_rounds(orc, w, a[i * 500:(i + 1) * 500], float(totals[i].item()), r, own_values(one))
        one.close()
        piece = a[i * 500:(i + 1) * 500]
        assert piece["g"].sum() <= w.cluster.G and piece["c"].sum() <= w.cluster.C
        n_same += bool(same)
        gaps.append(r["min_gap"])
        if (i + 1) % 16 == 0 or i + 1 == n_rounds:
            with capsys.disabled():
                print(f"\n  what-if: {i + 1} rounds compared, {n_same} with records equal to the oracle's "
                      f"({time.time() - t0:.0f} s)", flush=True)
    with capsys.disabled():
        print(f"  what-if: smallest slope gaps of the oracle's rounds from {min(gaps):.1e} to {max(gaps):.1e}", flush=True)
    # observed on all 256 rounds: every record equals the oracle's own round
    assert n_same == n_rounds
    run.close()
    run_s.close()
