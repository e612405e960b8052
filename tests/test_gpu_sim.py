"""GPU parity of the discrete-time simulation with the reconfiguration-penalty
gate (paper Sec. 5.2, 7.4) against the CPU oracle: on shared float32 curves
every per-job and per-tick result must be identical."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def run_on_gpu(run, r, arrival, work, delta, dt, n_ticks, gate, cluster=None, curves=None, policy=0, nodes=None):
    import paper_2408_08586_amd as rk
    torch = run.torch
    J = run.wl.n_jobs
    f64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).to(run.device)
    res = rk.SimResult(J, n_ticks, run.device)
    bt, bp, ct = curves if curves is not None else (run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]),
                                                    run.dev_f32(r["curve_thr"]))
    rk.rk_simulate(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster if cluster is None else cluster, bt, bp, ct,
                   f64(arrival), f64(work), f64(delta), dt, n_ticks, gate, res, policy=policy,
                   nodes=None if nodes is None else rk.rk_nodes(*nodes))
    rk.rk_sync(run.ctx)
    return dict(finish=res.finish.cpu().numpy()[:J], n_reconf=res.n_reconf.cpu().numpy()[:J].view(np.uint32),
                progress=res.progress.cpu().numpy()[:J], held=res.held.cpu().numpy()[:J],
                gpus_in_use=res.gpus_in_use.cpu().numpy()[:n_ticks].view(np.uint32),
                totals=res.totals.cpu().numpy()[:n_ticks], frozen=res.frozen.cpu().numpy()[:n_ticks].view(np.uint32))


def same(got, want):
    for k in ("finish", "n_reconf", "progress", "held", "gpus_in_use", "frozen"):
        assert np.array_equal(got[k], want[k]), k
    assert np.allclose(got["totals"], want["totals"], rtol=1e-6, atol=1e-12)


@pytest.mark.parametrize("name,hours,dt,n_ticks,scale", [("tiny", 0.5, 30.0, 200, 1.0), ("paper_scale", 2.0, 60.0, 300, 4.0),
                                                         ("large", 4.0, 120.0, 150, 2.0)])
def test_simulation_is_identical_on_shared_curves(gpu, orc, name, hours, dt, n_ticks, scale):
    wl = workloads.CONFIGS[name]()
    r = orc.schedule_round(wl, n_threads=16)
    tr = workloads.trace(wl.n_jobs, horizon_s=hours * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * scale
    run = gpu(wl)
    run.enumerate()
    for gate in (0.97, -np.inf, 1.0):
        want = orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                      r["curve_thr"], tr.arrival, work, tr.delta, dt, n_ticks, gate=gate)
        got = run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, gate)
        same(got, want)
        if gate == 0.97:
            fin = want["finish"] >= 0
            print(f"{name}: {int(fin.sum())}/{wl.n_jobs} jobs finish, {int(want['n_reconf'].sum())} reconfigurations, "
                  f"{int(want['frozen'].sum())} frozen job-ticks, mean JCT {np.mean((want['finish'] - tr.arrival)[fin]):.0f} s")
            assert fin.sum() > 0 and want["n_reconf"].sum() > 0 and want["frozen"].sum() > 0
    # a second run on the same context starts from a clean state
    got2 = run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, 1.0)
    same(got2, got)
    run.close()


@pytest.mark.parametrize("name,hours,dt,n_ticks,scale", [("tiny", 0.5, 30.0, 200, 1.0), ("paper_scale", 2.0, 60.0, 300, 4.0),
                                                         ("large", 4.0, 120.0, 150, 2.0)])
def test_simulation_with_the_loop_as_its_policy(gpu, orc, name, hours, dt, n_ticks, scale):
    """Algorithm 1's Schedule loop every tick (frozen jobs in state 2) instead of the greedy from scratch."""
    wl = workloads.CONFIGS[name]()
    r = orc.schedule_round(wl, n_threads=16)
    tr = workloads.trace(wl.n_jobs, horizon_s=hours * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * scale
    run = gpu(wl)
    run.enumerate()
    for gate in (0.97, -np.inf, 1.0):
        want = orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                      r["curve_thr"], tr.arrival, work, tr.delta, dt, n_ticks, gate=gate, policy="loop")
        got = run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, gate, policy=1)
        same(got, want)
        if gate == 0.97:
            fin = want["finish"] >= 0
            print(f"{name}, loop: {int(fin.sum())}/{wl.n_jobs} jobs finish, {int(want['n_reconf'].sum())} reconfigurations, "
                  f"{int(want['frozen'].sum())} frozen job-ticks, mean JCT {np.mean((want['finish'] - tr.arrival)[fin]):.0f} s")
            assert fin.sum() > 0
    # the two policies on one context, one after the other: neither leaves anything behind for the other
    a = run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, 0.97, policy=0)
    b = run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, 0.97, policy=1)
    same(a, orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"], r["curve_thr"],
                                   tr.arrival, work, tr.delta, dt, n_ticks))
    same(b, orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"], r["curve_thr"],
                                   tr.arrival, work, tr.delta, dt, n_ticks, policy="loop"))
    run.close()


@pytest.mark.parametrize("name", ["large", "trace_scale"])
def test_simulation_over_nodes(gpu, orc, name):
    """The loop with ScheduleJob searching node by node as the round of every tick: where the jobs are is carried from
    tick to tick on the device as in the oracle's simulation."""
    if name == "large":
        wl, nodes, hours, dt, n_ticks, scale = workloads.large(), (128, 8, 128, 2048.0), 4.0, 120.0, 100, 2.0
    else:                                                    # the trace experiment's shape with CPUs per GPU
        base = workloads.trace_scale()
        grid = workloads.Grid(np.array([1, 2, 4, 8, 16], np.uint32), 1, np.array([64.0], np.float32), 0)
        wl = workloads.Workload("trace_scale_per_gpu", base.coef, base.ints, base.bounds, grid, base.env,
                                workloads.Cluster(64, 8 * 128, 8 * 512.0))
        nodes, hours, dt, n_ticks, scale = (8, 8, 128, 512.0), 12.0, 60.0, 360, 4.0
    r = orc.schedule_round(wl, n_threads=16)
    tr = workloads.trace(wl.n_jobs, horizon_s=hours * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * scale
    run = gpu(wl)
    run.enumerate()
    for gate in (0.97, -np.inf):
        want = orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                      r["curve_thr"], tr.arrival, work, tr.delta, dt, n_ticks, gate=gate, policy="nodes",
                                      nodes=nodes)
        got = run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, gate, policy=2, nodes=nodes)
        same(got, want)
        if gate == 0.97:
            fin = want["finish"] >= 0
            print(f"{name}, over nodes: {int(fin.sum())}/{wl.n_jobs} jobs finish, {int(want['n_reconf'].sum())} reconfigurations, "
                  f"{int(want['frozen'].sum())} frozen job-ticks, mean GPUs in use {want['gpus_in_use'].mean():.1f}")
            assert fin.sum() > 0
    # the other policies still run on this context afterwards
    same(run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, 20, 0.97, policy=1),
         orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"], r["curve_thr"],
                                tr.arrival, work, tr.delta, dt, 20, policy="loop"))
    import paper_2408_08586_amd as rk
    with pytest.raises(rk.RkError) as e:
        run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, 5, 0.97, policy=2)            # no nodes
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    run.close()


def test_simulation_end_to_end_on_device_curves(gpu, orc):
    """Curves computed by the library itself (float32 model): the trajectory may
    part from the oracle's at a near-tie, so the aggregate figures are compared."""
    wl = workloads.paper_scale()
    r = orc.schedule_round(wl, n_threads=16)
    tr = workloads.trace(wl.n_jobs, horizon_s=2 * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * 4.0
    want = orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                  r["curve_thr"], tr.arrival, work, tr.delta, 60.0, 300)
    run = gpu(wl)
    run.enumerate()
    bt, bp, ct, cp, cg, n = run.fused()
    got = run_on_gpu(run, r, tr.arrival, work, tr.delta, 60.0, 300, 0.97, curves=(bt, bp, ct))
    fin_w, fin_g = want["finish"] >= 0, got["finish"] >= 0
    identical = all(np.array_equal(got[k], want[k]) for k in ("n_reconf", "gpus_in_use", "frozen"))
    print(f"end to end: trajectories identical: {identical}; finished {int(fin_g.sum())} vs {int(fin_w.sum())}")
    assert abs(int(fin_g.sum()) - int(fin_w.sum())) <= 2
    both = fin_w & fin_g
    jct_w, jct_g = np.mean((want["finish"] - tr.arrival)[both]), np.mean((got["finish"] - tr.arrival)[both])
    assert jct_g == pytest.approx(jct_w, rel=2e-2)
    assert np.all(got["gpus_in_use"] <= wl.cluster.G)
    if identical:
        assert np.allclose(got["finish"], want["finish"], rtol=1e-5)
    run.close()


def test_simulation_from_a_side_stream(gpu, orc):
    """The context sits on a stream of its own; the simulation's internal stream is ordered after the uploads made
    on that stream and the results are read on it afterwards."""
    import torch
    wl = workloads.paper_scale()
    r = orc.schedule_round(wl, n_threads=16)
    tr = workloads.trace(wl.n_jobs, horizon_s=3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * 2.0
    want = orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                  r["curve_thr"], tr.arrival, work, tr.delta, 60.0, 90)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run = gpu(wl)
        run.enumerate()
        for _ in range(2):
            same(run_on_gpu(run, r, tr.arrival, work, tr.delta, 60.0, 90, 0.97), want)
        run.close()


def test_simulation_edge_cases(gpu, orc):
    import paper_2408_08586_amd as rk
    wl = workloads.tiny()
    r = orc.schedule_round(wl, n_threads=4)
    run = gpu(wl)
    run.enumerate()
    J = wl.n_jobs
    # nobody ever arrives; everybody arrives at once with no work to speak of
    never = run_on_gpu(run, r, np.full(J, 1e12), np.ones(J), np.ones(J), 10.0, 5, 0.97)
    assert np.all(never["finish"] == -1) and np.all(never["gpus_in_use"] == 0) and np.all(never["progress"] == 0)
    want = orc.simulator.simulate(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                  r["curve_thr"], np.zeros(J), np.full(J, 1e-3), np.zeros(J), 10.0, 12)
    same(run_on_gpu(run, r, np.zeros(J), np.full(J, 1e-3), np.zeros(J), 10.0, 12, 0.97), want)
    assert np.all(want["finish"] >= 0)
    # an empty cluster
    empty = run_on_gpu(run, r, np.zeros(J), np.ones(J), np.ones(J), 10.0, 3, 0.97, cluster=rk.make_cluster(workloads.Cluster(0, 0, 0.0)))
    assert np.all(empty["finish"] == -1) and np.all(empty["gpus_in_use"] == 0)
    # argument errors
    f64 = lambda a: run.torch.from_numpy(np.asarray(a, np.float64)).to(run.device)
    res = rk.SimResult(J, 4, run.device)
    bt, bp, ct = run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]), run.dev_f32(r["curve_thr"])
    for dt, gate in ((0.0, 0.97), (-1.0, 0.97), (10.0, float("nan"))):
        with pytest.raises(rk.RkError) as e:
            rk.rk_simulate(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, bt, bp, ct, f64(np.zeros(J)),
                           f64(np.ones(J)), f64(np.ones(J)), dt, 4, gate, res)
        assert e.value.code == rk.RK_ERR_INVALID_ARG
    run.close()


def test_simulation_with_more_jobs_than_one_workgroup_selects(gpu, orc):
    """3,000 jobs per tick: the allocation takes its multi-workgroup path, with
    inactive and frozen jobs in it."""
    wl = workloads.stress(n_jobs=3000)
    wl.cluster = workloads.Cluster(1024, 128 * 128, 128 * 2048.0)
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    bts, bps = [], []
    for jb in range(0, wl.n_jobs, 500):
        thr, _ = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, jb, jb + 500, want_reason=False, n_threads=16)
        bt, bp = orc.best_plan(ot, wl.grid, thr, jb, jb + 500)
        bts.append(bt.astype(np.float32))
        bps.append(bp)
    bt, bp = np.concatenate(bts), np.concatenate(bps)
    ct, _, _ = orc.curves(ot, wl.grid, bt, bp)
    r = dict(table=ot, best_thr=bt, best_plan=bp, curve_thr=ct)
    tr = workloads.trace(wl.n_jobs, horizon_s=1800.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * 0.2
    n_ticks, dt = 24, 120.0
    want = orc.simulator.simulate(wl.coef[:, 16], ot, wl.grid, wl.cluster, bt, bp, ct, tr.arrival, work, tr.delta, dt, n_ticks)
    run = gpu(wl)
    run.enumerate()
    got = run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, 0.97)
    same(got, want)
    print(f"3000 jobs: {int((want['finish'] >= 0).sum())} finish, {int(want['n_reconf'].sum())} reconfigurations, "
          f"{int(want['frozen'].sum())} frozen job-ticks, GPUs in use at the end {int(want['gpus_in_use'][-1])}")
    assert want["frozen"].sum() > 0 and (want["finish"] >= 0).sum() > 0
    run.close()
