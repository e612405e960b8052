"""GPU parity on randomly drawn small workloads: bounds, option masks, grids
in both modes, GPU memory caps and clusters vary from case to case (seeded),
jobs without any plan are mixed in, and every stage of the path is compared
with the CPU oracle as in the tests of the named configurations."""
import dataclasses

import numpy as np
import pytest

import workloads
from test_gpu_parity import check_best_in_band, check_thr, compare_rounds, oracle_table_equal
from test_gpu_sim import run_on_gpu, same
from test_gpu_sla import random_requests

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def draw_workload(rng, base, wide=False, mid=False):
    """A workload of a few jobs; wide: jobs with hundreds of GPU counts, a small grid; mid: hundreds of jobs with
    up to 256 GPUs each, a small grid."""
    if wide:
        n_jobs = int(rng.integers(1, 7))
        ints = np.stack([rng.choice([96, 60, 48, 120, 12, 7], n_jobs), rng.choice([5040, 2520, 1680, 720, 360, 64, 30], n_jobs),
                         rng.choice([1, 1, 2, 3], n_jobs)], 1).astype(np.uint32)
        g_max, pp_max = int(rng.choice([96, 128, 256, 720, 1024])), int(rng.choice([4, 16, 255]))
        n_cpu, n_mem = int(rng.integers(1, 4)), int(rng.integers(1, 3))
    else:
        n_jobs = int(rng.integers(48, 700)) if mid else int(rng.integers(1, 48))
        ints = np.stack([rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 24, 30, 32, 36, 40, 48, 60, 64, 80, 96], n_jobs),
                         rng.choice([1, 2, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256, 360], n_jobs),
                         rng.choice([1, 1, 1, 2, 2, 3, 4, 8], n_jobs)], 1).astype(np.uint32)
        for k in range(n_jobs):
            if rng.uniform() < 0.03:
                ints[k, rng.integers(0, 3)] = 0                      # no layers, no batch or no micro-batch: no plan
        g_max = int(rng.choice([16, 40, 64, 100, 128, 200, 256] if mid else [1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64]))
        pp_max = int(rng.choice([1, 2, 3, 4, 8, 16]))
        n_cpu, n_mem = (int(rng.integers(1, 5)), int(rng.integers(1, 4))) if mid else (int(rng.integers(1, 9)), int(rng.integers(1, 7)))
    coef = base.coef[rng.integers(0, base.coef.shape[0], n_jobs)].copy()
    b = workloads.Bounds(g_max=g_max, tp_max=int(rng.choice([1, 2, 4, 8])), pp_max=pp_max, zero_mask=int(rng.integers(1, 16)),
                         gc_mask=int(rng.integers(1, 4)), off_mask=int(rng.integers(1, 4)), mu_mask=int(rng.integers(1, 16)))
    cpu = np.sort(rng.choice(np.arange(1, 33), n_cpu, replace=False)).astype(np.uint32)
    mem = np.sort(rng.choice(np.array([0, 4, 8, 16, 32, 64, 100, 256, 1024], np.float32), n_mem, replace=False))
    grid = workloads.Grid(cpu, int(rng.integers(0, 2)), mem.astype(np.float32), int(rng.integers(0, 2)))
    env = dataclasses.replace(base.env, gpu_mem_cap=float(rng.choice([1e9, 2e9, 4e9, 8e9, 16e9, 40e9, 80e9])),
                              gpus_per_node=int(rng.choice([1, 2, 4, 8])))
    G = int(rng.integers(0, 2 * g_max + 2))
    cl = workloads.Cluster(G, int(rng.integers(0, 40 * max(G, 1))), float(rng.choice([0.0, 16.0, 100.0, 1000.0, 1e6])))
    return workloads.Workload("random", coef, ints, b, grid, env, cl)


def check_path(gpu, orc, wl, rng):
    """Every stage against the oracle; returns the number of candidates compared."""
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    if int(np.diff(ot.triple_off).max()) > 2048:
        return 0                                                     # beyond the library's documented width
    r = orc.schedule_round(wl, n_threads=8)
    run = gpu(wl)
    try:
        run.enumerate()
        oracle_table_equal(run.table_numpy(), ot)
        if ot.triple_off[-1] == 0:
            a, t = run.schedule_round()
            assert (a["g"] == 0).all() and t == 0.0
            return 0
        thr, feas, n = run.eval()
        check_thr(run.host(thr, n), run.host(feas, n), r["thr"], r["reason"])
        o32 = r["thr"].astype(np.float32)
        bt, bp, ns = run.best(run.dev_f32(o32))
        e_bt, e_bp = orc.best_plan(ot, wl.grid, o32)
        assert np.array_equal(run.host(bt, ns), e_bt) and np.array_equal(run.host(bp, ns).view(np.uint32), e_bp)
        ct, cp, cg = run.curves(bt, bp)
        for got, want in zip((ct, cp, cg), orc.curves(ot, wl.grid, e_bt, e_bp)):
            assert np.array_equal(run.host(got, ns).view(want.dtype), want)
        bt2, bp2, _ = run.best(thr)
        o_bt, o_bp = orc.best_plan(ot, wl.grid, r["thr"])
        check_best_in_band(ot, run.n_rows, 0, wl.n_jobs, r["thr"], o_bt, o_bp, run.host(bt2, ns), run.host(bp2, ns).view(np.uint32))
        fused = run.fused()
        for a, c in zip(fused[:5], (bt2, bp2) + run.curves(bt2, bp2)):
            assert np.array_equal(run.host(a, ns), run.host(c, ns))
        assign, _ = run.allocate(run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]), run.dev_f32(r["curve_thr"]))
        assert np.array_equal(assign, r["assign"])
        own = (run.host(fused[0], ns).copy(), run.host(fused[1], ns).view(np.uint32).copy(), run.host(fused[2], ns).copy())
        compare_rounds(orc, wl, *run.schedule_round(), r, own)
        # a job range gives the same bits as the full call
        jb = int(rng.integers(0, wl.n_jobs))
        je = int(rng.integers(jb, wl.n_jobs + 1))
        t3, _, n3 = run.eval(jb, je, want_feas=False)
        at = 16 * run.n_rows * int(ot.triple_off[jb])
        assert np.array_equal(run.host(t3, n3), run.host(thr, n)[at:at + n3])
        if n3:
            sa = run.n_rows * int(ot.seg_off[jb])
            f3 = run.fused(jb, je)
            ns3 = f3[5]
            for a, c in zip(f3[:5], fused[:5]):
                assert np.array_equal(run.host(a, ns3), run.host(c, ns)[sa:sa + ns3])
        return n
    finally:
        run.close()


def test_random_small_workloads(gpu, orc):
    base = workloads.paper_scale()
    n = 0
    for seed in range(300):
        rng = np.random.default_rng(90000 + seed)
        n += check_path(gpu, orc, draw_workload(rng, base), rng)
    print(f"300 random workloads, {n} candidates compared")
    assert n > 10 ** 7


def test_random_mid_size_workloads(gpu, orc):
    base = workloads.paper_scale()
    n = 0
    for seed in range(60):
        rng = np.random.default_rng(93000 + seed)
        n += check_path(gpu, orc, draw_workload(rng, base, mid=True), rng)
    print(f"60 random workloads of 48 to 699 jobs, {n} candidates compared")
    assert n > 10 ** 7


def test_random_wide_workloads(gpu, orc):
    base = workloads.paper_scale()
    n = 0
    for seed in range(150):
        rng = np.random.default_rng(91000 + seed)
        n += check_path(gpu, orc, draw_workload(rng, base, wide=True), rng)
    print(f"150 random workloads of wide jobs, {n} candidates compared")
    assert n > 10 ** 6


def test_random_service_levels_placement_and_simulation(gpu, orc):
    """On the oracle's float32 curves, so that every record must be identical: minimum demands, the allocation from
    floors under quotas, the node-level placement of its result, and a short simulation."""
    import torch
    import paper_2408_08586_amd as rk
    base = workloads.paper_scale()
    done = 0
    for seed in range(150):
        rng = np.random.default_rng(92000 + seed)
        wl = draw_workload(rng, base)
        r = orc.schedule_round(wl, n_threads=8)
        ot, J = r["table"], wl.n_jobs
        if ot.triple_off[-1] == 0:
            continue
        n_cpu, n_mem = len(wl.grid.cpu_levels), len(wl.grid.mem_levels_gb)
        bt, bp, ct = r["best_thr"], r["best_plan"], r["curve_thr"]
        run = gpu(wl)
        run.enumerate()
        d_bt, d_bp, d_ct = run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct)
        guaranteed, req_g, req_c, req_m, b0 = random_requests(rng, ot, J, n_cpu, n_mem, bt, n_cpu * n_mem,
                                                              frac=float(rng.uniform(0, 1)))
        n_ten = int(rng.integers(1, 9))
        tenant = rng.integers(0, n_ten + 1, J).astype(np.uint32)
        sla = rk.Sla(guaranteed, tenant, [1] * n_ten, [1] * n_ten, req_g, req_c, req_m, b0)
        ms, mc, mm = run.i32(J), run.i32(J), run.i32(J)
        rk.rk_min_res(run.ctx, run.table.c, run.grid, 0, J, d_bt, sla, ms, mc, mm)
        rk.rk_sync(run.ctx)
        e_s, e_c, e_m = orc.min_res(ot, wl.grid, bt, guaranteed, req_g, req_c, req_m, b0)
        assert np.array_equal(run.host(ms, J), e_s)
        assert np.array_equal(rk.u32(mc)[:J], e_c) and np.array_equal(rk.u32(mm)[:J], e_m)
        w = rng.uniform(0.5, 1.5, n_ten)
        w = w / w.sum() * float(rng.choice([0.2, 0.6, 1.0, 3.0]))
        quota_g, quota_c = np.floor(w * wl.cluster.G).astype(np.uint32), np.floor(w * wl.cluster.C).astype(np.uint32)
        e_assign, e_total, _ = orc.policy(wl.coef[:, 16], ot, wl.grid, wl.cluster, bt, bp, ct, guaranteed, tenant, e_s, e_c,
                                          quota_g, quota_c)
        assign, total = rk.new_assign(J, run.device), run.f32(1)
        rk.rk_allocate_sla(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, 0, J, d_bt, d_bp, d_ct,
                           rk.Sla(guaranteed, tenant, quota_g, quota_c), torch.from_numpy(e_s).to(run.device), run.dev_u32(e_c),
                           assign, total)
        rk.rk_sync(run.ctx)
        assert np.array_equal(rk.assign_to_numpy(assign), e_assign)
        assert float(total[0].item()) == pytest.approx(e_total, rel=1e-6, abs=1e-12)
        # placement of that allocation on nodes that may be too few or short of CPUs and memory
        gpn = int(rng.choice([1, 2, 4, 8]))
        n_nodes = int(max(1, -(-int(e_assign["g"].sum()) // gpn) + rng.integers(-1, 3)))
        cpn, mpn = int(rng.choice([gpn, 4 * gpn, 16 * gpn, 40 * gpn])), float(rng.choice([0.0, 64.0, 512.0, 1e5]))
        w_off, w_ent, w_st = orc.place(e_assign, n_nodes, gpn, cpn, mpn)
        cap = n_nodes * gpn
        off = torch.full((J + 1,), -1, dtype=torch.int32, device=run.device)
        status = torch.full((J,), -1, dtype=torch.int32, device=run.device)
        ent = rk.new_place_entries(cap, run.device)
        res = rk.rk_place(run.ctx, rk.rk_nodes(n_nodes, gpn, cpn, mpn), J, assign, off, ent, cap, status)
        assert np.array_equal(rk.u32(off), w_off) and np.array_equal(rk.u32(status)[:J], w_st)
        assert res.n_entries == len(w_ent)
        g_ent = rk.place_entries_to_numpy(ent, res.n_entries)
        for f in ("node", "g", "c", "mem_gb"):
            assert np.array_equal(g_ent[f], w_ent[f]), f
        # a short simulation
        tr = workloads.trace(J, horizon_s=600.0, seed=int(rng.integers(0, 1 << 30)))
        work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * float(rng.choice([0.01, 0.1, 1.0]))
        dt, n_ticks = float(rng.choice([10.0, 60.0])), int(rng.integers(1, 25))
        gate = float(rng.choice([0.97, 0.5, 1.0, -np.inf]))
        want = orc.simulator.simulate(wl.coef[:, 16], ot, wl.grid, wl.cluster, bt, bp, ct, tr.arrival, work, tr.delta, dt,
                                      n_ticks, gate=gate)
        same(run_on_gpu(run, r, tr.arrival, work, tr.delta, dt, n_ticks, gate), want)
        run.close()
        done += 1
    assert done > 120
