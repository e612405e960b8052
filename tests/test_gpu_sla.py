"""GPU parity of the service-level part (paper Sec. 5.2): point evaluation,
minimum demands, privileged phase and the greedy from the floors, each against
the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import workloads
from test_gpu_parity import REL, compare_rounds, oracle_table_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def requests_from_draws(wl, r, d):
    """Map the seeded draws onto the oracle's plan table: requested GPU count,
    original plan (a feasible plan of that GPU count at the requested CPUs and
    memory, if there is one) and the oracle's baseline throughput."""
    tb = r["table"]
    n_cpu, n_mem = len(wl.grid.cpu_levels), len(wl.grid.mem_levels_gb)
    rows = n_cpu * n_mem
    J = wl.n_jobs
    req_g, plan, base = np.zeros(J, np.uint32), np.zeros(J, np.uint32), np.zeros(J, np.float32)
    for j in range(J):
        s0, s1 = int(tb.seg_off[j]), int(tb.seg_off[j + 1])
        t0, nt = int(tb.triple_off[j]), int(tb.triple_off[j + 1] - tb.triple_off[j])
        ns = s1 - s0
        if ns == 0:
            continue
        s = min(int(d.u_seg[j] * ns), ns - 1)
        req_g[j] = tb.seg_g[s0 + s]
        first = int(tb.seg_first[s0 + s])
        last = int(tb.seg_first[s0 + s + 1]) if s + 1 < ns else nt
        row = int(d.req_c[j]) * n_mem + int(d.req_m[j])
        at = 16 * rows * t0 + row * nt * 16
        seg = r["thr"][at + first * 16: at + last * 16]
        ok = np.flatnonzero(seg > 0)
        plan[j] = first * 16
        if ok.size:
            k = ok[min(int(d.u_plan[j] * ok.size), ok.size - 1)]
            plan[j] = first * 16 + k
            base[j] = np.float32(seg[k])
    return req_g, plan, base


def near_jobs(wl, tb, best_thr, base, band=1e-5):
    """Jobs where some per-segment maximum lies within `band` of the baseline
    without being equal to it: float32 noise may decide their minimum demand."""
    rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
    out = np.zeros(wl.n_jobs, bool)
    for j in range(wl.n_jobs):
        blk = best_thr[rows * int(tb.seg_off[j]): rows * int(tb.seg_off[j + 1])]
        if base[j] > 0 and blk.size:
            rel = np.abs(blk.astype(np.float64) - base[j]) / base[j]
            out[j] = bool(np.any((rel < band) & (blk != base[j])))
    return out


@pytest.mark.parametrize("name", ["tiny", "paper_scale", "large"])
def test_eval_points_match_oracle_and_candidates(gpu, orc, name):
    import paper_2408_08586_amd as rk
    wl = workloads.CONFIGS[name]()
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    n_cpu, n_mem = len(wl.grid.cpu_levels), len(wl.grid.mem_levels_gb)
    rng = np.random.default_rng(5)
    je = min(wl.n_jobs, 40)                               # the oracle tensor of these jobs fits in memory
    o_thr, o_reason = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, 0, je, n_threads=16)
    g_thr, g_feas, n = run.eval(0, je)
    g_thr, g_feas = run.host(g_thr, n), run.host(g_feas, n)
    P = 20000
    pj = rng.integers(0, je, P).astype(np.uint32)
    nt = (ot.triple_off[pj + 1] - ot.triple_off[pj]).astype(np.int64)
    pp = (rng.uniform(size=P) * nt * 16).astype(np.uint32)
    pc = rng.integers(0, n_cpu, P).astype(np.uint32)
    pm = rng.integers(0, n_mem, P).astype(np.uint32)
    # a few points out of range: plan, level, tier, job
    bad = np.arange(0, 40)
    pp[bad[:10]] = (nt[bad[:10]] * 16).astype(np.uint32)
    pc[bad[10:20]] = n_cpu
    pm[bad[20:30]] = n_mem
    pj[bad[30:40]] = wl.n_jobs
    thr = run.f32(P)
    feas = run.torch.empty(P, dtype=run.torch.uint8, device=run.device)
    rk.rk_eval_points(run.ctx, run.jobs, run.table.c, run.grid, run.env, run.dev_u32(pj), run.dev_u32(pp),
                      run.dev_u32(pc), run.dev_u32(pm), thr, feas)
    rk.rk_sync(run.ctx)
    thr, feas = run.host(thr, P), run.host(feas, P)
    assert np.all(thr[bad] == 0) and np.all(feas[bad] == 1)
    good = np.setdiff1d(np.arange(P), bad)
    rows = n_cpu * n_mem
    idx = (16 * rows * ot.triple_off[pj[good]].astype(np.int64)
           + (pc[good].astype(np.int64) * n_mem + pm[good]) * nt[good] * 16 + pp[good])
    # the same bits as the candidate tensor of the library, the oracle's value within the tolerance
    assert np.array_equal(thr[good], g_thr[idx]) and np.array_equal(feas[good], g_feas[idx])
    assert np.array_equal(feas[good], o_reason[idx])
    want = o_thr[idx]
    assert np.array_equal(thr[good] == 0, want == 0)
    nz = want > 0
    assert np.max(np.abs(thr[good][nz] - want[nz]) / want[nz]) <= REL
    assert nz.sum() > P // 20 and (~nz).sum() > P // 20
    run.close()


def random_segment_values(orc, rng, ot, n_jobs, n_rows, grid):
    """Per-segment maxima drawn here (produced by neither implementation)."""
    n = ot.n_segments(n_rows)
    g_of = np.concatenate([np.tile(ot.seg_g[ot.seg_off[j]:ot.seg_off[j + 1]], n_rows) for j in range(n_jobs)])
    bt = (g_of ** rng.uniform(0.3, 1.0, n)) * rng.uniform(0.5, 1.5, n)
    bt = np.round(bt * 8) / 8
    bt[rng.uniform(size=n) < 0.15] = 0
    bt = bt.astype(np.float32)
    bp = rng.integers(0, 1000, n).astype(np.uint32)
    bp[bt == 0] = 0xFFFFFFFF
    ct, _, _ = orc.curves(ot, grid, bt, bp)
    return bt, bp, ct


def random_requests(rng, ot, J, n_cpu, n_mem, bt, n_rows, frac=0.4):
    guaranteed = (rng.uniform(size=J) < frac).astype(np.uint32)
    g_max = np.array([ot.seg_g[ot.seg_off[j + 1] - 1] if ot.seg_off[j + 1] > ot.seg_off[j] else 1 for j in range(J)])
    req_g = np.maximum((g_max * rng.uniform(size=J) ** 2).astype(np.uint32), rng.integers(0, 3, J).astype(np.uint32))
    req_c = rng.integers(0, n_cpu + 2, J).astype(np.uint32)          # some above the grid: clamped
    req_m = rng.integers(0, n_mem + 2, J).astype(np.uint32)
    # baselines: a multiple of some value of the job (coarse values: many exact equalities), or zero
    base = np.zeros(J, np.float32)
    for j in range(J):
        blk = bt[n_rows * int(ot.seg_off[j]): n_rows * int(ot.seg_off[j + 1])]
        if blk.size:
            base[j] = blk[rng.integers(0, blk.size)] * rng.choice([0.0, 0.5, 1.0, 1.0, 1.25])
    return guaranteed, req_g, req_c, req_m, base


@pytest.mark.parametrize("g_max,n_jobs", [(64, 3000), (1024, 400)])
def test_min_res_is_exact_on_shared_inputs(gpu, orc, g_max, n_jobs):
    import paper_2408_08586_amd as rk
    rng = np.random.default_rng(g_max)
    base_wl = workloads.stress(n_jobs=n_jobs)
    ints = base_wl.ints
    if g_max > 64:                                        # highly divisible batch sizes and depths: many valid GPU counts
        ints = np.stack([rng.choice([96, 60, 48, 120], n_jobs), rng.choice([5040, 2520, 1680, 720, 360], n_jobs),
                         np.ones(n_jobs, np.int64)], 1).astype(np.uint32)
    wl = workloads.Workload("minres", base_wl.coef, ints, workloads.Bounds(g_max=g_max), base_wl.grid,
                            base_wl.env, base_wl.cluster)
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    n_cpu, n_mem = 5, 4
    bt, bp, ct = random_segment_values(orc, rng, ot, n_jobs, n_cpu * n_mem, wl.grid)
    guaranteed, req_g, req_c, req_m, base = random_requests(rng, ot, n_jobs, n_cpu, n_mem, bt, n_cpu * n_mem)
    if g_max > 64:
        assert int(np.max(np.diff(ot.seg_off))) > 64                  # walks longer than a wavefront
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    sla = rk.Sla(guaranteed, np.zeros(n_jobs, np.uint32), [1], [1], req_g, req_c, req_m, base)
    for jb, je in ((0, n_jobs), (n_jobs // 3, n_jobs // 3 + 101)):
        rows = n_cpu * n_mem
        sub = bt[rows * int(ot.seg_off[jb]): rows * int(ot.seg_off[je])]
        ms, mc, mm = run.i32(je - jb), run.i32(je - jb), run.i32(je - jb)
        rk.rk_min_res(run.ctx, run.table.c, run.grid, jb, je, run.dev_f32(sub), sla, ms, mc, mm)
        rk.rk_sync(run.ctx)
        e_s, e_c, e_m = orc.min_res(ot, wl.grid, sub, guaranteed, req_g, req_c, req_m, base, jb, je)
        n = je - jb
        assert np.array_equal(run.host(ms, n), e_s)
        assert np.array_equal(rk.u32(mc)[:n], e_c) and np.array_equal(rk.u32(mm)[:n], e_m)
        assert (e_s >= 0).sum() > n // 5 and (e_s < 0).sum() > n // 5
    run.close()


@pytest.mark.parametrize("n_jobs,n_tenants", [(3000, 6), (12288, 200)])
def test_allocate_sla_is_exact_on_shared_inputs(gpu, orc, n_jobs, n_tenants):
    """Privileged phase and greedy from the floors on inputs drawn here: the
    records must be identical to the oracle's, under loose and tight quotas."""
    import paper_2408_08586_amd as rk
    rng = np.random.default_rng(n_jobs + 1)
    base_wl = workloads.stress(n_jobs=n_jobs)
    wl = workloads.Workload("alloc_sla", base_wl.coef, base_wl.ints, workloads.Bounds(g_max=64), base_wl.grid,
                            base_wl.env, workloads.Cluster(4096, 30000, 2.0e5))
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    n_cpu, n_mem, rows = 5, 4, 20
    bt, bp, ct = random_segment_values(orc, rng, ot, n_jobs, rows, wl.grid)
    guaranteed, req_g, req_c, req_m, base = random_requests(rng, ot, n_jobs, n_cpu, n_mem, bt, rows)
    req_g = np.minimum(req_g, 16)
    tenant = rng.integers(0, n_tenants + 1, n_jobs).astype(np.uint32)      # index n_tenants: unknown tenant
    min_seg, min_c, _ = orc.min_res(ot, wl.grid, bt, guaranteed, req_g, req_c, req_m, base)
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    d_bt, d_bp, d_ct = run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct)
    d_ms = run.torch.from_numpy(min_seg).to(run.device)
    d_mc = run.dev_u32(min_c)
    ref = wl.coef[:, 16]
    n_waiting = []
    for (G, Cc, M), share in (((4096, 30000, 2.0e5), 1.0), ((4096, 30000, 2.0e5), 0.2), ((4096, 4000, 1.0e9), 1.0),
                              ((500, 100000, 3000.0), 3.0), ((20000, 10 ** 6, 1.0e9), 10.0), ((0, 0, 0.0), 1.0)):
        cl = workloads.Cluster(G, Cc, M)
        w = rng.uniform(0.5, 1.5, n_tenants)
        w = w / w.sum() * share
        quota_g, quota_c = np.floor(w * G).astype(np.uint32), np.floor(w * Cc).astype(np.uint32)
        e_assign, e_total, _ = orc.policy(ref, ot, wl.grid, cl, bt, bp, ct, guaranteed, tenant, min_seg, min_c,
                                          quota_g, quota_c)
        sla = rk.Sla(guaranteed, tenant, quota_g, quota_c)
        assign = rk.new_assign(n_jobs, run.device)
        total = run.f32(1)
        rk.rk_allocate_sla(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, rk.make_cluster(cl), 0, n_jobs, d_bt, d_bp,
                           d_ct, sla, d_ms, d_mc, assign, total)
        rk.rk_sync(run.ctx)
        assign = rk.assign_to_numpy(assign)
        assert np.array_equal(assign, e_assign), (G, Cc, M, share)
        assert float(total[0].item()) == pytest.approx(e_total, rel=1e-6, abs=1e-12)
        assert assign["g"].sum() <= G and assign["c"].sum() <= Cc
        n_waiting.append(int(((guaranteed != 0) & (assign["g"] == 0)).sum()))
    print(f"guaranteed jobs left waiting per case: {n_waiting} of {int(guaranteed.sum())}")
    assert min(n_waiting[:5]) < max(n_waiting[:5])                         # quotas did bind in some cases only
    # no guaranteed job at all: the plain allocation
    zero = np.zeros(n_jobs, np.uint32)
    sla = rk.Sla(zero, zero, [0], [0])
    assign = rk.new_assign(n_jobs, run.device)
    total = run.f32(1)
    rk.rk_allocate_sla(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, 0, n_jobs, d_bt, d_bp, d_ct, sla,
                       d_ms, d_mc, assign, total)
    plain, plain_total = run.allocate(d_bt, d_bp, d_ct)
    assert np.array_equal(rk.assign_to_numpy(assign), plain) and float(total[0].item()) == plain_total
    run.close()


def test_service_levels_at_the_largest_grid_and_tenant_count(gpu, orc):
    """64 CPU levels x 16 memory tiers and 256 tenants (the most the library takes): minimum demands and the
    allocation from the floors on inputs drawn here, identical to the oracle's."""
    import paper_2408_08586_amd as rk
    rng = np.random.default_rng(64016)
    n_jobs, n_cpu, n_mem, n_tenants = 600, 64, 16, 256
    rows = n_cpu * n_mem
    base_wl = workloads.stress(n_jobs=n_jobs)
    grid = workloads.Grid(np.arange(1, 65, dtype=np.uint32), 1, (np.arange(16) * 12.5).astype(np.float32), 0)
    wl = workloads.Workload("sla_maxgrid", base_wl.coef, base_wl.ints, workloads.Bounds(g_max=16), grid, base_wl.env,
                            workloads.Cluster(600, 6000, 1.0e5))
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    bt, bp, ct = random_segment_values(orc, rng, ot, n_jobs, rows, wl.grid)
    guaranteed, req_g, req_c, req_m, base = random_requests(rng, ot, n_jobs, n_cpu, n_mem, bt, rows)
    tenant = rng.integers(0, n_tenants + 1, n_jobs).astype(np.uint32)
    run = gpu(wl)
    assert run.n_rows == rows
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    d_bt, d_bp, d_ct = run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct)
    sla = rk.Sla(guaranteed, tenant, [1] * n_tenants, [1] * n_tenants, req_g, req_c, req_m, base)
    ms, mc, mm = run.i32(n_jobs), run.i32(n_jobs), run.i32(n_jobs)
    rk.rk_min_res(run.ctx, run.table.c, run.grid, 0, n_jobs, d_bt, sla, ms, mc, mm)
    rk.rk_sync(run.ctx)
    min_seg, min_c, min_m = orc.min_res(ot, wl.grid, bt, guaranteed, req_g, req_c, req_m, base)
    assert np.array_equal(run.host(ms, n_jobs), min_seg)
    assert np.array_equal(rk.u32(mc)[:n_jobs], min_c) and np.array_equal(rk.u32(mm)[:n_jobs], min_m)
    assert len(set(min_c[min_seg >= 0].tolist())) > 8 and len(set(min_m[min_seg >= 0].tolist())) > 4
    ref = wl.coef[:, 16]
    levels = set()
    for (G, Cc, M), share in (((600, 6000, 1.0e5), 1.0), ((600, 6000, 1.0e5), 0.3), ((300, 100000, 2000.0), 2.0)):
        cl = workloads.Cluster(G, Cc, M)
        w = rng.uniform(0.5, 1.5, n_tenants)
        w = w / w.sum() * share
        quota_g, quota_c = np.ceil(w * G).astype(np.uint32), np.ceil(w * Cc).astype(np.uint32)
        e_assign, e_total, _ = orc.policy(ref, ot, wl.grid, cl, bt, bp, ct, guaranteed, tenant, min_seg, min_c,
                                          quota_g, quota_c)
        assign = rk.new_assign(n_jobs, run.device)
        total = run.f32(1)
        rk.rk_allocate_sla(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, rk.make_cluster(cl), 0, n_jobs, d_bt, d_bp,
                           d_ct, rk.Sla(guaranteed, tenant, quota_g, quota_c), run.torch.from_numpy(min_seg).to(run.device),
                           run.dev_u32(min_c), assign, total)
        rk.rk_sync(run.ctx)
        assign = rk.assign_to_numpy(assign)
        assert np.array_equal(assign, e_assign), (G, Cc, M, share)
        assert float(total[0].item()) == pytest.approx(e_total, rel=1e-6, abs=1e-12)
        got = e_assign[e_assign["g"] > 0]
        levels |= set((got["c"] // got["g"]).tolist())
        assert ((guaranteed != 0) & (e_assign["g"] > 0)).sum() > 0
    assert len(levels) > 8
    run.close()


def test_allocate_sla_on_a_job_range(gpu, orc):
    import paper_2408_08586_amd as rk
    wl = workloads.paper_scale()
    jb, je = 7, 41
    sub = wl.subset(np.arange(jb, je))
    sub.cluster = workloads.Cluster(40, 80, 900.0)
    r = orc.schedule_round(sub, n_threads=8)
    d = workloads.sla_draws(sub, frac_guaranteed=0.5, n_tenants=3, quota_share=0.6)
    req_g, _, base = requests_from_draws(sub, r, d)
    ms, mc, _ = orc.min_res(r["table"], sub.grid, r["best_thr"], d.guaranteed, req_g, d.req_c, d.req_m, base)
    e_assign, e_total, _ = orc.policy(sub.coef[:, 16], r["table"], sub.grid, sub.cluster, r["best_thr"], r["best_plan"],
                                      r["curve_thr"], d.guaranteed, d.tenant, ms, mc, d.quota_g, d.quota_c)
    run = gpu(wl)
    run.enumerate()
    pad = lambda a: np.concatenate([np.zeros(jb, a.dtype), a, np.zeros(wl.n_jobs - je, a.dtype)])   # per-job arrays are indexed by job
    sla = rk.Sla(pad(d.guaranteed), pad(d.tenant), d.quota_g, d.quota_c)
    assign = rk.new_assign(je - jb, run.device)
    total = run.f32(1)
    rk.rk_allocate_sla(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, rk.make_cluster(sub.cluster), jb, je,
                       run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]), run.dev_f32(r["curve_thr"]), sla,
                       run.torch.from_numpy(ms).to(run.device), run.dev_u32(mc), assign, total)
    rk.rk_sync(run.ctx)
    assert np.array_equal(rk.assign_to_numpy(assign), e_assign)
    assert float(total[0].item()) == pytest.approx(e_total, rel=1e-6)
    assert ((d.guaranteed != 0) & (e_assign["g"] > 0)).sum() > 0
    run.close()


@pytest.mark.parametrize("name,share", [("tiny", 1.0), ("paper_scale", 0.7), ("large", 0.5)])
def test_schedule_round_sla_end_to_end(gpu, orc, name, share):
    """Everything on the device, baseline included (rk_eval_points on the
    original plans), against the oracle's pipeline."""
    import paper_2408_08586_amd as rk
    wl = workloads.CONFIGS[name]()
    r = orc.schedule_round(wl, n_threads=16)
    tb = r["table"]
    d = workloads.sla_draws(wl, quota_share=share, **(dict(n_tenants=2, frac_guaranteed=0.6) if name == "tiny"
                                                      else dict(n_tenants=4)))
    req_g, plan, base = requests_from_draws(wl, r, d)
    e_ms, e_mc, e_mm = orc.min_res(tb, wl.grid, r["best_thr"], d.guaranteed, req_g, d.req_c, d.req_m, base)
    e_assign, e_total, e_gap = orc.policy(wl.coef[:, 16], tb, wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                          r["curve_thr"], d.guaranteed, d.tenant, e_ms, e_mc, d.quota_g, d.quota_c)
    J = wl.n_jobs
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), tb)
    # baseline on the device
    g_base = run.f32(J)
    rk.rk_eval_points(run.ctx, run.jobs, run.table.c, run.grid, run.env, run.dev_u32(np.arange(J)), run.dev_u32(plan),
                      run.dev_u32(d.req_c), run.dev_u32(d.req_m), g_base)
    rk.rk_sync(run.ctx)
    hb = run.host(g_base, J)
    assert np.array_equal(hb == 0, base == 0)
    nz = base > 0
    assert nz.sum() > 0 and np.max(np.abs(hb[nz].astype(np.float64) - base[nz]) / base[nz]) <= REL
    sla = rk.Sla(d.guaranteed, d.tenant, d.quota_g, d.quota_c, req_g, d.req_c, d.req_m, g_base[:J])
    # piecewise on the device: curves, minimum demands, allocation
    bt, bp, ct, cp, cg, n = run.fused()
    ms, mc, mm = run.i32(J), run.i32(J), run.i32(J)
    rk.rk_min_res(run.ctx, run.table.c, run.grid, 0, J, bt, sla, ms, mc, mm)
    rk.rk_sync(run.ctx)
    h_ms, h_mc, h_mm = run.host(ms, J), rk.u32(mc)[:J], rk.u32(mm)[:J]
    near = near_jobs(wl, tb, r["best_thr"], base)
    clear = ~near
    assert np.array_equal(h_ms[clear], e_ms[clear]) and np.array_equal(h_mc[clear], e_mc[clear])
    assert np.array_equal(h_mm[clear], e_mm[clear])
    floors_equal = np.array_equal(h_ms, e_ms) and np.array_equal(h_mc, e_mc)
    assign = rk.new_assign(J, run.device)
    total = run.f32(1)
    rk.rk_allocate_sla(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, 0, J, bt, bp, ct, sla, ms, mc,
                       assign, total)
    rk.rk_sync(run.ctx)
    a_piece, t_piece = rk.assign_to_numpy(assign), float(total[0].item())
    if floors_equal:
        own = (run.host(bt, n).copy(), run.host(bp, n).view(np.uint32).copy(), run.host(ct, n).copy())
        same = compare_rounds(orc, wl, a_piece, t_piece, dict(assign=e_assign, total=e_total, min_gap=e_gap, table=tb), own,
                              redo=lambda b_thr, b_plan, c_thr: orc.policy(wl.coef[:, 16], tb, wl.grid, wl.cluster, b_thr, b_plan,
                                                                           c_thr, d.guaranteed, d.tenant, h_ms, h_mc, d.quota_g,
                                                                           d.quota_c)[:2])
    else:
        same = False
        assert t_piece == pytest.approx(e_total, rel=1e-2)
    assert a_piece["g"].sum() <= wl.cluster.G and a_piece["c"].sum() <= wl.cluster.C
    # the single call gives the same bits as the pieces
    assign2 = rk.new_assign(J, run.device)
    total2 = run.f32(1)
    rk.rk_schedule_round_sla(run.ctx, run.jobs, run.bounds, run.grid, run.env, run.cluster, sla, assign2, total2)
    rk.rk_sync(run.ctx)
    assert np.array_equal(rk.assign_to_numpy(assign2), a_piece) and float(total2[0].item()) == t_piece
    granted = int(((d.guaranteed != 0) & (a_piece["g"] > 0)).sum())
    print(f"{name}: {int(d.guaranteed.sum())} guaranteed jobs, {granted} served, {int(near.sum())} with a baseline inside "
          f"the float32 band; floors equal: {floors_equal}; assignments equal: {same}; min slope gap {e_gap:.2e}")
    assert granted > 0
    run.close()


def test_sla_argument_errors(gpu, orc):
    import paper_2408_08586_amd as rk
    wl = workloads.tiny()
    run = gpu(wl)
    run.enumerate()
    J = wl.n_jobs
    z = np.zeros(J, np.uint32)
    bt, bp, ct, cp, cg, n = run.fused()
    assign, total = rk.new_assign(J, run.device), run.f32(1)
    ms, mc = run.i32(J), run.i32(J)
    too_many = rk.Sla(z, z, np.ones(rk.RK_MAX_TENANTS + 1, np.uint32), np.ones(rk.RK_MAX_TENANTS + 1, np.uint32))
    with pytest.raises(rk.RkError) as e:
        rk.rk_allocate_sla(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, 0, J, bt, bp, ct, too_many, ms,
                           mc, assign, total)
    assert e.value.code == rk.RK_ERR_UNSUPPORTED
    no_request = rk.Sla(z, z, [1], [1])
    with pytest.raises(rk.RkError) as e:
        rk.rk_schedule_round_sla(run.ctx, run.jobs, run.bounds, run.grid, run.env, run.cluster, no_request, assign, total)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    with pytest.raises(rk.RkError) as e:
        rk.rk_min_res(run.ctx, run.table.c, run.grid, 0, J, bt, no_request, ms, mc, mc)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    # an empty range is fine
    rk.rk_min_res(run.ctx, run.table.c, run.grid, 3, 3, bt, no_request, ms, mc, mc)
    rk.rk_eval_points(run.ctx, run.jobs, run.table.c, run.grid, run.env, None, None, None, None, run.f32(0)[:0])
    run.close()


def test_privileged_jobs_for_the_loop(gpu, orc):
    """rk_privileged against the oracle on drawn service levels and states: floors and states bit for bit; then the loop
    from them on both sides (service levels -> minimum demands -> who is privileged -> Algorithm 1's loop)."""
    import torch
    import paper_2408_08586_amd as rk
    from test_gpu_reschedule import random_round, on_gpu as loop_on_gpu, same as same_round
    n_wait = n_floor = 0
    for seed in range(120):
        rng = np.random.default_rng(61000 + seed)
        big = seed % 10 == 9
        wl, tb, bt, bp, ct, cur_seg, cur_c, _, _, state = random_round(rng, orc, 3000 if big else None, 12 if big else None)
        J = wl.n_jobs
        T = int(rng.choice([1, 3, 17, 256]))
        guaranteed = (rng.uniform(size=J) < 0.5).astype(np.uint32)
        tenant = rng.integers(0, T + 2, J).astype(np.uint32)                 # a few unknown tenants
        ns = np.diff(tb.seg_off)
        min_seg = np.where(rng.uniform(size=J) < 0.85, rng.integers(0, np.maximum(ns, 1)), -1).astype(np.int32)
        min_seg[rng.uniform(size=J) < 0.03] = 10 ** 6                        # not an index of the job's list
        min_c = rng.integers(0, len(wl.grid.cpu_levels) + 1, J).astype(np.uint32)        # one level beyond the grid: clamped
        scale = max(1, J // max(T, 1))
        quota_g = rng.integers(0, 4 * scale + 2, T).astype(np.uint32)
        quota_c = rng.integers(0, 16 * scale + 2, T).astype(np.uint32)
        use_state = seed % 3 != 0
        st_in = state if use_state else None
        want = orc.privileged(tb, wl.grid, guaranteed, tenant, min_seg, min_c, quota_g, quota_c, cur_seg, cur_c, state=st_in)
        run = gpu(wl)
        run.enumerate()
        dev = run.device
        sla = rk.Sla(guaranteed, tenant, quota_g, quota_c, device=dev)
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
        fs, fc = torch.full((J,), -7, dtype=torch.int32, device=dev), torch.full((J,), -7, dtype=torch.int32, device=dev)
        so = torch.full((J,), 77, dtype=torch.uint8, device=dev)
        rk.rk_privileged(run.ctx, run.table.c, run.grid, sla, i32(min_seg), run.dev_u32(min_c), i32(cur_seg), run.dev_u32(cur_c),
                         fs, fc, so, state=None if st_in is None else torch.from_numpy(st_in).to(dev))
        rk.rk_sync(run.ctx)
        g_fs, g_fc, g_so = fs.cpu().numpy(), fc.cpu().numpy().view(np.uint32), so.cpu().numpy()
        assert np.array_equal(g_fs, want[0]) and np.array_equal(g_fc, want[1]) and np.array_equal(g_so, want[2]), seed
        n_wait += int(((want[2] == 1) & ((st_in if st_in is not None else 0) == 0)).sum())
        n_floor += int((want[0] >= 0).sum())
        if seed % 4 == 0:                                                    # ... and the loop from these floors and states
            w_round = orc.reschedule(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct, cur_seg, cur_c, want[0], want[1],
                                     state=want[2])
            same_round(loop_on_gpu(run, bt, bp, ct, wl.cluster, cur_seg, cur_c, g_fs, g_fc, g_so), w_round)
        run.close()
    print(f"120 cases: {n_floor} floors granted, {n_wait} jobs wait")
    assert n_floor > 500 and n_wait > 500
