"""GPU parity of the placement that feeds the plan (rk_place_plans,
rk_schedule_round_placed) against the oracle's ork_place_plans on shared
inputs: the allocation and the per-segment maxima come from one side and go
to both, so parts, statuses and placed amounts must be identical; the plan
chosen on the split must be the oracle's, or one whose float64 throughput is
within 1e-5 of the oracle's maximum; throughputs within 1e-5."""
import dataclasses

import numpy as np
import pytest

import workloads
from test_gpu_random_workloads import draw_workload
from test_oracle_placed import HAND_ENV, HAND_JOB, PLAIN, make_job

pytestmark = pytest.mark.gpu
REL = 1e-5
GIB = float(2 ** 30)


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def place_on_gpu(run, best_thr, assign, floors, n_nodes, gpn, cpn, mpn, prev=None):
    """prev = (place_off, entries) of an earlier placement as numpy arrays, or None."""
    import torch
    import paper_2408_08586_amd as rk
    J = run.wl.n_jobs
    dev = run.device
    d_assign = torch.from_numpy(np.ascontiguousarray(assign).view(np.uint8).copy()).to(dev)
    d_floor = None if floors is None else torch.from_numpy(np.ascontiguousarray(floors, dtype=np.int32)).to(dev)
    p_off = p_ent = None
    if prev is not None:
        p_off = torch.from_numpy(np.ascontiguousarray(prev[0], dtype=np.uint32).view(np.int32).copy()).to(dev)
        ent = np.ascontiguousarray(prev[1], dtype=rk.PLACE_DTYPE)
        p_ent = torch.from_numpy((ent if ent.size else np.zeros(1, rk.PLACE_DTYPE)).view(np.uint8).copy()).to(dev)
    placed = rk.new_assign(J, dev)
    cap = n_nodes * gpn
    off = torch.full((J + 1,), -1, dtype=torch.int32, device=dev)
    status = torch.full((max(J, 1),), -1, dtype=torch.int32, device=dev)
    ent = rk.new_place_entries(cap, dev)
    total = run.f32(1)
    res = rk.rk_place_plans(run.ctx, run.jobs, run.table.c, run.grid, run.env, rk.rk_nodes(n_nodes, gpn, cpn, mpn),
                            run.dev_f32(best_thr), d_assign, d_floor, placed, off, ent, cap, status, total,
                            prev_off=p_off, prev_entries=p_ent)
    return (rk.assign_to_numpy(placed), rk.u32(off), rk.place_entries_to_numpy(ent, res.n_entries), rk.u32(status)[:J],
            float(total[0].item()), res)


def compare(orc, wl, tb, want, got):
    """want = oracle's (placed, off, entries, status, total); got = the library's, plus the result struct."""
    w_out, w_off, w_ent, w_st, w_total = want
    g_out, g_off, g_ent, g_st, g_total, res = got
    assert np.array_equal(g_st, w_st)
    assert np.array_equal(g_off, w_off)
    assert res.n_entries == len(w_ent)
    for f in ("node", "g", "c", "mem_gb"):
        assert np.array_equal(g_ent[f], w_ent[f]), f
    for f in ("g", "c", "mem_gb"):
        assert np.array_equal(g_out[f], w_out[f]), f
    assert res.n_placed == int(((w_st == 1) | (w_st == 2)).sum()) and res.n_failed == int((w_st == 3).sum())
    on = w_out["g"] > 0
    assert np.array_equal(g_out["plan"] == 0xFFFFFFFF, ~on) and np.all(g_out["thr"][~on] == 0)
    rel = np.abs(g_out["thr"][on].astype(np.float64) - w_out["thr"][on]) / w_out["thr"][on]
    assert rel.size == 0 or rel.max() <= REL
    n_band = 0
    for j in np.flatnonzero(on & (g_out["plan"] != w_out["plan"])).tolist():
        # another plan is fine only inside the band of the oracle's maximum, in the oracle's own float64 arithmetic
        d, t, p, v = (int(x) for x in tb.triples[tb.triple_off[j] + g_out["plan"][j] // 16])
        o = int(g_out["plan"][j]) % 16
        parts = w_ent["g"][w_off[j]:w_off[j + 1]].tolist()
        host = np.float32(w_out["mem_gb"][j]) * np.float32(GIB)
        reason, x = orc.eval_one_placed(wl.coef[j], wl.ints[j], wl.bounds, wl.env, d, t, p, o >> 2, (o >> 1) & 1, o & 1,
                                        int(w_out["c"][j]), float(host), parts, v=v)
        assert reason == 0 and d * t * p == w_out["g"][j]
        assert x["thr"] >= float(w_out["thr"][j]) * (1 - REL), f"job {j}: plan {g_out['plan'][j]} is outside the tie band"
        n_band += 1
    assert g_total == pytest.approx(w_total, rel=1e-5, abs=1e-12)
    return n_band


def test_hand_cases_on_the_device(gpu, orc):
    """The two-node cases worked by hand for the oracle: a 3 + 1 split flips the best plan, a job that does not fit
    takes a smaller count, floors, amounts per GPU."""
    coef, ints = make_job(**HAND_JOB)
    fill_c, fill_i = make_job(**dict(HAND_JOB, layers=1, gbatch=6))
    coef2, ints2 = np.stack([fill_c, coef]), np.stack([fill_i, ints])
    tb = orc.enumerate_plans(ints2, PLAIN)
    counts = tb.seg_g[tb.seg_off[1]:tb.seg_off[2]].tolist()
    cases = [(0, 4, None, 2, False, (2, 2, 1)), (1, 4, None, 2, False, (1, 1, 4)), (2, 4, None, 2, False, (1, 2, 2)),
             (3, 8, None, 2, False, (1, 1, 4)), (3, 8, 8, 2, False, None), (3, 8, 6, 2, False, None), (3, 8, 4, 2, False, (1, 1, 4)),
             (3, 8, None, 2, True, (1, 1, 4)), (3, 8, None, 3, False, None)]
    for filler_g, asked, floor, n_nodes, per_gpu, plan in cases:
        grid = workloads.Grid(np.array([2], np.uint32), 1, np.array([10.0], np.float32), 1) if per_gpu else \
            workloads.Grid(np.array([1], np.uint32), 0, np.array([64.0], np.float32), 0)
        wl = workloads.Workload("hand", coef2, ints2, PLAIN, grid, HAND_ENV, workloads.Cluster(8, 16, 1000.0))
        thr, _ = orc.eval_jobs(coef2, ints2, PLAIN, tb, grid, HAND_ENV)
        bt = orc.best_plan(tb, grid, thr)[0].astype(np.float32)
        a = np.zeros(2, orc.ASSIGN_DTYPE)
        a["g"] = [filler_g, asked]
        a["c"], a["mem_gb"] = ([2 * filler_g, 2 * asked], [10.0 * filler_g, 10.0 * asked]) if per_gpu else \
            ([1 if filler_g else 0, 1], [64.0 if filler_g else 0.0, 64.0])
        floors = None if floor is None else np.array([-1, counts.index(floor)], np.int32)
        mpn = 40.0 if per_gpu else 1000.0
        want = orc.place_plans(coef2, ints2, PLAIN, tb, grid, HAND_ENV, bt, a, n_nodes, 4, 8, mpn, min_seg=floors)
        run = gpu(wl)
        run.enumerate()
        got = place_on_gpu(run, bt, a, floors, n_nodes, 4, 8, mpn)
        assert compare(orc, wl, tb, want, got) == 0
        if plan is not None:
            assert tuple(int(x) for x in tb.triples[tb.triple_off[1] + got[0]["plan"][1] // 16][:3]) == plan
        run.close()


@pytest.mark.parametrize("cpn,mpn", [(64, 4096.0), (2, 4096.0), (64, 100.0)])
def test_generated_round_on_nodes(gpu, orc, cpn, mpn):
    wl = dataclasses.replace(workloads.paper_scale(), bounds=workloads.Bounds(g_max=6))
    r = orc.schedule_round(wl, n_threads=8)
    floors = np.full(wl.n_jobs, -1, np.int32)
    floors[::5] = 1
    want = orc.place_plans(wl.coef, wl.ints, wl.bounds, r["table"], wl.grid, wl.env, r["best_thr"], r["assign"], 8, 8, cpn, mpn,
                           min_seg=floors)
    run = gpu(wl)
    run.enumerate()
    got = place_on_gpu(run, r["best_thr"], r["assign"], floors, 8, 8, cpn, mpn)
    compare(orc, wl, r["table"], want, got)
    run.close()


def test_random_workloads_on_random_nodes(gpu, orc):
    """Seeded random small workloads (both grid modes, option masks, micro-batch shifts) on nodes that may be too few
    or short of CPUs and memory, with random floors."""
    base = workloads.paper_scale()
    done = n_multi = n_smaller = n_failed = n_band = n_changed = 0
    for seed in range(250):
        rng = np.random.default_rng(94000 + seed)
        wl = draw_workload(rng, base, mid=seed % 5 == 0)
        r = orc.schedule_round(wl, n_threads=8)
        ot = r["table"]
        if ot.triple_off[-1] == 0 or int(np.diff(ot.triple_off).max()) > 2048:
            continue
        a = r["assign"]
        gpn = int(rng.choice([1, 2, 4, 8]))
        n_nodes = int(max(1, -(-int(a["g"].sum()) // gpn) + rng.integers(-3, 2)))
        cpn = int(min(65535, rng.choice([gpn, 4 * gpn, 16 * gpn, 40 * gpn])))
        mpn = float(rng.choice([16.0, 64.0, 512.0, 1e5, 1e5]))
        floors = np.where(rng.uniform(size=wl.n_jobs) < 0.15, rng.integers(0, 4, wl.n_jobs), -1).astype(np.int32)
        env = dataclasses.replace(wl.env, gpus_per_node=gpn, B_inter=float(rng.choice([100e9, 25e9, 5e9])))
        wl = dataclasses.replace(wl, env=env)
        want = orc.place_plans(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, r["best_thr"], a, n_nodes, gpn, cpn, mpn,
                               min_seg=floors)
        run = gpu(wl)
        run.enumerate()
        got = place_on_gpu(run, r["best_thr"], a, floors, n_nodes, gpn, cpn, mpn)
        n_band += compare(orc, wl, ot, want, got)
        run.close()
        st, off = want[3], want[1]
        n_multi += int((np.diff(off) > 1).sum())
        n_smaller += int((st == 2).sum())
        n_failed += int((st == 3).sum())
        n_changed += int(((want[0]["plan"] != a["plan"]) & (st == 1)).sum())
        done += 1
    print(f"{done} rounds: {n_multi} jobs over several nodes, {n_smaller} placed with fewer GPUs, {n_failed} not placed, "
          f"{n_changed} plans changed by the split, {n_band} plans differ inside the band")
    assert done > 200 and n_multi > 100 and n_smaller >= 20 and n_failed > 20 and n_changed >= 20


def test_stress_round_on_its_nodes(gpu, orc):
    """The 10,000-job round on 512 nodes of 8 GPUs: the library's own allocation and maxima go to both sides; roomy
    nodes (all jobs at once) and nodes with 6 CPUs (job by job, smaller counts, failures)."""
    wl = workloads.stress()
    run = gpu(wl)
    assign, _ = run.schedule_round()
    run.enumerate()
    bt, _, _, _, _, n = run.fused()
    bt = run.host(bt, n).copy()
    ot = orc.enumerate_plans(wl.ints, wl.bounds, n_threads=16)
    for cpn in (128, 6):
        want = orc.place_plans(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, bt, assign, 512, 8, cpn, 2048.0)
        got = place_on_gpu(run, bt, assign, None, 512, 8, cpn, 2048.0)
        compare(orc, wl, ot, want, got)
        st = want[3]
        print(f"{cpn} CPUs per node: {int((st == 1).sum())} placed as asked, {int((st == 2).sum())} with fewer GPUs, "
              f"{int((st == 3).sum())} not placed; job-by-job stage: {bool(got[5].in_order)}")
        assert bool(got[5].in_order) == (cpn == 6)
    assert (st == 2).sum() + (st == 3).sum() > 0
    # a second round on roomy nodes: a tenth of the running jobs leave, the others stay where they are
    first = orc.place_plans(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, bt, assign, 512, 8, 128, 2048.0)
    rng = np.random.default_rng(7)
    a2 = first[0].copy()
    gone = np.flatnonzero(a2["g"] > 0)[rng.uniform(size=int((a2["g"] > 0).sum())) < 0.1]
    a2[gone] = (0, 0, 0.0, orc.NO_PLAN, 0.0)
    prev = (first[1], first[2])
    want = orc.place_plans(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, bt, a2, 512, 8, 128, 2048.0, prev=prev)
    got = place_on_gpu(run, bt, a2, None, 512, 8, 128, 2048.0, prev=prev)
    compare(orc, wl, ot, want, got)
    stay = np.flatnonzero(a2["g"] > 0)
    assert gone.size > 5 and all(np.array_equal(want[2][want[1][j]:want[1][j + 1]], first[2][first[1][j]:first[1][j + 1]])
                                 for j in stay)
    run.close()


@pytest.mark.parametrize("with_sla", [False, True])
def test_whole_round_on_nodes_is_its_pieces(gpu, orc, with_sla):
    """rk_schedule_round_placed = rk_schedule_round[_sla] on the nodes' totals, then rk_place_plans with the floors."""
    import torch
    import paper_2408_08586_amd as rk
    from test_gpu_sla import requests_from_draws
    wl = dataclasses.replace(workloads.paper_scale(), bounds=workloads.Bounds(g_max=12))
    n_nodes, gpn, cpn, mpn = 8, 8, 12, 512.0
    wl = dataclasses.replace(wl, cluster=workloads.Cluster(n_nodes * gpn, n_nodes * cpn, n_nodes * mpn))
    J = wl.n_jobs
    run = gpu(wl)
    run.enumerate()
    dev = run.device
    nodes = rk.rk_nodes(n_nodes, gpn, cpn, mpn)
    sla, floors = None, None
    bt, bp, ct, _, _, n = run.fused()
    if with_sla:
        r = orc.schedule_round(wl, n_threads=8)
        d = workloads.sla_draws(wl, quota_share=0.7, n_tenants=4)
        req_g, plan, base = requests_from_draws(wl, r, d)
        g_base = run.f32(J)
        rk.rk_eval_points(run.ctx, run.jobs, run.table.c, run.grid, run.env, run.dev_u32(np.arange(J)), run.dev_u32(plan),
                          run.dev_u32(d.req_c), run.dev_u32(d.req_m), g_base)
        sla = rk.Sla(d.guaranteed, d.tenant, d.quota_g, d.quota_c, req_g, d.req_c, d.req_m, g_base[:J])
        ms, mc, mm = run.i32(J), run.i32(J), run.i32(J)
        rk.rk_min_res(run.ctx, run.table.c, run.grid, 0, J, bt, sla, ms, mc, mm)
        floors = ms
    # the pieces
    a1, t1 = rk.new_assign(J, dev), run.f32(1)
    if with_sla:
        rk.rk_schedule_round_sla(run.ctx, run.jobs, run.bounds, run.grid, run.env, run.cluster, sla, a1, t1)
    else:
        rk.rk_schedule_round(run.ctx, run.jobs, run.bounds, run.grid, run.env, run.cluster, a1, t1)
    cap = n_nodes * gpn
    mk = lambda: (rk.new_assign(J, dev), torch.zeros(J + 1, dtype=torch.int32, device=dev), rk.new_place_entries(cap, dev),
                  torch.zeros(J, dtype=torch.int32, device=dev), run.f32(1))
    p1, o1, e1, s1, tt1 = mk()
    res1 = rk.rk_place_plans(run.ctx, run.jobs, run.table.c, run.grid, run.env, nodes, bt, a1, floors, p1, o1, e1, cap, s1, tt1)
    # the single call
    a2 = rk.new_assign(J, dev)
    p2, o2, e2, s2, tt2 = mk()
    res2 = rk.rk_schedule_round_placed(run.ctx, run.jobs, run.bounds, run.grid, run.env, nodes, sla, a2, p2, o2, e2, cap, s2, tt2)
    assert torch.equal(a1, a2) and torch.equal(p1, p2) and torch.equal(o1, o2) and torch.equal(s1, s2)
    assert tt1[0].item() == tt2[0].item() and res1.n_entries == res2.n_entries and res1.n_placed == res2.n_placed
    ne = res1.n_entries * rk.PLACE_DTYPE.itemsize
    assert torch.equal(e1[:ne], e2[:ne])
    # and the oracle on the same allocation
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    want = orc.place_plans(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, run.host(bt, n), rk.assign_to_numpy(a1),
                           n_nodes, gpn, cpn, mpn, min_seg=None if floors is None else run.host(floors, J))
    got = (rk.assign_to_numpy(p1), rk.u32(o1), rk.place_entries_to_numpy(e1, res1.n_entries), rk.u32(s1)[:J],
           float(tt1[0].item()), res1)
    compare(orc, wl, ot, want, got)
    assert res1.n_placed > 3
    run.close()


def test_argument_errors_and_amounts_off_the_grid(gpu, orc):
    """Error codes of rk_place_plans, and records that are not an allocation on this table and grid: such a job is
    not placed (status 3), books nothing, and the others are placed as if it had asked for nothing."""
    import torch
    import paper_2408_08586_amd as rk
    wl = dataclasses.replace(workloads.paper_scale(), bounds=workloads.Bounds(g_max=6))
    r = orc.schedule_round(wl, n_threads=8)
    J = wl.n_jobs
    run = gpu(wl)
    run.enumerate()
    dev = run.device
    a = r["assign"].copy()
    served = np.flatnonzero(a["g"] > 0)
    assert served.size >= 6
    bad = a.copy()
    j0, j1, j2 = (int(x) for x in served[:3])
    counts = r["table"].seg_g[r["table"].seg_off[j0]:r["table"].seg_off[j0 + 1]].tolist()
    bad["g"][j0] = next(g for g in range(2, 64) if g not in counts)          # not a GPU count of the job
    bad["c"][j1] += 1000                                                     # not a CPU level of the grid
    bad["mem_gb"][j2] = 3.0                                                  # not a memory tier of the grid
    gone = a.copy()
    for j in (j0, j1, j2):
        gone[j] = (0, 0, 0.0, orc.NO_PLAN, 0.0)
    want = orc.place_plans(wl.coef, wl.ints, wl.bounds, r["table"], wl.grid, wl.env, r["best_thr"], gone, 8, 8, 64, 4096.0)
    got = place_on_gpu(run, r["best_thr"], bad, None, 8, 8, 64, 4096.0)
    st = got[3].copy()
    assert st[j0] == 3 and st[j1] == 3 and st[j2] == 3 and got[5].n_failed == 3
    st[[j0, j1, j2]] = 0
    assert np.array_equal(st, want[3]) and np.array_equal(got[1], want[1])
    for f in ("node", "g", "c", "mem_gb"):
        assert np.array_equal(got[2][f], want[2][f])
    for f in ("g", "c", "mem_gb", "plan"):
        assert np.array_equal(got[0][f], want[0][f]), f

    d_assign = torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).copy()).to(dev)
    cap = 64
    mk = lambda: (rk.new_assign(J, dev), torch.zeros(J + 1, dtype=torch.int32, device=dev), rk.new_place_entries(cap, dev),
                  torch.zeros(J, dtype=torch.int32, device=dev), run.f32(1))
    bt = run.dev_f32(r["best_thr"])

    def call(nodes=None, placed="ok", cap_entries=cap, total="ok", best="ok", jobs=None):
        p, o, e, s, t = mk()
        return rk.rk_place_plans(run.ctx, jobs or run.jobs, run.table.c, run.grid, run.env, nodes or rk.rk_nodes(8, 8, 64, 4096.0),
                                 bt if best == "ok" else None, d_assign, None, p if placed == "ok" else None, o, e, cap_entries, s,
                                 t if total == "ok" else None)

    assert call().n_placed == served.size
    for kwargs, code in (({"placed": None}, rk.RK_ERR_INVALID_ARG), ({"total": None}, rk.RK_ERR_INVALID_ARG),
                         ({"best": None}, rk.RK_ERR_INVALID_ARG), ({"cap_entries": 63}, rk.RK_ERR_CAPACITY),
                         ({"nodes": rk.rk_nodes(5000, 8, 64, 4096.0)}, rk.RK_ERR_UNSUPPORTED),
                         ({"nodes": rk.rk_nodes(8, 0, 64, 4096.0)}, rk.RK_ERR_UNSUPPORTED)):
        with pytest.raises(rk.RkError) as e:
            call(**kwargs)
        assert e.value.code == code, kwargs
    other = rk.Jobs(wl.coef[:5], wl.ints[:5], dev)
    with pytest.raises(rk.RkError) as e:
        call(jobs=other)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    assert call().n_placed == served.size                                   # the context works on after the errors
    run.close()


def test_running_jobs_stay_on_their_nodes(gpu, orc):
    """The hand cases of the oracle's pins on the device: jobs that stay, a newcomer with a lower index, changed
    amounts, and an earlier placement that does not fit (the library then places everything anew)."""
    from test_oracle_placed import stay_jobs
    coef, ints, tb, grid, bt = stay_jobs(4)
    wl = workloads.Workload("stay", coef, ints, PLAIN, grid, HAND_ENV, workloads.Cluster(8, 16, 1000.0))
    run = gpu(wl)
    run.enumerate()

    def records(gs):
        a = np.zeros(4, orc.ASSIGN_DTYPE)
        a["g"], a["c"], a["mem_gb"] = gs, [1 if g else 0 for g in gs], [64.0 if g else 0.0 for g in gs]
        return a

    def both(gs, prev=None, cpn=8):
        a = records(gs)
        want = orc.place_plans(coef, ints, PLAIN, tb, grid, HAND_ENV, bt, a, 2, 4, cpn, 1000.0, prev=prev)
        got = place_on_gpu(run, bt, a, None, 2, 4, cpn, 1000.0, prev=prev)
        assert compare(orc, wl, tb, want, got) == 0
        return want, got

    w1, g1 = both([3, 4, 1, 0])
    prev = (g1[1], g1[2])                                            # the library's own earlier placement
    w2, g2 = both([0, 4, 1, 3], prev=prev)
    assert [(int(e["node"]), int(e["g"])) for e in g2[2]] == [(0, 1), (1, 3), (1, 1), (0, 3)] and bool(g2[5].in_order)
    both([0, 4, 1, 3])                                               # and without it job 1 moves to node 0
    both([0, 3, 1, 3], prev=prev)                                    # job 1 shrank: placed again
    both([4, 4, 0, 0], prev=(w2[1], w2[2]))                          # job 0 arrives ahead of the kept job 1
    both([8, 4, 0, 0], prev=(w2[1], w2[2]))                          # ... and falls back to what is left
    # an earlier placement that claims both 4-GPU jobs on node 0: the oracle refuses, the library ignores it
    w, g = both([4, 4, 0, 0])
    bad = g[2].copy()
    bad["node"][:] = 0
    with pytest.raises(AssertionError):
        orc.place_plans(coef, ints, PLAIN, tb, grid, HAND_ENV, bt, records([4, 4, 0, 0]), 2, 4, 8, 1000.0, prev=(g[1], bad))
    again = place_on_gpu(run, bt, records([4, 4, 0, 0]), None, 2, 4, 8, 1000.0, prev=(g[1], bad))
    assert compare(orc, wl, tb, w, again) == 0
    run.close()


def test_random_second_rounds_with_an_earlier_placement(gpu, orc):
    """Seeded random workloads on random nodes, two rounds each: the first placement, then some jobs leave, some change
    their amounts, some arrive (amounts of other valid points of their grid), and the second placement keeps what it can."""
    base = workloads.paper_scale()
    done = n_kept = n_moved = n_failed = 0
    for seed in range(200):
        rng = np.random.default_rng(99000 + seed)
        wl = draw_workload(rng, base, mid=seed % 4 == 0)
        r = orc.schedule_round(wl, n_threads=8)
        ot = r["table"]
        if ot.triple_off[-1] == 0 or int(np.diff(ot.triple_off).max()) > 2048:
            continue
        a1 = r["assign"]
        gpn = int(rng.choice([2, 4, 8]))
        n_nodes = int(max(1, -(-int(a1["g"].sum()) // gpn) + rng.integers(0, 3)))
        cpn = int(min(65535, rng.choice([4 * gpn, 16 * gpn, 40 * gpn])))
        mpn = float(rng.choice([64.0, 512.0, 1e5]))
        wl = dataclasses.replace(wl, env=dataclasses.replace(wl.env, gpus_per_node=gpn))
        args = (wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, r["best_thr"])
        w1 = orc.place_plans(*args, a1, n_nodes, gpn, cpn, mpn)
        run = gpu(wl)
        run.enumerate()
        g1 = place_on_gpu(run, r["best_thr"], a1, None, n_nodes, gpn, cpn, mpn)
        compare(orc, wl, ot, w1, g1)
        # second round: what the jobs hold, minus those that leave, with some amounts changed to other feasible points
        a2 = w1[0].copy()
        rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
        n_mem = len(wl.grid.mem_levels_gb)
        for j in range(wl.n_jobs):
            u = rng.uniform()
            if a2["g"][j] > 0 and u < 0.2:
                a2[j] = (0, 0, 0.0, orc.NO_PLAN, 0.0)
            elif u < 0.45:
                ns = int(ot.seg_off[j + 1] - ot.seg_off[j])
                bt_j = r["best_thr"][rows * int(ot.seg_off[j]):rows * int(ot.seg_off[j + 1])].reshape(rows, ns) if ns else None
                ok = np.argwhere(bt_j > 0) if ns else np.zeros((0, 2), int)
                if len(ok):
                    row, s = (int(x) for x in ok[rng.integers(0, len(ok))])
                    g = int(ot.seg_g[ot.seg_off[j] + s])
                    ci, mi = row // n_mem, row % n_mem
                    c = int(wl.grid.cpu_levels[ci]) * (g if wl.grid.cpu_mode else 1)
                    m = np.float32(wl.grid.mem_levels_gb[mi]) * (np.float32(g) if wl.grid.mem_mode else np.float32(1))
                    a2[j] = (g, c, float(m), 0, 0.0)
        prev = (g1[1], g1[2])
        w2 = orc.place_plans(*args, a2, n_nodes, gpn, cpn, mpn, prev=prev)
        g2 = place_on_gpu(run, r["best_thr"], a2, None, n_nodes, gpn, cpn, mpn, prev=prev)
        compare(orc, wl, ot, w2, g2)
        run.close()
        same = (a2["g"] > 0) & (a2["g"] == w1[0]["g"]) & (a2["c"] == w1[0]["c"]) & (a2["mem_gb"] == w1[0]["mem_gb"])
        for j in np.flatnonzero(same):
            assert np.array_equal(w2[2][w2[1][j]:w2[1][j + 1]], w1[2][w1[1][j]:w1[1][j + 1]])
        n_kept += int(same.sum())
        n_moved += int(((a2["g"] > 0) & ~same & (w2[3] > 0) & (w2[3] < 3)).sum())
        n_failed += int((w2[3] == 3).sum())
        done += 1
    print(f"{done} workloads: {n_kept} jobs stayed, {n_moved} placed again or new, {n_failed} not placed")
    assert done > 150 and n_kept > 100 and n_moved > 150 and n_failed > 100
