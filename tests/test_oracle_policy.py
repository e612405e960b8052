"""Pins for the oracle's service-level part (paper Sec. 5.2, "Scheduling
algorithm design"): the minimum demand of guaranteed jobs and the greedy that
starts from these floors under tenant quotas."""
import itertools

import numpy as np
import pytest

import workloads


def one_job_table(orc, g_max=8):
    ints = np.array([[8, 8, 1]], np.uint32)            # valid GPU counts 1, 2, 4, 8
    return orc.enumerate_plans(ints, workloads.Bounds(g_max=g_max))


GRID = workloads.Grid(np.array([1, 2, 4], np.uint32), 0, np.array([10.0, 100.0], np.float32), 0)


def test_min_res_hand_cases(orc):
    tb = one_job_table(orc)
    assert tb.seg_g.tolist() == [1, 2, 4, 8]
    # layout [cpu][mem][segment]
    bt = np.zeros((3, 2, 4), np.float32)
    bt[0, 0] = [1.0, 2.0, 3.0, 3.5]
    bt[0, 1] = [1.0, 2.0, 3.0, 3.5]
    bt[1, 0] = [1.2, 2.6, 3.2, 3.6]
    bt[1, 1] = [1.2, 2.6, 3.2, 3.6]
    bt[2, 0] = [1.3, 3.1, 3.3, 3.7]
    bt[2, 1] = [1.3, 3.1, 3.3, 4.0]
    flat = bt.reshape(-1)
    run = lambda g, c, m, base, gu=1: tuple(int(x[0]) for x in orc.min_res(tb, GRID, flat, [gu], [g], [c], [m], [base]))
    # the request (4 GPUs, level 0) runs at 3.0: 2 GPUs with 4 CPUs do better -> but CPUs may not exceed the request
    assert run(4, 0, 1, 3.0) == (2, 0, 0)
    # with more CPUs in the request, fewer GPUs reach the baseline: fewest GPUs first, then fewest CPUs, then memory
    assert run(4, 2, 1, 3.0) == (1, 2, 0)
    assert run(4, 1, 1, 2.5) == (1, 1, 0)
    # equality counts as reaching the baseline
    assert run(8, 2, 1, 4.0) == (3, 2, 1)
    # nothing reaches the baseline: the request itself
    assert run(4, 1, 0, 9.0) == (2, 1, 0)
    # a request between valid GPU counts is rounded down to a valid one
    assert run(7, 0, 0, 9.0) == (2, 0, 0)
    # a baseline of zero (original plan infeasible): the smallest feasible allocation
    assert run(8, 2, 1, 0.0) == (0, 0, 0)
    # best-effort jobs and requests below the smallest valid count have no minimum
    assert run(4, 2, 1, 1.0, gu=0) == (-1, 0, 0)
    assert run(0, 2, 1, 1.0) == (-1, 0, 0)
    # infeasible points never qualify
    bt2 = bt.copy(); bt2[:, :, 0] = 0
    assert tuple(int(x[0]) for x in orc.min_res(tb, GRID, bt2.reshape(-1), [1], [8], [2], [1], [0.0])) == (1, 0, 0)


def test_min_res_matches_brute_force(orc):
    wl = workloads.large()
    sub = wl.subset(np.arange(60))
    r = orc.schedule_round(sub, n_threads=4)
    tb = r["table"]
    rng = np.random.default_rng(2)
    J = sub.n_jobs
    n_cpu, n_mem = len(sub.grid.cpu_levels), len(sub.grid.mem_levels_gb)
    guaranteed = (rng.uniform(size=J) < 0.7).astype(np.uint32)
    req_g = rng.choice([1, 2, 3, 8, 16, 64, 100, 1024], J).astype(np.uint32)
    req_c = rng.integers(0, n_cpu, J).astype(np.uint32)
    req_m = rng.integers(0, n_mem, J).astype(np.uint32)
    # baseline: throughput of some plan at the requested resources, sometimes unreachable, sometimes zero
    base = np.zeros(J, np.float32)
    rows = n_cpu * n_mem
    for j in range(J):
        ns = int(tb.seg_off[j + 1] - tb.seg_off[j])
        blk = r["best_thr"][rows * int(tb.seg_off[j]):rows * int(tb.seg_off[j + 1])].reshape(n_cpu, n_mem, ns)
        base[j] = blk.max() * rng.choice([0.0, 0.3, 0.6, 0.9, 1.0, 1.5])
    seg, c, m = orc.min_res(tb, sub.grid, r["best_thr"], guaranteed, req_g, req_c, req_m, base)
    for j in range(J):
        ns = int(tb.seg_off[j + 1] - tb.seg_off[j])
        g_list = tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]]
        blk = r["best_thr"][rows * int(tb.seg_off[j]):rows * int(tb.seg_off[j + 1])].reshape(n_cpu, n_mem, ns)
        ok_s = [s for s in range(ns) if g_list[s] <= req_g[j]]
        if not guaranteed[j] or not ok_s:
            assert (seg[j], c[j], m[j]) == (-1, 0, 0)
            continue
        cands = [(s, cc, mm) for s, cc, mm in itertools.product(ok_s, range(req_c[j] + 1), range(req_m[j] + 1))
                 if blk[cc, mm, s] > 0 and blk[cc, mm, s] >= base[j]]
        want = min(cands) if cands else (max(ok_s), int(req_c[j]), int(req_m[j]))
        assert (int(seg[j]), int(c[j]), int(m[j])) == want


def floors_case(orc, curves, guaranteed, tenant, min_seg, min_c, quota_g, quota_c, G, C=10 ** 6, host=1e9, ref=None,
                grid=None):
    """curves[j][s]: best throughput of job j at g = 1, 2, 4, 8 (same at every CPU level unless a 3-d array is given)."""
    J = len(curves)
    ints = np.tile(np.array([[8, 8, 1]], np.uint32), (J, 1))
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=8))
    grid = grid or workloads.Grid(np.array([1, 2], np.uint32), 0, np.array([1.0], np.float32), 0)
    n_cpu = len(grid.cpu_levels)
    bt = np.zeros((J, n_cpu, 1, 4), np.float32)
    for j, cv in enumerate(curves):
        cv = np.asarray(cv, np.float32)
        bt[j, :, 0, :] = cv if cv.ndim == 2 else cv[None, :]
    bt = bt.reshape(-1)
    bp = np.arange(bt.size, dtype=np.uint32)
    bp[bt == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, bt, bp)
    ref = np.ones(J, np.float32) if ref is None else np.asarray(ref, np.float32)
    return orc.policy(ref, tb, grid, workloads.Cluster(G, C, host), bt, bp, ct, guaranteed, tenant, min_seg, min_c,
                      quota_g, quota_c)


def test_policy_floor_is_granted_before_slopes(orc):
    steep = [4.0, 8.0, 12.0, 17.0]
    flat = [1.0, 1.1, 1.2, 1.3]
    # 8 GPUs: without floors the steep job takes everything
    a, _, _ = floors_case(orc, [flat, steep], [0, 0], [0, 0], [-1, -1], [0, 0], [100], [100], G=8)
    assert a["g"].tolist() == [0, 8]
    # the flat job is guaranteed 4 GPUs: it gets them first, the steep job the rest
    a, total, _ = floors_case(orc, [flat, steep], [1, 0], [0, 0], [2, -1], [0, 0], [100], [100], G=8)
    assert a["g"].tolist() == [4, 4]
    assert total == pytest.approx(1.2 + 12.0)
    # the floor's CPU level is kept and charged
    a, _, _ = floors_case(orc, [flat, steep], [1, 0], [0, 0], [2, -1], [1, 0], [100], [100], G=8, C=3)
    assert a["g"].tolist() == [4, 4] and a["c"].tolist() == [2, 1]


def test_policy_quota_and_capacity(orc):
    c = [1.0, 2.0, 3.0, 4.0]
    # tenant 0 has quota for one 4-GPU floor only: the second guaranteed job waits (gets nothing at all)
    a, _, _ = floors_case(orc, [c, c, c], [1, 1, 0], [0, 0, 1], [2, 2, -1], [0, 0, 0], [6, 100], [100, 100], G=16)
    assert a["g"][1] == 0 and a["g"][0] >= 4 and a["g"][2] > 0
    assert a["g"].sum() <= 16
    # separate tenants: both floors granted
    a, _, _ = floors_case(orc, [c, c, c], [1, 1, 0], [0, 1, 1], [2, 2, -1], [0, 0, 0], [6, 6], [100, 100], G=16)
    assert a["g"][0] >= 4 and a["g"][1] >= 4
    # CPU quota blocks as well (floor needs level 1 = 2 CPUs)
    a, _, _ = floors_case(orc, [c, c], [1, 1], [0, 0], [1, 1], [1, 1], [100], [3], G=16)
    assert a["g"][0] >= 2 and a["g"][1] == 0
    # free capacity smaller than the floor: waits
    a, _, _ = floors_case(orc, [c, c], [1, 0], [0, 0], [3, -1], [0, 0], [100], [100], G=4)
    assert a["g"].tolist() == [0, 4]
    # a guaranteed job without a minimum, or with an unknown tenant, waits
    a, _, _ = floors_case(orc, [c, c], [1, 1], [0, 7], [-1, 1], [0, 0], [100], [100], G=8)
    assert a["g"].tolist() == [0, 0]


def test_policy_without_guaranteed_jobs_is_the_plain_greedy(orc):
    wl = workloads.paper_scale()
    r = orc.schedule_round(wl, n_threads=4)
    J = wl.n_jobs
    z = np.zeros(J, np.uint32)
    a, total, _ = orc.policy(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                             r["curve_thr"], z, z, np.full(J, -1, np.int32), z, [0], [0])
    assert np.array_equal(a, r["assign"]) and total == r["total"]


def test_policy_invariants_on_generated_workload(orc):
    wl = workloads.large().subset(np.arange(300))
    wl.cluster = workloads.Cluster(512, 3000, 64 * 2048.0)
    r = orc.schedule_round(wl, n_threads=4)
    tb = r["table"]
    J = wl.n_jobs
    rng = np.random.default_rng(9)
    guaranteed = (rng.uniform(size=J) < 0.3).astype(np.uint32)
    tenant = rng.integers(0, 4, J).astype(np.uint32)
    req_g = rng.choice([1, 2, 4, 8, 16, 32], J).astype(np.uint32)
    req_c = rng.integers(0, 5, J).astype(np.uint32)
    base = np.zeros(J, np.float32)
    rows = 5
    for j in range(J):
        ns = int(tb.seg_off[j + 1] - tb.seg_off[j])
        blk = r["best_thr"][rows * int(tb.seg_off[j]):rows * int(tb.seg_off[j + 1])].reshape(5, 1, ns)
        base[j] = 0.8 * blk[req_c[j], 0, :max(1, np.searchsorted(tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]], req_g[j], side="right"))].max()
    seg, mc, mm = orc.min_res(tb, wl.grid, r["best_thr"], guaranteed, req_g, req_c, np.zeros(J, np.uint32), base)
    quota_g, quota_c = np.array([60, 40, 200, 10], np.uint32), np.array([500, 100, 3000, 40], np.uint32)
    a, total, _ = orc.policy(wl.coef[:, 16], tb, wl.grid, wl.cluster, r["best_thr"], r["best_plan"], r["curve_thr"],
                             guaranteed, tenant, seg, mc, quota_g, quota_c)
    assert a["g"].sum() <= wl.cluster.G and a["c"].sum() <= wl.cluster.C
    granted_floor = 0
    for j in np.flatnonzero(guaranteed):
        if a["g"][j] == 0:
            continue
        g_floor = tb.seg_g[tb.seg_off[j] + seg[j]]
        assert seg[j] >= 0 and a["g"][j] >= g_floor             # never below its floor
        # and it reaches the guaranteed performance unless memory cut it
        granted_floor += 1
    assert granted_floor > 0
    # floors granted per tenant stay within the quota
    for t in range(4):
        js = [j for j in np.flatnonzero(guaranteed) if tenant[j] == t and a["g"][j] > 0]
        assert sum(int(tb.seg_g[tb.seg_off[j] + seg[j]]) for j in js) <= quota_g[t]


def privileged_case(orc, guaranteed, tenant, min_g, min_c, quota_g, quota_c, hold, state=None, levels=(1, 2), mode=0):
    """min_g[j], hold[j]: GPUs (0 = none) out of the counts 1, 2, 4, 8."""
    J = len(guaranteed)
    tb = orc.enumerate_plans(np.tile(np.array([[8, 8, 1]], np.uint32), (J, 1)), workloads.Bounds(g_max=8))
    grid = workloads.Grid(np.array(levels, np.uint32), mode, np.array([1.0], np.float32), 0)
    seg = lambda g: [1, 2, 4, 8].index(g) if g else -1
    return orc.privileged(tb, grid, guaranteed, tenant, [seg(g) for g in min_g], min_c, quota_g, quota_c,
                          [seg(g) for g in hold], np.zeros(J, np.uint32), state=state)


def test_privileged_jobs_for_the_loop(orc):
    # three queued guaranteed jobs of one tenant with 4-GPU minima and a quota of 10 GPUs: the first two get their floor
    # (the loop will serve them first), the third waits
    fs, fc, st = privileged_case(orc, [1, 1, 1], [0, 0, 0], [4, 4, 4], [0, 0, 0], [10], [100], [0, 0, 0])
    assert fs.tolist() == [2, 2, -1] and st.tolist() == [0, 0, 1]
    # a running guaranteed job is charged first, whatever its index: job 2 runs, so only one queued job fits beside it
    fs, fc, st = privileged_case(orc, [1, 1, 1], [0, 0, 0], [4, 4, 4], [0, 0, 0], [10], [100], [0, 0, 8])
    assert fs.tolist() == [2, -1, 2] and st.tolist() == [0, 1, 0]
    # ... and keeps taking part even when the quota would not admit it today (its floor stays, nothing is left)
    fs, fc, st = privileged_case(orc, [1, 1], [0, 0], [4, 4], [0, 0], [3], [100], [8, 0])
    assert fs.tolist() == [2, -1] and st.tolist() == [0, 1]
    # a running job's CPUs are charged too: its minimum at level 1 takes 2 of the tenant's 3 CPUs, the queued job needs 2
    fs, fc, st = privileged_case(orc, [1, 1], [0, 0], [2, 2], [1, 1], [100], [3], [4, 0])
    assert fs.tolist() == [1, -1] and st.tolist() == [0, 1]
    # tenants have separate quotas; the CPU quota binds as well (level 1 = 2 CPUs per job here)
    fs, fc, st = privileged_case(orc, [1, 1], [0, 1], [4, 4], [0, 0], [5, 5], [100, 100], [0, 0])
    assert st.tolist() == [0, 0]
    fs, fc, st = privileged_case(orc, [1, 1], [0, 0], [2, 2], [1, 1], [100], [3], [0, 0])
    assert fs.tolist() == [1, -1] and fc.tolist() == [1, 0] and st.tolist() == [0, 1]
    # with CPUs per GPU the demand is level * GPUs: 2 GPUs at 2 per GPU need 4
    fs, fc, st = privileged_case(orc, [1], [0], [2], [1], [100], [3], [0], mode=1)
    assert st.tolist() == [1]
    # no minimum demand, or an unknown tenant: a queued job waits, a running one goes on without a floor
    fs, fc, st = privileged_case(orc, [1, 1, 1, 1], [0, 9, 0, 9], [0, 4, 0, 4], [0] * 4, [100], [100], [0, 0, 4, 4])
    assert fs.tolist() == [-1] * 4 and st.tolist() == [1, 1, 0, 0]
    # best-effort jobs are left alone; states that are given are kept (a job that takes no part charges nothing,
    # a job that keeps what it holds is charged like any running job)
    fs, fc, st = privileged_case(orc, [0, 1, 1, 1], [0, 0, 0, 0], [4, 4, 4, 4], [0] * 4, [8], [100], [2, 4, 4, 0],
                                 state=[0, 1, 2, 0])
    assert fs.tolist() == [-1, -1, 2, 2] and st.tolist() == [0, 1, 2, 0]


def test_privileged_from_an_empty_cluster_is_the_privileged_phase_of_the_allocation(orc):
    """With nobody running and capacity to spare, the jobs that get a floor here are the jobs the allocation from scratch
    grants their minimum (its privileged phase has the same quota rule, pinned above)."""
    rng = np.random.default_rng(31)
    for trial in range(200):
        J, T = int(rng.integers(1, 12)), int(rng.integers(1, 4))
        guaranteed = (rng.uniform(size=J) < 0.6).astype(np.uint32)
        tenant = rng.integers(0, T + 1, J).astype(np.uint32)                # T = unknown tenant
        min_g = [int(rng.choice([0, 1, 2, 4, 8])) for _ in range(J)]
        min_c = rng.integers(0, 2, J).astype(np.uint32)
        quota_g, quota_c = rng.integers(0, 20, T).astype(np.uint32), rng.integers(0, 12, T).astype(np.uint32)
        fs, fc, st = privileged_case(orc, guaranteed, tenant, min_g, min_c, quota_g, quota_c, [0] * J)
        c = [1.0, 2.0, 3.0, 4.0]
        seg = [[1, 2, 4, 8].index(g) if g else -1 for g in min_g]
        a, _, _ = floors_case(orc, [c] * J, guaranteed, tenant, seg, min_c, quota_g, quota_c, G=10 ** 5)
        for j in range(J):
            if guaranteed[j]:
                assert (st[j] == 0) == (a["g"][j] > 0), (trial, j)                   # waits there, waits here
                assert (fs[j] >= 0) == (a["g"][j] > 0)
            else:
                assert st[j] == 0 and fs[j] == -1
