"""GPU parity: every entry point of the library against the CPU oracle on the
same seeded inputs.  Integer results (tables, feasibility bits, argmax on
given values, curves, allocation on given curves) must be bit-exact; predicted
throughputs must agree within 1e-5 relative; a best plan computed from the
GPU's own float32 throughputs may differ from the oracle's only where the
oracle's value of the GPU's choice is within 1e-5 relative of its maximum."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

REL = 1e-5


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from gpu_harness import DeviceRun
    return DeviceRun


def oracle_table_equal(tn, ot):
    assert np.array_equal(tn["triple_off"], ot.triple_off)
    assert np.array_equal(tn["seg_off"], ot.seg_off)
    assert np.array_equal(tn["triples"], ot.triples)
    assert np.array_equal(tn["seg_g"], ot.seg_g)
    assert np.array_equal(tn["seg_first"], ot.seg_first)


def check_thr(gpu_thr, gpu_feas, o_thr, o_reason):
    assert np.array_equal(gpu_feas, o_reason), "feasibility bits differ"
    assert np.array_equal(gpu_thr == 0, o_reason != 0)
    ok = o_reason == 0
    rel = np.abs(gpu_thr[ok].astype(np.float64) - o_thr[ok]) / o_thr[ok]
    assert rel.size == 0 or rel.max() <= REL, f"max rel err {rel.max():.3e}"
    return float(rel.max()) if rel.size else 0.0


def check_best_in_band(ot, n_rows, jb, je, o_thr, o_bt, o_bp, g_bt, g_bp):
    """g_* computed from the GPU's float32 throughputs; o_* from the oracle's float64."""
    assert np.array_equal(g_bp == 0xFFFFFFFF, o_bp == 0xFFFFFFFF)
    has = o_bp != 0xFFFFFFFF
    rel = np.abs(g_bt[has].astype(np.float64) - o_bt[has]) / o_bt[has]
    assert rel.size == 0 or rel.max() <= REL
    mism = np.flatnonzero(g_bp != o_bp)
    # oracle value of the GPU's choice must be inside the band
    if mism.size:
        seg_cnt = (ot.seg_off[jb + 1:je + 1] - ot.seg_off[jb:je]).astype(np.int64) * n_rows
        seg_end = np.cumsum(seg_cnt)
        job_of = np.searchsorted(seg_end, mism, side="right")
        for k, jl in zip(mism.tolist(), job_of.tolist()):
            j = jb + jl
            ns = int(ot.seg_off[j + 1] - ot.seg_off[j])
            nt = int(ot.triple_off[j + 1] - ot.triple_off[j])
            local = k - (seg_end[jl] - seg_cnt[jl])
            r = local // ns
            cbase = 16 * n_rows * int(ot.triple_off[j] - ot.triple_off[jb]) + r * nt * 16
            v = o_thr[cbase + int(g_bp[k])]
            assert v >= o_bt[k] * (1 - REL), f"segment {k}: GPU plan {g_bp[k]} is outside the tie band"
    return mism.size


@pytest.mark.parametrize("name", ["tiny", "paper_scale"])
def test_enumerate_small_configs(gpu, orc, name):
    wl = workloads.CONFIGS[name]()
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), orc.enumerate_plans(wl.ints, wl.bounds))
    run.close()


def test_enumerate_odd_jobs_and_bounds(gpu, orc):
    ints = np.array([[12, 32, 1], [24, 64, 2], [40, 128, 4], [7, 6, 1], [32, 32, 4], [96, 48, 2],
                     [5, 7, 2],           # micro-batch does not divide the batch: no plan
                     [1, 1, 1], [60, 360, 1], [97, 128, 1]], np.uint32)
    coef = np.tile(workloads.tiny().coef[:1], (len(ints), 1))
    for b in (workloads.Bounds(g_max=8), workloads.Bounds(g_max=24, tp_max=4, pp_max=3),
              workloads.Bounds(g_max=720, tp_max=2), workloads.Bounds(g_max=1, tp_max=1, pp_max=1),
              workloads.Bounds(g_max=65535, tp_max=8, pp_max=4095)):        # the largest bounds the library takes
        wl = workloads.Workload("odd", coef, ints, b, workloads.tiny().grid, workloads.Env(), workloads.Cluster(8, 8, 64.0))
        run = gpu(wl)
        run.enumerate()
        oracle_table_equal(run.table_numpy(), orc.enumerate_plans(ints, b))
        run.close()


def test_enumerate_jobs_that_share_a_search(gpu, orc):
    """Equal jobs are searched once (leader election through a hash table): all jobs equal,
    all jobs different, a few kinds in random order, equal b/mu from different (b, mu),
    and jobs without plans among them."""
    rng = np.random.default_rng(17)
    base = workloads.tiny()
    b = workloads.Bounds(g_max=64, tp_max=8, pp_max=16, mu_mask=0b11)
    same = np.tile(np.array([[24, 64, 2]], np.uint32), (5000, 1))
    ls, bs = np.meshgrid(np.arange(1, 71), np.arange(1, 61))
    different = np.stack([ls.ravel(), bs.ravel(), np.ones(ls.size, np.int64)], axis=1).astype(np.uint32)   # 4,200 kinds
    kinds = np.array([[12, 32, 1], [12, 64, 2], [12, 128, 4], [24, 32, 1], [5, 7, 2], [0, 8, 1], [8, 0, 1], [8, 8, 0],
                      [96, 96, 1], [40, 120, 3], [40, 80, 2], [6, 9, 2]], np.uint32)
    mixed = kinds[rng.integers(0, len(kinds), size=3001)]
    for ints in (same, different, mixed, mixed[:1], mixed[:257]):
        coef = np.tile(base.coef[:1], (len(ints), 1))
        wl = workloads.Workload("shared", coef, ints, b, base.grid, workloads.Env(), workloads.Cluster(8, 8, 64.0))
        run = gpu(wl)
        for _ in range(2):                   # the second call finds the context's buffers in place
            run.enumerate()
            oracle_table_equal(run.table_numpy(), orc.enumerate_plans(ints, b))
        run.close()


def test_enumerate_wide_jobs_and_limits(gpu, orc):
    """Jobs with far more triples than usual (the two-pass hand-over inside the
    enumeration has to widen its slots), and a job beyond the documented limit."""
    import paper_2408_08586_amd as rk
    base = workloads.tiny()
    ints = np.array([[96, 5040, 1], [60, 2520, 1], [12, 32, 1], [96, 1680, 1]], np.uint32)
    coef = np.tile(base.coef[:1], (len(ints), 1))
    b = workloads.Bounds(g_max=1024)
    wl = workloads.Workload("wide", coef, ints, b, base.grid, workloads.Env(), workloads.Cluster(8, 8, 64.0))
    ot = orc.enumerate_plans(ints, b)
    assert 1000 < int(ot.triple_off[1] - ot.triple_off[0]) <= 2048
    for _ in range(2):                       # first context call widens, later calls take the direct path
        run = gpu(wl)
        run.enumerate()
        oracle_table_equal(run.table_numpy(), ot)
        run.enumerate()
        oracle_table_equal(run.table_numpy(), ot)
        o_thr, o_reason = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, n_threads=8)
        thr, feas, n = run.eval()
        check_thr(run.host(thr, n), run.host(feas, n), o_thr, o_reason)
        bt, bp, ns = run.best(thr)
        o_bt, o_bp = orc.best_plan(ot, wl.grid, o_thr)
        check_best_in_band(ot, run.n_rows, 0, wl.n_jobs, o_thr, o_bt, o_bp, run.host(bt, ns), run.host(bp, ns).view(np.uint32))
        fbt, fbp, fct, fcp, fcg, _ = run.fused()
        assert np.array_equal(run.host(fbt, ns), run.host(bt, ns)) and np.array_equal(run.host(fbp, ns), run.host(bp, ns))
        # curves of rows far longer than a wavefront, on the oracle's best values: exact
        assert int(np.diff(ot.seg_off).max()) > 64
        e_bt, e_bp = orc.best_plan(ot, wl.grid, o_thr.astype(np.float32))
        ct, cp, cg = run.curves(run.dev_f32(e_bt), run.dev_u32(e_bp))
        e_ct, e_cp, e_cg = orc.curves(ot, wl.grid, e_bt, e_bp)
        assert np.array_equal(run.host(ct, ns), e_ct)
        assert np.array_equal(run.host(cp, ns).view(np.uint32), e_cp)
        assert np.array_equal(run.host(cg, ns).view(np.uint32), e_cg)
        ct2, cp2, cg2 = run.curves(bt, bp)
        for a, b in ((fct, ct2), (fcp, cp2), (fcg, cg2)):
            assert np.array_equal(run.host(a, ns), run.host(b, ns))
        run.close()
    too_wide = workloads.Workload("too_wide", coef[:1], np.array([[96, 720720, 1]], np.uint32), workloads.Bounds(g_max=4096),
                                  base.grid, workloads.Env(), workloads.Cluster(8, 8, 64.0))
    run = gpu(too_wide)
    with pytest.raises(rk.RkError) as e:
        run.enumerate()
    assert e.value.code == rk.RK_ERR_UNSUPPORTED
    run.close()


def test_enumerate_stress_sample(gpu, orc):
    wl = workloads.stress()
    run = gpu(wl)
    t = run.enumerate()
    tn = run.table_numpy()
    assert t.n_jobs == 10000
    pick = np.sort(np.random.default_rng(3).choice(wl.n_jobs, 150, replace=False))
    ot = orc.enumerate_plans(wl.ints[pick], wl.bounds)
    for i, j in enumerate(pick.tolist()):
        a, b = tn["triple_off"][j], tn["triple_off"][j + 1]
        assert np.array_equal(tn["triples"][a:b], ot.triples[ot.triple_off[i]:ot.triple_off[i + 1]])
        a, b = tn["seg_off"][j], tn["seg_off"][j + 1]
        assert np.array_equal(tn["seg_g"][a:b], ot.seg_g[ot.seg_off[i]:ot.seg_off[i + 1]])
        assert np.array_equal(tn["seg_first"][a:b], ot.seg_first[ot.seg_off[i]:ot.seg_off[i + 1]])
    run.close()


@pytest.mark.parametrize("name", ["tiny", "paper_scale", "large"])
def test_eval_and_selection_full_configs(gpu, orc, name):
    wl = workloads.CONFIGS[name]()
    run = gpu(wl)
    run.enumerate()
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    o_thr, o_reason = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, n_threads=16)
    thr, feas, n = run.eval()
    g_thr, g_feas = run.host(thr, n), run.host(feas, n)
    err = check_thr(g_thr, g_feas, o_thr, o_reason)
    # best plan on the oracle's own float32 values: exact
    o32 = o_thr.astype(np.float32)
    bt, bp, ns = run.best(run.dev_f32(o32))
    e_bt, e_bp = orc.best_plan(ot, wl.grid, o32)
    assert np.array_equal(run.host(bt, ns), e_bt) and np.array_equal(run.host(bp, ns).view(np.uint32), e_bp)
    # best plan on the GPU's values against the oracle's float64 search: tie band
    bt2, bp2, _ = run.best(thr)
    o_bt, o_bp = orc.best_plan(ot, wl.grid, o_thr)
    n_mis = check_best_in_band(ot, run.n_rows, 0, wl.n_jobs, o_thr, o_bt, o_bp, run.host(bt2, ns),
                               run.host(bp2, ns).view(np.uint32))
    assert n_mis <= 0.01 * ns
    # curves on the oracle's best values: exact
    ct, cp, cg = run.curves(run.dev_f32(e_bt), run.dev_u32(e_bp))
    e_ct, e_cp, e_cg = orc.curves(ot, wl.grid, e_bt, e_bp)
    assert np.array_equal(run.host(ct, ns), e_ct)
    assert np.array_equal(run.host(cp, ns).view(np.uint32), e_cp)
    assert np.array_equal(run.host(cg, ns).view(np.uint32), e_cg)
    # the fused entry point gives exactly what the three calls give
    fbt, fbp, fct, fcp, fcg, _ = run.fused()
    ct2, cp2, cg2 = run.curves(bt2, bp2)
    for a, b in ((fbt, bt2), (fbp, bp2), (fct, ct2), (fcp, cp2), (fcg, cg2)):
        assert np.array_equal(run.host(a, ns), run.host(b, ns))
    print(f"{name}: {n} candidates, max rel err {err:.2e}, {n_mis}/{ns} best plans differ inside the band")
    run.close()


def test_eval_job_ranges_match_full_run(gpu, orc):
    wl = workloads.paper_scale()
    run = gpu(wl)
    run.enumerate()
    thr, feas, n = run.eval()
    full = run.host(thr, n)
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    for jb, je in ((0, 1), (5, 23), (63, 64), (17, 17)):
        t2, _, n2 = run.eval(jb, je, want_feas=False)
        a = 16 * run.n_rows * int(ot.triple_off[jb])
        assert np.array_equal(run.host(t2, n2), full[a:a + n2])
        if n2:
            bt, bp, ns = run.best(t2, jb, je)
            o_thr, _ = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, jb, je)
            o_bt, o_bp = orc.best_plan(ot, wl.grid, o_thr, jb, je)
            check_best_in_band(ot, run.n_rows, jb, je, o_thr, o_bt, o_bp, run.host(bt, ns),
                               run.host(bp, ns).view(np.uint32))
    run.close()


def test_stress_config_sampled_jobs(gpu, orc):
    """Full 10,000-job configuration in the chunking the benchmark uses;
    the oracle checks a seeded sample of jobs one by one."""
    wl = workloads.stress()
    run = gpu(wl)
    t = run.enumerate()
    tn = run.table_numpy()
    rng = np.random.default_rng(5)
    n_chunks = 3
    edges = np.linspace(0, wl.n_jobs, n_chunks + 1).astype(int)
    worst, n_mis, n_seg = 0.0, 0, 0
    parts = []
    for jb, je in zip(edges[:-1], edges[1:]):
        thr, feas, n = run.eval(int(jb), int(je))
        bt, bp, ns = run.best(thr, int(jb), int(je))
        ct, cp, cg = run.curves(bt, bp, int(jb), int(je))
        g_thr, g_feas = run.host(thr, n), run.host(feas, n)
        g_bt, g_bp = run.host(bt, ns), run.host(bp, ns).view(np.uint32)
        g_ct, g_cp, g_cg = run.host(ct, ns), run.host(cp, ns).view(np.uint32), run.host(cg, ns).view(np.uint32)
        parts.append((g_bt, g_bp, g_ct, g_cp, g_cg))
        for j in np.sort(rng.choice(np.arange(jb, je), 12, replace=False)).tolist():
            # curves at full size, by their definition on the library's own best values: running maximum along every
            # row, plan and GPU count of the first segment that reaches it
            nsj = int(tn["seg_off"][j + 1] - tn["seg_off"][j])
            s_at = run.n_rows * int(tn["seg_off"][j] - tn["seg_off"][jb])
            seg_g = tn["seg_g"][tn["seg_off"][j]:tn["seg_off"][j + 1]]
            for r in range(run.n_rows):
                row = slice(s_at + r * nsj, s_at + (r + 1) * nsj)
                v = g_bt[row]
                top = np.maximum.accumulate(v)
                first = np.array([int(np.argmax(v[:k + 1] == top[k])) for k in range(nsj)])
                assert np.array_equal(g_ct[row], top)
                assert np.array_equal(g_cp[row], np.where(top > 0, g_bp[row][first], 0xFFFFFFFF))
                assert np.array_equal(g_cg[row], np.where(top > 0, seg_g[first], 0))
            sub = wl.subset([j])
            ot = orc.enumerate_plans(sub.ints, sub.bounds)
            o_thr, o_reason = orc.eval_jobs(sub.coef, sub.ints, sub.bounds, ot, sub.grid, sub.env)
            a = 16 * run.n_rows * int(tn["triple_off"][j] - tn["triple_off"][jb])
            worst = max(worst, check_thr(g_thr[a:a + o_thr.size], g_feas[a:a + o_thr.size], o_thr, o_reason))
            o_bt, o_bp = orc.best_plan(ot, sub.grid, o_thr)
            s = run.n_rows * int(tn["seg_off"][j] - tn["seg_off"][jb])
            n_mis += check_best_in_band(ot, run.n_rows, 0, 1, o_thr, o_bt, o_bp, g_bt[s:s + o_bt.size],
                                        g_bp[s:s + o_bt.size])
            n_seg += o_bt.size
    print(f"stress: max rel err {worst:.2e}; {n_mis}/{n_seg} sampled best plans differ inside the band")
    assert n_mis <= 0.01 * n_seg
    # the benchmark takes the curves of all jobs in one call after the last chunk: same values as chunk by chunk
    whole = [np.concatenate([p[k] for p in parts]) for k in range(5)]
    ct, cp, cg = run.curves(run.dev_f32(whole[0]), run.dev_u32(whole[1]))
    for got, want in zip((ct, cp, cg), whole[2:]):
        assert np.array_equal(run.host(got, want.size).view(want.dtype), want)
    run.close()


@pytest.mark.parametrize("name", ["tiny", "paper_scale", "large"])
def test_allocate_on_oracle_curves_is_exact(gpu, orc, name):
    wl = workloads.CONFIGS[name]()
    r = orc.schedule_round(wl, n_threads=16)
    run = gpu(wl)
    run.enumerate()
    assign, total = run.allocate(run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]), run.dev_f32(r["curve_thr"]))
    assert np.array_equal(assign, r["assign"])
    assert total == pytest.approx(r["total"], rel=1e-6)
    # scarce capacities exercise the admissibility and memory rules
    for G, Cc, M in ((wl.cluster.G // 3, wl.cluster.C // 50 + 3, wl.cluster.host_mem_gb / 7), (1, 1, 64.0), (0, 0, 0.0)):
        cl = workloads.Cluster(G, Cc, M)
        e_assign, e_total, _ = orc.greedy(wl.coef[:, 16], r["table"], wl.grid, cl, r["best_thr"], r["best_plan"], r["curve_thr"])
        import paper_2408_08586_amd as rk
        assign, total = run.allocate(run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]),
                                     run.dev_f32(r["curve_thr"]), cluster=rk.make_cluster(cl))
        assert np.array_equal(assign, e_assign)
        assert total == pytest.approx(e_total, rel=1e-6, abs=1e-12)
    run.close()


@pytest.mark.parametrize("n_jobs,n_cpu", [(3000, 5), (12288, 5), (3000, 32), (12288, 7)])
def test_allocate_many_jobs_random_curves(gpu, orc, n_jobs, n_cpu):
    """The allocation alone at its largest sizes: the per-segment values are
    drawn here (not produced by either implementation), so both sides see the
    same float32 inputs and must return identical records.  With 5 CPU levels
    one workgroup selects the CPU pass of a round; with 32 levels (3,000 jobs)
    and 7 levels (12,288 jobs) the walks are too many for that and the
    histogram kernels take it."""
    import paper_2408_08586_amd as rk
    rng = np.random.default_rng(n_jobs + n_cpu)
    base = workloads.stress(n_jobs=n_jobs)
    b = workloads.Bounds(g_max=64)
    grid = base.grid if n_cpu == 5 else workloads.Grid(np.arange(1, n_cpu + 1, dtype=np.uint32), base.grid.cpu_mode,
                                                       base.grid.mem_levels_gb, base.grid.mem_mode)
    wl = workloads.Workload("alloc", base.coef, base.ints, b, grid, base.env, workloads.Cluster(4096, 30000, 2.0e5))
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    n_rows = n_cpu * len(grid.mem_levels_gb)
    n = ot.n_segments(n_rows)
    # throughput grows roughly with g, is noisy, sometimes infeasible, sometimes exactly tied
    g_of = np.concatenate([np.tile(ot.seg_g[ot.seg_off[j]:ot.seg_off[j + 1]], n_rows) for j in range(n_jobs)])
    bt = (g_of ** rng.uniform(0.3, 1.0, n)) * rng.uniform(0.5, 1.5, n)
    bt = np.round(bt * 8) / 8                                    # coarse values: many exact ties
    bt[rng.uniform(size=n) < 0.15] = 0
    bt = bt.astype(np.float32)
    bp = rng.integers(0, 1000, n).astype(np.uint32)
    bp[bt == 0] = 0xFFFFFFFF
    ct, _, _ = orc.curves(ot, wl.grid, bt, bp)
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    d_bt, d_bp, d_ct = run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct)
    for G, Cc, M in ((4096, 30000, 2.0e5), (4096, 5000, 1.0e9), (300, 100000, 3000.0), (20000, 10 ** 6, 1.0e9)):
        cl = workloads.Cluster(G, Cc, M)
        e_assign, e_total, _ = orc.greedy(wl.coef[:, 16], ot, wl.grid, cl, bt, bp, ct)
        assign, total = run.allocate(d_bt, d_bp, d_ct, cluster=rk.make_cluster(cl))
        assert np.array_equal(assign, e_assign), (G, Cc, M)
        assert total == pytest.approx(e_total, rel=1e-6)
        assert assign["g"].sum() <= G and assign["c"].sum() <= Cc
    run.close()


@pytest.mark.parametrize("g_max", [128, 1024])
def test_allocate_jobs_with_many_gpu_counts(gpu, orc, g_max):
    """Jobs with more than 32 (one wavefront per job) and more than 64 valid GPU
    counts (several rounds of 64 amounts inside a walk), on drawn values."""
    import paper_2408_08586_amd as rk
    rng = np.random.default_rng(g_max)
    base = workloads.tiny()
    kinds = np.array([[96, 5040, 1], [60, 2520, 1], [12, 32, 1], [96, 1680, 1]], np.uint32)
    ints = kinds[rng.integers(0, len(kinds), 120)]
    coef = np.tile(base.coef[:1], (len(ints), 1))
    coef[:, 16] = rng.uniform(0.5, 4.0, len(ints)).astype(np.float32)
    wl = workloads.Workload("many_counts", coef, ints, workloads.Bounds(g_max=g_max), base.grid, workloads.Env(),
                            workloads.Cluster(8, 8, 64.0))
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    widest = int(np.diff(ot.seg_off).max())
    assert widest > 64 if g_max == 1024 else 32 < widest <= 64
    n_rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
    n = ot.n_segments(n_rows)
    g_of = np.concatenate([np.tile(ot.seg_g[ot.seg_off[j]:ot.seg_off[j + 1]], n_rows) for j in range(wl.n_jobs)])
    bt = (g_of ** rng.uniform(0.3, 1.0, n)) * rng.uniform(0.5, 1.5, n)
    bt = np.round(bt * 8) / 8
    bt[rng.uniform(size=n) < 0.15] = 0
    bt = bt.astype(np.float32)
    bp = rng.integers(0, 1000, n).astype(np.uint32)
    bp[bt == 0] = 0xFFFFFFFF
    ct, _, _ = orc.curves(ot, wl.grid, bt, bp)
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    d_bt, d_bp, d_ct = run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct)
    for G, Cc, M in ((3000, 50000, 1.0e6), (700, 2000, 1.0e6), (12000, 10 ** 6, 5000.0)):
        cl = workloads.Cluster(G, Cc, M)
        e_assign, e_total, _ = orc.greedy(wl.coef[:, 16], ot, wl.grid, cl, bt, bp, ct)
        assign, total = run.allocate(d_bt, d_bp, d_ct, cluster=rk.make_cluster(cl))
        assert np.array_equal(assign, e_assign), (G, Cc, M)
        assert total == pytest.approx(e_total, rel=1e-6)
    run.close()


def test_allocate_on_a_job_range(gpu, orc):
    """rk_allocate on jobs [5, 23) of a larger table, arrays in the layout of that range."""
    import paper_2408_08586_amd as rk
    wl = workloads.paper_scale()
    jb, je = 5, 23
    sub = wl.subset(np.arange(jb, je))
    sub.cluster = workloads.Cluster(20, 40, 600.0)
    r = orc.schedule_round(sub, n_threads=8)
    run = gpu(wl)
    run.enumerate()
    assign, total = run.allocate(run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]), run.dev_f32(r["curve_thr"]),
                                 cluster=rk.make_cluster(sub.cluster), jb=jb, je=je)
    assert np.array_equal(assign, r["assign"])
    assert total == pytest.approx(r["total"], rel=1e-6)
    run.close()


def test_schedule_rounds_uneven_batch(gpu, orc):
    """Rounds of different sizes in one batch, one of them empty."""
    import paper_2408_08586_amd as rk
    import torch
    sizes = [37, 0, 120, 5, 64]
    rounds = [workloads.what_if(10 + i, n_jobs=max(n, 1)).subset(np.arange(n)) for i, n in enumerate(sizes)]
    for i, w in enumerate(rounds):
        w.cluster = workloads.Cluster(40 + 30 * i, 300 + 200 * i, 3000.0 * (i + 1))
    coef = np.concatenate([w.coef for w in rounds])
    ints = np.concatenate([w.ints for w in rounds])
    base = rounds[0]
    wl = workloads.Workload("batch", coef, ints, base.bounds, base.grid, base.env, base.cluster)
    run = gpu(wl)
    round_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint32)
    assign = rk.new_assign(wl.n_jobs)
    totals = torch.zeros(len(sizes), dtype=torch.float32, device="cuda:0")
    rk.rk_schedule_rounds(run.ctx, run.jobs, run.bounds, run.grid, run.env, round_off,
                          [rk.make_cluster(w.cluster) for w in rounds], assign, totals)
    rk.rk_sync(run.ctx)
    a = rk.assign_to_numpy(assign)
    for i, w in enumerate(rounds):
        lo, hi = int(round_off[i]), int(round_off[i + 1])
        if hi == lo:
            assert float(totals[i].item()) == 0.0
            continue
        r = orc.schedule_round(w, n_threads=8)
        one = gpu(w)
        compare_rounds(orc, w, a[lo:hi], float(totals[i].item()), r, own_values(one))
        one.close()
        assert a[lo:hi]["g"].sum() <= w.cluster.G and a[lo:hi]["c"].sum() <= w.cluster.C
    run.close()


def own_values(run, jb=0, je=None):
    """The library's own per-segment maxima, best plans and curves of the run's jobs (rk_job_curves), as numpy."""
    if run.table is None:
        run.enumerate()
    bt, bp, ct, _, _, n = run.fused(jb, je)
    return run.host(bt, n).copy(), run.host(bp, n).view(np.uint32).copy(), run.host(ct, n).copy()


def compare_rounds(orc, wl, assign, total, r, own, expect_same=False, redo=None):
    """End-to-end result of a round against the oracle.  Three statements, the first two on every call:

    1. the oracle's greedy, run on the library's own float32 maxima and curves (`own`, from rk_job_curves), returns
       the library's records bit for bit (`redo(bt, bp, ct)` replaces the plain greedy, e.g. by the policy with floors);
    2. those values are the oracle's within the tolerance: maxima within 1e-5 relative of the float64 ones, the same
       segments empty, best plans equal or inside the 1e-5 band of the oracle's maximum;
    3. against the oracle's own round `r`: records equal where that is asked for (`expect_same`: the named
       configurations) or where every decision of the oracle's greedy was clear (smallest relative gap between a
       winning slope and its runner-up above 1e-5; a job may then still hold another CPU level where that changes its
       throughput by less than the tolerance), totals within 1e-5 there and wherever the same jobs are served.
       A near-tie that changes which jobs are served can move the total by a whole job, so nothing is asked of the
       total then; statements 1 and 2 still hold.
    Returns whether the records equal the oracle's."""
    table = r["table"] if "table" in r else orc.enumerate_plans(wl.ints, wl.bounds)
    bt, bp, ct = own
    if redo is None:
        e_assign, e_total, _ = orc.greedy(wl.coef[:, 16], table, wl.grid, wl.cluster, bt, bp, ct)
    else:
        e_assign, e_total = redo(bt, bp, ct)
    assert np.array_equal(assign, e_assign), "the library's allocation is not the oracle's greedy on the library's own curves"
    assert total == pytest.approx(e_total, rel=1e-6, abs=1e-12)
    if "thr" in r:
        n_rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
        check_best_in_band(table, n_rows, 0, wl.n_jobs, r["thr"], r["best_thr64"], r["best_plan"], bt, bp)
        e_ct, _, _ = orc.curves(table, wl.grid, bt, bp)
        assert np.array_equal(ct, e_ct)
    ra = r["assign"]
    same_gc = np.array_equal(assign["g"], ra["g"]) and np.array_equal(assign["c"], ra["c"])
    sched = assign["g"] > 0
    same = same_gc and np.array_equal(assign["mem_gb"], ra["mem_gb"]) and np.array_equal(assign["plan"], ra["plan"])
    if same_gc:
        assert np.array_equal(assign["mem_gb"], ra["mem_gb"])
        rel = np.abs(assign["thr"][sched].astype(np.float64) - ra["thr"][sched]) / ra["thr"][sched]
        assert rel.size == 0 or rel.max() <= REL
        # a plan may differ only inside the band, which statement 2 has checked segment by segment
    if expect_same:
        assert same, "records differ from the oracle's round"
    clear = r["min_gap"] > REL
    if clear and not same_gc:
        assert np.array_equal(assign["g"], ra["g"])
        moved = assign["c"] != ra["c"]
        want = ra["thr"][moved].astype(np.float64)
        assert np.all(np.abs(assign["thr"][moved] - want) <= REL * want)
    if clear or np.array_equal(sched, ra["g"] > 0):
        assert total == pytest.approx(r["total"], rel=REL)
    return same


@pytest.mark.parametrize("name", ["tiny", "paper_scale", "large"])
def test_schedule_round_end_to_end(gpu, orc, name):
    wl = workloads.CONFIGS[name]()
    r = orc.schedule_round(wl, n_threads=16)
    run = gpu(wl)
    assign, total = run.schedule_round()
    same = compare_rounds(orc, wl, assign, total, r, own_values(run), expect_same=True)
    assert assign["g"].sum() <= wl.cluster.G and assign["c"].sum() <= wl.cluster.C
    assert assign["mem_gb"].sum() <= wl.cluster.host_mem_gb * (1 + 1e-6)
    # a second run is bit-identical
    assign2, total2 = run.schedule_round()
    assert np.array_equal(assign, assign2) and total == total2
    print(f"{name}: assignments equal to the oracle's: {same}; oracle min slope gap {r['min_gap']:.2e}")
    run.close()


def test_schedule_round_stress_against_stored_oracle(gpu, orc):
    """Whole round on the 10,000-job workload against the oracle's stored result
    (tests/golden/stress_round.json, written by make_stress_round.py from the oracle alone)."""
    import json
    import os
    import paper_2408_08586_amd as rk
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "stress_round.json")))
    wl = workloads.stress()
    assert g["n_jobs"] == wl.n_jobs
    ref = np.zeros(wl.n_jobs, rk.ASSIGN_DTYPE)
    ref["plan"] = 0xFFFFFFFF
    for j, gg, c, mem, plan, thr in g["scheduled"]:
        ref[j] = (gg, c, mem, plan, thr)
    run = gpu(wl)
    assign, total = run.schedule_round()
    same = compare_rounds(orc, wl, assign, total, dict(assign=ref, total=g["total"], min_gap=g["min_gap"]), own_values(run),
                          expect_same=True)
    assert assign["g"].sum() <= wl.cluster.G and assign["c"].sum() <= wl.cluster.C
    assert run_table_counts(run) == (g["n_triples"], g["n_segments"])
    # the materialising entry points, chunked as in the benchmark, end in the same allocation
    t = run.enumerate()
    ns = t.n_segments(run.n_rows)
    bt, bp = run.f32(ns), run.i32(ns)
    ct, cp, cg = run.f32(ns), run.i32(ns), run.i32(ns)
    edges = np.linspace(0, wl.n_jobs, 4).astype(int)
    for jb, je in zip(edges[:-1], edges[1:]):
        thr, _, n = run.eval(int(jb), int(je), want_feas=False)
        s0 = run.n_rows * int(t.h_seg_off[jb])
        rk.rk_best_plan(run.ctx, t.c, run.grid, int(jb), int(je), thr, bt[s0:], bp[s0:])
        rk.rk_curves(run.ctx, t.c, run.grid, int(jb), int(je), bt[s0:], bp[s0:], ct[s0:], cp[s0:], cg[s0:])
    assign2, total2 = run.allocate(bt, bp, ct)
    assert np.array_equal(assign, assign2) and total == total2
    print(f"stress round: {int((assign['g'] > 0).sum())} jobs scheduled, equal to the oracle's records: {same}")
    run.close()


def run_table_counts(run):
    t = run.enumerate()
    return t.n_triples, t.n_segs


def test_schedule_rounds_batch_what_if(gpu, orc):
    import paper_2408_08586_amd as rk
    import torch
    rounds = [workloads.what_if(i, n_jobs=120) for i in range(6)]
    coef = np.concatenate([w.coef for w in rounds])
    ints = np.concatenate([w.ints for w in rounds])
    base = rounds[0]
    wl = workloads.Workload("batch", coef, ints, base.bounds, base.grid, base.env, base.cluster)
    run = gpu(wl)
    round_off = np.arange(0, 121 * 6, 120, dtype=np.uint32)[:7]
    assign = rk.new_assign(wl.n_jobs)
    totals = torch.zeros(6, dtype=torch.float32, device="cuda:0")
    rk.rk_schedule_rounds(run.ctx, run.jobs, run.bounds, run.grid, run.env, round_off,
                          [rk.make_cluster(w.cluster) for w in rounds], assign, totals)
    rk.rk_sync(run.ctx)
    a = rk.assign_to_numpy(assign)
    for i, w in enumerate(rounds):
        r = orc.schedule_round(w, n_threads=8)
        one = gpu(w)
        compare_rounds(orc, w, a[i * 120:(i + 1) * 120], float(totals[i].item()), r, own_values(one))
        one.close()
    run.close()


def test_rounds_that_share_jobs(gpu, orc):
    """The same what-if rounds with every distinct job listed once: record for
    record what the concatenated batch gives, and the oracle's rounds."""
    import paper_2408_08586_amd as rk
    import torch
    n_rounds, n_jobs = 6, 120
    wl, round_off, round_jobs, clusters = workloads.what_if_shared(n_rounds, n_jobs=n_jobs)
    assert wl.n_jobs == n_jobs + n_rounds * (n_jobs // 10)
    run = gpu(wl)
    assign = rk.new_assign(n_rounds * n_jobs)
    totals = torch.zeros(n_rounds, dtype=torch.float32, device="cuda:0")
    c_clusters = [rk.make_cluster(c) for c in clusters]
    rk.rk_schedule_rounds_shared(run.ctx, run.jobs, run.bounds, run.grid, run.env, round_off, round_jobs, c_clusters,
                                 assign, totals)
    rk.rk_sync(run.ctx)
    a = rk.assign_to_numpy(assign)
    # the concatenated batch on the same context
    rounds = [workloads.what_if(i, n_jobs=n_jobs) for i in range(n_rounds)]
    cat = workloads.Workload("batch", np.concatenate([w.coef for w in rounds]), np.concatenate([w.ints for w in rounds]),
                             wl.bounds, wl.grid, wl.env, wl.cluster)
    run2 = gpu(cat)
    assign2 = rk.new_assign(n_rounds * n_jobs)
    totals2 = torch.zeros(n_rounds, dtype=torch.float32, device="cuda:0")
    rk.rk_schedule_rounds(run2.ctx, run2.jobs, run2.bounds, run2.grid, run2.env, round_off, c_clusters, assign2, totals2)
    rk.rk_sync(run2.ctx)
    assert np.array_equal(a, rk.assign_to_numpy(assign2)) and torch.equal(totals, totals2)
    for i, w in enumerate(rounds):
        one = gpu(w)
        compare_rounds(orc, w, a[i * n_jobs:(i + 1) * n_jobs], float(totals[i].item()), orc.schedule_round(w, n_threads=8),
                       own_values(one))
        one.close()
    # a round may be empty, a job may serve no round at all; a bad index is an error
    off2 = np.array([0, 0, 5, 5], np.uint32)
    jobs2 = np.array([7, 3, 150, 3 + n_jobs, 0], np.uint32)
    assign3 = rk.new_assign(5)
    totals3 = torch.zeros(3, dtype=torch.float32, device="cuda:0")
    rk.rk_schedule_rounds_shared(run.ctx, run.jobs, run.bounds, run.grid, run.env, off2, jobs2, c_clusters[:3], assign3, totals3)
    rk.rk_sync(run.ctx)
    sub = wl.subset(jobs2)
    sub.cluster = clusters[1]
    r = orc.schedule_round(sub, n_threads=4)
    one = gpu(sub)
    compare_rounds(orc, sub, rk.assign_to_numpy(assign3), float(totals3[1].item()), r, own_values(one))
    one.close()
    assert float(totals3[0].item()) == 0.0 and float(totals3[2].item()) == 0.0
    with pytest.raises(rk.RkError) as e:
        rk.rk_schedule_rounds_shared(run.ctx, run.jobs, run.bounds, run.grid, run.env, off2,
                                     np.array([7, 3, wl.n_jobs, 1, 0], np.uint32), c_clusters[:3], assign3, totals3)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    run.close()
    run2.close()


def test_edge_cases(gpu, orc):
    import paper_2408_08586_amd as rk
    base = workloads.tiny()
    # zero jobs
    wl = workloads.Workload("empty", base.coef[:0], base.ints[:0], base.bounds, base.grid, base.env, base.cluster)
    run = gpu(wl)
    t = run.enumerate()
    assert t.n_triples == 0 and t.n_segs == 0
    thr, feas, n = run.eval()
    assert n == 0
    assign, total = run.schedule_round()
    assert assign.size == 0 and total == 0.0
    run.close()
    # jobs, none of which has a plan: the table has no segment, the value arrays are empty (null pointers are fine)
    ints = np.array([[5, 7, 2], [0, 8, 1], [8, 0, 1]], np.uint32)
    wl = workloads.Workload("noplans", base.coef[:3], ints, base.bounds, base.grid, base.env, base.cluster)
    run = gpu(wl)
    t = run.enumerate()
    assert t.n_triples == 0 and t.n_segs == 0
    assign, total = run.allocate(None, None, None)
    assert (assign["g"] == 0).all() and (assign["plan"] == 0xFFFFFFFF).all() and total == 0.0
    assign, total = run.schedule_round()
    assert (assign["g"] == 0).all() and total == 0.0
    run.close()
    # a job without any plan among jobs that have plans; a cap nothing fits in
    ints = base.ints.copy()
    ints[3] = (5, 7, 2)
    env = workloads.Env(gpu_mem_cap=1.0)
    wl = workloads.Workload("nofit", base.coef, ints, base.bounds, base.grid, env, base.cluster)
    run = gpu(wl)
    run.enumerate()
    tn = run.table_numpy()
    assert tn["triple_off"][4] == tn["triple_off"][3]
    thr, feas, n = run.eval()
    assert (run.host(thr, n) == 0).all() and (run.host(feas, n) != 0).all()
    bt, bp, ns = run.best(thr)
    assert (run.host(bp, ns).view(np.uint32) == 0xFFFFFFFF).all() and (run.host(bt, ns) == 0).all()
    assign, total = run.schedule_round()
    assert (assign["g"] == 0).all() and (assign["plan"] == 0xFFFFFFFF).all() and total == 0.0
    # capacity errors report the needed size and leave the context usable
    small = run.f32(16)
    with pytest.raises(rk.RkError) as e:
        rk.rk_eval_candidates(run.ctx, run.jobs, run.table.c, run.grid, run.env, 0, wl.n_jobs, small, None)
    assert e.value.code == rk.RK_ERR_CAPACITY
    tbl = rk.PlanTable(wl.n_jobs, 3, 3)
    with pytest.raises(rk.RkError) as e:
        rk.rk_enumerate_plans(run.ctx, run.jobs, run.bounds, tbl.c)
    assert e.value.code == rk.RK_ERR_CAPACITY and tbl.n_triples == run.table.n_triples
    rk.rk_sync(run.ctx)            # the fill kernel is launched before the counts are known and must have held back
    assert not tbl.triples.any().item() and not tbl.seg_g.any().item() and not tbl.seg_first.any().item()
    bad = rk.make_grid(workloads.Grid(np.array([4, 2], np.uint32), 0, np.array([1.0], np.float32), 0))
    with pytest.raises(rk.RkError) as e:
        rk.rk_eval_candidates(run.ctx, run.jobs, run.table.c, bad, run.env, 0, wl.n_jobs, thr, None)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    with pytest.raises(rk.RkError) as e:
        rk.rk_eval_candidates(run.ctx, run.jobs, run.table.c, run.grid, run.env, 5, 3, thr, None)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    thr2, _, n2 = run.eval()
    assert np.array_equal(run.host(thr2, n2), run.host(thr, n))
    run.close()


def test_two_contexts_and_a_side_stream(gpu, orc):
    """Two contexts alive at once, one of them on a stream of its own (default priority): calls taken in turns
    give what each context gives alone."""
    import torch
    wl1, wl2 = workloads.tiny(), workloads.paper_scale()
    alone = []
    for wl in (wl1, wl2):
        run = gpu(wl)
        alone.append(run.schedule_round())
        run.close()
    side = torch.cuda.Stream()
    r1 = gpu(wl1)
    with torch.cuda.stream(side):
        r2 = gpu(wl2)                                    # the context takes the stream that is current: the side stream
    for _ in range(3):
        with torch.cuda.stream(side):
            b2 = r2.schedule_round()
            r2.enumerate()
            thr2, _, n2 = r2.eval(want_feas=False)
        b1 = r1.schedule_round()
        r1.enumerate()
        thr1, _, n1 = r1.eval(want_feas=False)
        assert np.array_equal(b1[0], alone[0][0]) and b1[1] == alone[0][1]
        assert np.array_equal(b2[0], alone[1][0]) and b2[1] == alone[1][1]
        with torch.cuda.stream(side):
            bt2, bp2, ns2 = r2.best(thr2)
            f2 = r2.fused()
            assert np.array_equal(r2.host(bt2, ns2), r2.host(f2[0], ns2))
        bt1, bp1, ns1 = r1.best(thr1)
        assert np.array_equal(r1.host(bt1, ns1), r1.host(r1.fused()[0], ns1))
    r1.close()
    with torch.cuda.stream(side):
        r2.close()


def test_option_masks_and_memory_modes(gpu, orc):
    base = workloads.paper_scale()
    b = workloads.Bounds(g_max=32, tp_max=4, pp_max=8, zero_mask=0b1101, gc_mask=0b11, off_mask=0b11)
    grid = workloads.Grid(np.array([1, 3, 4], np.uint32), 1, np.array([0.0, 8.0, 40.0], np.float32), 1)
    env = workloads.Env(gpu_mem_cap=40e9, gpus_per_node=4)
    wl = workloads.Workload("modes", base.coef[:24], base.ints[:24], b, grid, env, workloads.Cluster(40, 100, 900.0))
    run = gpu(wl)
    run.enumerate()
    ot = orc.enumerate_plans(wl.ints, wl.bounds)
    oracle_table_equal(run.table_numpy(), ot)
    o_thr, o_reason = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, n_threads=8)
    thr, feas, n = run.eval()
    check_thr(run.host(thr, n), run.host(feas, n), o_thr, o_reason)
    r = orc.schedule_round(wl, n_threads=8)
    assign, total = run.allocate(run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]), run.dev_f32(r["curve_thr"]))
    assert np.array_equal(assign, r["assign"])
    a2, t2 = run.schedule_round()
    compare_rounds(orc, wl, a2, t2, r, own_values(run))
    run.close()


def test_largest_allocation_grid(gpu, orc):
    """64 CPU levels x 16 host-memory tiers (the most the grid takes, 1,024 rows per job) on GPUs so small that
    offloaded plans, which need CPUs and host memory, are chosen: every stage against the oracle."""
    import dataclasses
    base = workloads.paper_scale()
    b = workloads.Bounds(g_max=16, tp_max=8, pp_max=8)
    grid = workloads.Grid(np.arange(1, 65, dtype=np.uint32), 1, (np.arange(16) * 12.5).astype(np.float32), 0)
    env = dataclasses.replace(base.env, gpu_mem_cap=4e9)
    used_levels, used_tiers = set(), set()
    for cl in (workloads.Cluster(64, 700, 300.0), workloads.Cluster(64, 20000, 1e5), workloads.Cluster(64, 700, 40.0)):
        wl = workloads.Workload("maxgrid", base.coef[:24], base.ints[:24], b, grid, env, cl)
        r = orc.schedule_round(wl, n_threads=16)
        run = gpu(wl)
        assert run.n_rows == 1024
        run.enumerate()
        ot = r["table"]
        oracle_table_equal(run.table_numpy(), ot)
        thr, feas, n = run.eval()
        check_thr(run.host(thr, n), run.host(feas, n), r["thr"], r["reason"])
        o32 = r["thr"].astype(np.float32)
        bt, bp, ns = run.best(run.dev_f32(o32))
        e_bt, e_bp = orc.best_plan(ot, wl.grid, o32)
        assert np.array_equal(run.host(bt, ns), e_bt) and np.array_equal(run.host(bp, ns).view(np.uint32), e_bp)
        ct, cp, cg = run.curves(bt, bp)
        e_ct, e_cp, e_cg = orc.curves(ot, wl.grid, e_bt, e_bp)
        for got, want in ((ct, e_ct), (cp, e_cp), (cg, e_cg)):
            assert np.array_equal(run.host(got, ns).view(want.dtype), want)
        bt2, bp2, _ = run.best(thr)
        fbt, fbp, fct, fcp, fcg, _ = run.fused()
        for a, c in zip((fbt, fbp, fct, fcp, fcg), (bt2, bp2) + run.curves(bt2, bp2)):
            assert np.array_equal(run.host(a, ns), run.host(c, ns))
        assign, total = run.allocate(run.dev_f32(r["best_thr"]), run.dev_u32(r["best_plan"]), run.dev_f32(r["curve_thr"]))
        assert np.array_equal(assign, r["assign"])
        a2, t2 = run.schedule_round()
        compare_rounds(orc, wl, a2, t2, r, own_values(run))
        got = r["assign"][r["assign"]["g"] > 0]
        used_levels |= set((got["c"] // got["g"]).tolist())
        used_tiers |= set(got["mem_gb"].tolist())
        run.close()
    assert len(used_levels) >= 5 and max(used_levels) == 64 and len(used_tiers) >= 3    # the case is not a trivial one


def test_fused_rows_that_do_not_fit_in_lds_at_once(gpu, orc):
    """Jobs with hundreds of GPU counts on 16 memory tiers: the keys of one CPU level's rows exceed what the fused
    kernel keeps in LDS, so it passes over the tiers as well.  Same bits as the three separate calls, the oracle's
    values, and the whole round."""
    base = workloads.paper_scale()
    ints = np.array([[2, 21621600, 1], [1, 21621600, 1], [24, 64, 2], [2, 3603600, 2]], np.uint32)
    coef = base.coef[[60, 61, 62, 63]].copy()                     # 5 to 60 billion parameters
    b = workloads.Bounds(g_max=20000, tp_max=2, pp_max=2)
    grid = workloads.Grid(np.array([1, 2, 6], np.uint32), 1, np.arange(16, dtype=np.float32), 1)     # GiB per GPU
    env = workloads.Env(gpu_mem_cap=3e9)
    wl = workloads.Workload("many_segments", coef, ints, b, grid, env, workloads.Cluster(30000, 200000, 1500.0))
    r = orc.schedule_round(wl, n_threads=16)
    ot = r["table"]
    assert int(np.diff(ot.seg_off).max()) * 16 * 8 > 48 * 1024 and int(np.diff(ot.triple_off).max()) <= 2048
    run = gpu(wl)
    run.enumerate()
    oracle_table_equal(run.table_numpy(), ot)
    thr, feas, n = run.eval()
    check_thr(run.host(thr, n), run.host(feas, n), r["thr"], r["reason"])
    bt, bp, ns = run.best(thr)
    ct, cp, cg = run.curves(bt, bp)
    for jb, je in ((0, wl.n_jobs), (1, 3)):
        f = run.fused(jb, je)
        s0, s1 = run.n_rows * int(ot.seg_off[jb]), run.n_rows * int(ot.seg_off[je])
        assert f[5] == s1 - s0
        for got, want in zip(f[:5], (bt, bp, ct, cp, cg)):
            assert np.array_equal(run.host(got, f[5]), run.host(want, ns)[s0:s1])
    # the tiers matter here: the best value of some segment differs between neighbouring tiers
    per_tier = run.host(bt, ns)[:run.n_rows * int(ot.seg_off[1])].reshape(3, 16, -1)
    assert (np.diff(per_tier, axis=1) > 0).sum() > 100
    a2, t2 = run.schedule_round()
    compare_rounds(orc, wl, a2, t2, r, own_values(run))
    run.close()


def test_micro_batch_sizes_as_a_plan_dimension(gpu, orc):
    """Bounds that allow micro-batches of mu, 2mu, 4mu and 8mu samples (Sec. 4.1
    "Gradient Accumulation"): table, candidates, best plans and the whole round
    against the oracle; with only mu allowed nothing changes."""
    import dataclasses
    for name, mask in (("tiny", 0xF), ("paper_scale", 0xF), ("paper_scale", 0x5)):
        base = workloads.CONFIGS[name]()
        wl = dataclasses.replace(base, bounds=dataclasses.replace(base.bounds, mu_mask=mask))
        ot = orc.enumerate_plans(wl.ints, wl.bounds)
        assert np.any(ot.triples[:, 3] > 0)
        run = gpu(wl)
        run.enumerate()
        oracle_table_equal(run.table_numpy(), ot)
        je = min(wl.n_jobs, 24)
        o_thr, o_reason = orc.eval_jobs(wl.coef, wl.ints, wl.bounds, ot, wl.grid, wl.env, 0, je, n_threads=16)
        thr, feas, n = run.eval(0, je)
        check_thr(run.host(thr, n), run.host(feas, n), o_thr, o_reason)
        bt, bp, ns = run.best(thr, 0, je)
        o_bt, o_bp = orc.best_plan(ot, wl.grid, o_thr, 0, je)
        check_best_in_band(ot, run.n_rows, 0, je, o_thr, o_bt, o_bp, run.host(bt, ns), run.host(bp, ns).view(np.uint32))
        fbt, fbp, fct, fcp, fcg, _ = run.fused(0, je)
        assert np.array_equal(run.host(fbt, ns), run.host(bt, ns)) and np.array_equal(run.host(fbp, ns), run.host(bp, ns))
        r = orc.schedule_round(wl, n_threads=16)
        assign, total = run.schedule_round()
        same = compare_rounds(orc, wl, assign, total, r, own_values(run))
        # some chosen plans do use a larger micro-batch
        sched = np.flatnonzero(assign["g"] > 0)
        shifts = [int(ot.triples[ot.triple_off[j] + assign["plan"][j] // 16, 3]) for j in sched]
        print(f"{name} mask {mask:#x}: assignments equal: {same}; micro-batch shifts of the chosen plans: {sorted(set(shifts))}")
        run.close()
    # the default mask leaves the table as it was
    base = workloads.paper_scale()
    wl = dataclasses.replace(base, bounds=dataclasses.replace(base.bounds, mu_mask=1))
    run = gpu(wl)
    run.enumerate()
    assert np.all(run.table_numpy()["triples"][:, 3] == 0)
    run.close()
    import paper_2408_08586_amd as rk
    bad = dataclasses.replace(base, bounds=dataclasses.replace(base.bounds, mu_mask=0))
    run = gpu(bad)
    with pytest.raises(rk.RkError) as e:
        run.enumerate()
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    run.close()
