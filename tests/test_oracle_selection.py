"""Pins for the oracle's plan enumeration, best-plan search, curves and greedy
(paper Sec. 5.2) against brute force, numpy routines and invariants."""
import itertools

import numpy as np
import pytest

import workloads


# ---------------------------------------------------------------- enumeration
def brute_triples(l, b, mu, g_max, tp_max, pp_max, mu_mask=1):
    out = []
    for g in range(1, g_max + 1):
        found = []
        for d in range(1, g + 1):
            for t in range(1, g + 1):
                for p in range(1, g + 1):
                    if d * t * p != g:
                        continue
                    if t not in (1, 2, 4, 8) or t > tp_max or p > pp_max:
                        continue
                    if l % p:
                        continue
                    for v in range(4):                  # micro-batches of mu * 2^v samples
                        if (mu_mask >> v) & 1 and b % (d * mu * 2 ** v) == 0:
                            found.append((g, t, p, v, d))
        out += sorted(found)
    return [(d, t, p, v) for g, t, p, v, d in out]


@pytest.mark.parametrize("g_max,tp_max,pp_max,mu_mask", [(8, 8, 255, 1), (24, 4, 3, 1), (32, 2, 255, 1), (24, 8, 255, 0xF),
                                                       (16, 2, 4, 0x6)])
def test_enumeration_matches_brute_force(orc, g_max, tp_max, pp_max, mu_mask):
    ints = np.array([[12, 32, 1], [24, 64, 2], [40, 128, 4], [7, 6, 1], [32, 32, 4], [96, 48, 2]], np.uint32)
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=g_max, tp_max=tp_max, pp_max=pp_max, mu_mask=mu_mask))
    if mu_mask == 0xF:
        assert np.any(tb.triples[:, 3] == 3) and np.any(tb.triples[:, 3] == 0)
    for j, (l, b, mu) in enumerate(ints.tolist()):
        want = brute_triples(l, b, mu, g_max, tp_max, pp_max, mu_mask)
        got = [tuple(r) for r in tb.triples[tb.triple_off[j]:tb.triple_off[j + 1]].tolist()]
        assert got == want
        gs = [d * t * p for d, t, p, v in want]
        seg_g = tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]].tolist()
        assert seg_g == sorted(set(gs))
        firsts = tb.seg_first[tb.seg_off[j]:tb.seg_off[j + 1]].tolist()
        assert firsts == [gs.index(g) for g in seg_g]


def test_enumeration_jobs_without_plans(orc):
    # Sec. 3: a plan splits the global batch b into n = b/(d*mu) >= 1 micro-batches per replica and the l layers
    # into p stages; no layers, an empty batch, no micro-batch size, or a micro-batch that does not divide the
    # batch leave nothing to enumerate, whatever the neighbours are
    ints = np.array([[12, 32, 1], [0, 8, 1], [8, 0, 1], [8, 8, 0], [5, 7, 2], [12, 32, 1]], np.uint32)
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=16, mu_mask=0xF))
    n = np.diff(tb.triple_off).tolist()
    assert n[1:5] == [0, 0, 0, 0] and n[0] == n[5] > 0
    assert np.diff(tb.seg_off).tolist()[1:5] == [0, 0, 0, 0]


def test_enumeration_counts_ordered_factorisations(orc):
    # with the constraints lifted (layers and batch divisible by everything)
    # the triples of g are its ordered factorisations into three factors:
    # prod C(e_i + 2, 2) over the prime exponents -> g=1:1, 2:3, 4:6, 8:10
    ints = np.array([[840, 840 * 8, 1]], np.uint32)
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=8))
    g = tb.triples[:, :3].prod(axis=1)
    assert [(g == v).sum() for v in (1, 2, 4, 8)] == [1, 3, 6, 10]
    # g = 6 has 9 of them, 3 of which need t in {3, 6}
    assert (g == 6).sum() == 6


# ---------------------------------------------------------- argmax and curves
@pytest.fixture(scope="module")
def tiny_round(orc):
    wl = workloads.tiny()
    return wl, orc.schedule_round(wl)


def test_best_plan_matches_flat_argmax(orc, tiny_round):
    wl, r = tiny_round
    tb = r["table"]
    rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
    thr = r["thr"]
    k = 0
    for j in range(wl.n_jobs):
        nt = int(tb.triple_off[j + 1] - tb.triple_off[j])
        ns = int(tb.seg_off[j + 1] - tb.seg_off[j])
        block = thr[16 * rows * int(tb.triple_off[j]):16 * rows * int(tb.triple_off[j + 1])].reshape(rows, nt * 16)
        g_of_plan = np.repeat(tb.triples[tb.triple_off[j]:tb.triple_off[j + 1], :3].prod(axis=1), 16)
        for row in range(rows):
            for s in range(ns):
                g = tb.seg_g[tb.seg_off[j] + s]
                idx = np.flatnonzero(g_of_plan == g)
                vals = block[row, idx]
                want_thr = vals.max()
                want_plan = idx[np.argmax(vals)] if want_thr > 0 else orc.NO_PLAN   # argmax: first maximum
                assert r["best_thr64"][k] == want_thr
                assert r["best_plan"][k] == want_plan
                k += 1
    assert k == r["best_plan"].size


def test_best_plan_f32_and_ties(orc):
    ints = np.array([[8, 8, 1]], np.uint32)
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=4))
    grid = workloads.Grid(np.array([1], np.uint32), 0, np.array([1.0], np.float32), 0)
    n = tb.n_candidates(1)
    thr = np.zeros(n, np.float32)
    bt, bp = orc.best_plan(tb, grid, thr)
    assert (bp == orc.NO_PLAN).all() and (bt == 0).all()
    # equal maxima: the lowest plan index wins
    first2 = int(tb.seg_first[1]) * 16
    thr[first2 + 5] = 3.0
    thr[first2 + 9] = 3.0
    thr[first2 + 2] = 1.0
    bt, bp = orc.best_plan(tb, grid, thr)
    assert bp[1] == first2 + 5 and bt[1] == 3.0 and bp[0] == orc.NO_PLAN


def test_infeasible_never_chosen_and_monotone(orc):
    wl = workloads.stress(n_jobs=24)
    r = orc.schedule_round(wl, n_threads=4)
    tb = r["table"]
    n_cpu, n_mem = len(wl.grid.cpu_levels), len(wl.grid.mem_levels_gb)
    rows = n_cpu * n_mem
    assert ((r["thr"] > 0) == (r["reason"] == 0)).all()
    for j in range(wl.n_jobs):
        nt = int(tb.triple_off[j + 1] - tb.triple_off[j])
        ns = int(tb.seg_off[j + 1] - tb.seg_off[j])
        cb = 16 * rows * int(tb.triple_off[j])
        sb = rows * int(tb.seg_off[j])
        bt = r["best_thr"][sb:sb + rows * ns].reshape(n_cpu, n_mem, ns)
        bp = r["best_plan"][sb:sb + rows * ns].reshape(n_cpu, n_mem, ns)
        reason = r["reason"][cb:cb + rows * nt * 16].reshape(n_cpu, n_mem, nt * 16)
        for c, m, s in itertools.product(range(n_cpu), range(n_mem), range(ns)):
            if bp[c, m, s] != orc.NO_PLAN:
                assert reason[c, m, bp[c, m, s]] == 0
            else:
                assert bt[c, m, s] == 0
        # more CPUs per GPU or more host memory never hurts (fixed plan space)
        assert (np.diff(bt, axis=0) >= 0).all()
        assert (np.diff(bt, axis=1) >= 0).all()
        ct = r["curve_thr"][sb:sb + rows * ns].reshape(n_cpu, n_mem, ns)
        assert (np.diff(ct, axis=2) >= 0).all()


def test_curves_match_numpy_prefix_max(orc, tiny_round):
    wl, r = tiny_round
    tb = r["table"]
    rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
    for j in range(wl.n_jobs):
        ns = int(tb.seg_off[j + 1] - tb.seg_off[j])
        sb = rows * int(tb.seg_off[j])
        bt = r["best_thr"][sb:sb + rows * ns].reshape(rows, ns)
        bp = r["best_plan"][sb:sb + rows * ns].reshape(rows, ns)
        ct = r["curve_thr"][sb:sb + rows * ns].reshape(rows, ns)
        cp = r["curve_plan"][sb:sb + rows * ns].reshape(rows, ns)
        cg = r["curve_g"][sb:sb + rows * ns].reshape(rows, ns)
        assert (ct == np.maximum.accumulate(bt, axis=1)).all()
        seg_g = tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]]
        for row in range(rows):
            for s in range(ns):
                if ct[row, s] == 0:
                    assert cp[row, s] == orc.NO_PLAN and cg[row, s] == 0
                else:
                    first = int(np.argmax(bt[row, :s + 1] == ct[row, s]))   # smallest count reaching it
                    assert cg[row, s] == seg_g[first] and cp[row, s] == bp[row, first]


def test_curve_is_flat_over_useless_counts(orc):
    # hand-made best values: the curve keeps the earlier maximum (Fig. 6)
    ints = np.array([[8, 8, 1]], np.uint32)
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=8))
    assert tb.seg_g.tolist() == [1, 2, 4, 8]
    grid = workloads.Grid(np.array([1], np.uint32), 0, np.array([1.0], np.float32), 0)
    bt = np.array([2.0, 5.0, 0.0, 4.0], np.float32)
    bp = np.array([3, 17, orc.NO_PLAN, 99], np.uint32)
    ct, cp, cg = orc.curves(tb, grid, bt, bp)
    assert ct.tolist() == [2.0, 5.0, 5.0, 5.0]
    assert cp.tolist() == [3, 17, 17, 17] and cg.tolist() == [1, 2, 2, 2]


# -------------------------------------------------------------------- greedy
def exhaustive_best(values, G):
    """values[j][g] = normalised throughput of job j with g GPUs (g = 0..G)."""
    J = len(values)
    best = 0.0
    for alloc in itertools.product(range(G + 1), repeat=J):
        if sum(alloc) <= G:
            best = max(best, sum(values[j][alloc[j]] for j in range(J)))
    return best


def run_greedy_on(orc, curve_pts, G, ref=None, C=10 ** 6, host=1e9):
    """curve_pts[j] = list of best throughput at g = 1..g_max (every g valid)."""
    J, g_max = len(curve_pts), len(curve_pts[0])
    ints = np.tile(np.array([[1, 1, 1]], np.uint32), (J, 1))
    # batch 1 would forbid d > 1; use a batch divisible by every d <= g_max
    import math
    lcm = 1
    for v in range(1, g_max + 1):
        lcm = lcm * v // math.gcd(lcm, v)
    ints[:, 1] = lcm
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=g_max, tp_max=1))
    assert tb.seg_g.tolist() == list(range(1, g_max + 1)) * J
    grid = workloads.Grid(np.array([1], np.uint32), 0, np.array([1.0], np.float32), 0)
    bt = np.array(curve_pts, np.float32).reshape(-1)
    bp = np.arange(bt.size, dtype=np.uint32)
    bp[bt == 0] = orc.NO_PLAN
    ct, cp, cg = orc.curves(tb, grid, bt, bp)
    ref = np.ones(J, np.float32) if ref is None else np.asarray(ref, np.float32)
    cl = workloads.Cluster(G, C, host)
    return orc.greedy(ref, tb, grid, cl, bt, bp, ct)


def test_greedy_optimal_on_concave_curves(orc):
    rng = np.random.default_rng(7)
    for trial in range(20):
        J, G = 3, 6
        pts = []
        for _ in range(J):
            inc = np.sort(rng.uniform(0.1, 2.0, size=G))[::-1]            # decreasing gains -> concave
            pts.append(np.cumsum(inc).astype(np.float32).tolist())
        assign, total, _ = run_greedy_on(orc, pts, G)
        values = [[0.0] + p for p in pts]
        assert total == pytest.approx(exhaustive_best(values, G), rel=1e-6)
        assert assign["g"].sum() <= G


def test_greedy_is_where_unit_transfers_stop(orc):
    # Sec. 5.2, Algorithm 1's shrinking rule written out as a loop: the job with the lowest
    # slope gives one GPU to a job whose slope is higher, until no such pair is left.  On
    # concave curves with distinct gains that state is unique, whatever the starting point,
    # and it is the allocation the slope-ordered greedy computes in one go.
    rng = np.random.default_rng(23)
    for trial in range(20):
        J, G = 5, 12
        gains = np.sort(rng.uniform(0.1, 2.0, size=(J, G)).astype(np.float32), axis=1)[:, ::-1]
        assert np.unique(gains).size == gains.size
        pts = np.cumsum(gains.astype(np.float64), axis=1).astype(np.float32)
        values = np.concatenate([np.zeros((J, 1), np.float32), pts], axis=1)
        assign, total, _ = run_greedy_on(orc, pts.tolist(), G)
        for start in range(3):
            cuts = np.sort(rng.integers(0, G + 1, size=J - 1))
            held = np.diff(np.concatenate([[0], cuts, [G]])).astype(int)      # a random full split
            for _ in range(10 * G):
                down = [values[j][held[j]] - values[j][held[j] - 1] if held[j] else np.inf for j in range(J)]
                up = [values[j][held[j] + 1] - values[j][held[j]] if held[j] < G else -np.inf for j in range(J)]
                shrink = int(np.argmin(down))
                grow = int(np.argmax([up[j] if j != shrink else -np.inf for j in range(J)]))
                if not up[grow] > down[shrink]:
                    break
                held[shrink] -= 1
                held[grow] += 1
            else:
                raise AssertionError("the transfers did not stop")
            assert held.tolist() == assign["g"].tolist(), (trial, start)


def test_greedy_never_beats_optimum_and_respects_capacity(orc):
    rng = np.random.default_rng(11)
    for trial in range(20):
        J, G = 4, 7
        pts = []
        for _ in range(J):
            v = np.maximum.accumulate(rng.uniform(0, 3, size=8) * (rng.uniform(size=8) > 0.3))
            pts.append(v.astype(np.float32).tolist())
        assign, total, _ = run_greedy_on(orc, pts, G)
        values = [[0.0] + p for p in pts]
        assert total <= exhaustive_best(values, G) * (1 + 1e-6)
        assert assign["g"].sum() <= G
        for j in range(J):
            if assign["g"][j]:
                assert assign["thr"][j] == np.float32(pts[j][assign["g"][j] - 1])


def test_greedy_steeper_job_gets_more_than_even_split(orc):
    # two jobs on four GPUs, in the spirit of the paper's two-job micro-benchmark
    # (Sec. 7.2): the job that keeps gaining from GPUs gets 3, the flat one gets 1
    scaling = [1.0, 1.9, 2.7, 3.4]
    flat = [1.0, 1.1, 1.15, 1.18]
    assign, total, _ = run_greedy_on(orc, [flat, scaling], 4)
    assert assign["g"].tolist() == [1, 3]
    assert total == pytest.approx(1.0 + 2.7, rel=1e-6)


def test_greedy_crosses_flats_and_breaks_ties_low(orc):
    # job 0 only gains at g = 4 (flat before); look-ahead slope 4/4 = 1 per GPU
    # ties with job 1's 1 per GPU: lower job index first, then the rest to job 1
    a = [0.0, 0.0, 0.0, 4.0]
    b = [1.0, 2.0, 3.0, 4.0]
    assign, total, _ = run_greedy_on(orc, [a, b], 6)
    assert assign["g"].tolist() == [4, 2]
    assign, total, _ = run_greedy_on(orc, [a, b], 3)      # job 0's only step does not fit
    assert assign["g"].tolist() == [0, 3]
    # reference throughput normalises the gains
    assign, total, _ = run_greedy_on(orc, [b, b], 4, ref=[1.0, 0.5])
    assert assign["g"].tolist() == [0, 4] and total == pytest.approx(8.0)


def test_greedy_cpu_pass_and_memory_step(orc):
    # one valid GPU count per job (g = 1), three CPU levels, two memory tiers
    ints = np.array([[1, 1, 1], [1, 1, 1]], np.uint32)
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=1))
    grid = workloads.Grid(np.array([1, 2, 4], np.uint32), 0, np.array([10.0, 100.0], np.float32), 0)
    # layout [job][cpu][mem][seg]
    bt = np.array([[[1.0, 1.0], [1.5, 1.5], [1.6, 1.6]],        # job 0: same at both tiers
                   [[0.0, 1.0], [0.0, 3.0], [0.0, 3.2]]],       # job 1: needs the large tier
                  np.float32)
    bp = np.arange(bt.size, dtype=np.uint32).reshape(bt.shape)
    bp[bt == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, bt.reshape(-1), bp.reshape(-1))
    ref = np.ones(2, np.float32)
    # CPUs: 2 base + 3 spare: job 1's step 1->2 (gain 2/CPU) then job 0's 1->2 (0.5), then 1 CPU left:
    # job 1's 2->4 needs 2 -> no; job 0's 2->4 needs 2 -> no
    assign, total, _ = orc.greedy(ref, tb, grid, workloads.Cluster(2, 5, 110.0), bt.reshape(-1), bp.reshape(-1), ct)
    assert assign["c"].tolist() == [2, 2]
    assert assign["mem_gb"].tolist() == [10.0, 100.0]          # job 0 takes the small tier, leaving room
    assert assign["thr"].tolist() == [1.5, 3.0]
    assert assign["plan"].tolist() == [int(bp[0, 1, 0]), int(bp[1, 1, 1])]
    assert total == pytest.approx(4.5)
    # host memory too small for job 1's tier: it is dropped, its resources stay unused
    assign, total, _ = orc.greedy(ref, tb, grid, workloads.Cluster(2, 5, 50.0), bt.reshape(-1), bp.reshape(-1), ct)
    assert assign["g"].tolist() == [1, 0] and assign["plan"][1] == orc.NO_PLAN
    assert total == pytest.approx(1.5)
    # CPU capacity limits the GPU pass too: only one job can start with 1 CPU
    assign, total, _ = orc.greedy(ref, tb, grid, workloads.Cluster(2, 1, 500.0), bt.reshape(-1), bp.reshape(-1), ct)
    assert assign["g"].tolist() == [1, 0]                      # equal slopes: lower job index


def test_round_invariants_on_generated_configs(orc):
    for wl in (workloads.tiny(), workloads.paper_scale(), workloads.what_if(3, n_jobs=60)):
        r = orc.schedule_round(wl, n_threads=4)
        a = r["assign"]
        assert a["g"].sum() <= wl.cluster.G
        assert a["c"].sum() <= wl.cluster.C
        assert a["mem_gb"].sum() <= wl.cluster.host_mem_gb * (1 + 1e-6)
        sched = a["g"] > 0
        assert (a["plan"][sched] != orc.NO_PLAN).all() and (a["thr"][sched] > 0).all()
        assert (a["thr"][~sched] == 0).all()
        ref = wl.coef[:, 16].astype(np.float64)
        assert r["total"] == pytest.approx((a["thr"] / ref).sum(), rel=1e-6)
        # the granted plan uses exactly the granted GPUs and is feasible there
        tb = r["table"]
        for j in np.flatnonzero(sched):
            d, t, p, _ = tb.triples[tb.triple_off[j] + a["plan"][j] // 16]
            assert d * t * p == a["g"][j]


def test_threads_over_jobs_change_nothing(orc):
    # the oracle's enumeration, evaluation and best-plan search may share the jobs among host threads
    # (the benchmark times them that way): same arrays as on one thread, also with more threads than jobs
    wl = workloads.stress(n_jobs=11)
    one = orc.schedule_round(wl, n_threads=1)
    for n in (3, 16):
        many = orc.schedule_round(wl, n_threads=n)
        for k in ("triple_off", "triples", "seg_off", "seg_g", "seg_first"):
            assert np.array_equal(getattr(one["table"], k), getattr(many["table"], k))
        for k in ("thr", "reason", "best_thr64", "best_plan", "curve_thr", "assign"):
            assert np.array_equal(one[k], many[k])
