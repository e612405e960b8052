"""GPU parity of rk_reschedule (Algorithm 1's Schedule as a loop from the jobs'
present state) against the oracle's ork_reschedule_f32 on shared float32
inputs: records, totals and the number of committed steps must be identical."""
import math

import numpy as np
import pytest

import workloads
from test_oracle_reschedule import table_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def on_gpu(run, bt, bp, ct, cluster, cur_seg, cur_c, floor_seg, floor_c, state):
    import torch
    import paper_2408_08586_amd as rk
    J = run.wl.n_jobs
    dev = run.device
    i32 = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    u8 = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(dev)
    assign, total = rk.new_assign(J, dev), run.f32(1)
    moves = torch.zeros(4, dtype=torch.int32, device=dev)
    rk.rk_reschedule(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, rk.make_cluster(cluster), run.dev_f32(bt), run.dev_u32(bp),
                     run.dev_f32(ct), i32(cur_seg), run.dev_u32(cur_c), assign, total, state=u8(state), floor_seg=i32(floor_seg),
                     floor_c=None if floor_c is None else run.dev_u32(floor_c), n_moves=moves)
    rk.rk_sync(run.ctx)
    return rk.assign_to_numpy(assign), float(total[0].item()), int(moves[0].item())


def same(got, want):
    assert np.array_equal(got[0], want[0]), np.flatnonzero(got[0] != want[0])[:5]
    assert got[1] == pytest.approx(want[1], rel=1e-6, abs=1e-12)
    assert got[2] == want[2]


def random_round(rng, orc, J=None, g_max=None):
    """A round on drawn values: every GPU count 1..g_max is a segment, some counts are not valid (value 0), several CPU
    levels and memory tiers in either mode, a random present state with floors and jobs that take no part."""
    if J is None:
        J, g_max = int(rng.integers(1, 41)), int(rng.integers(2, 17))
    big = J > 64
    n_cpu, n_mem = int(rng.integers(1, 5)), int(rng.integers(1, 4))
    tb = table_for(orc, J, g_max)
    grid = workloads.Grid(np.sort(rng.choice(np.arange(1, 9), n_cpu, replace=False)).astype(np.uint32), int(rng.integers(0, 2)),
                          np.sort(rng.choice(np.array([0, 4, 16, 64], np.float32), n_mem, replace=False)).astype(np.float32),
                          int(rng.integers(0, 2)))
    bt = np.zeros((J, n_cpu, n_mem, g_max), np.float32)
    for j in range(J):
        valid = np.unique(np.concatenate([[1], rng.choice(np.arange(1, g_max + 1), int(rng.integers(1, 6)))]))
        base = np.zeros(g_max)
        base[valid - 1] = np.cumsum(np.sort(rng.uniform(0.2, 2.0, len(valid)))[::-1] * rng.uniform(0.5, 1.5, len(valid)))
        base = np.round(base * 16) / 16                                      # coarse: exact ties do occur
        for c in range(n_cpu):
            for m in range(n_mem):
                v = base * (1 + 0.25 * c * rng.uniform(0, 1)) * (1.0 if m == n_mem - 1 else rng.choice([0.0, 0.8, 1.0]))
                bt[j, c, m] = np.round(v * 16) / 16
        bt[j] = np.maximum.accumulate(np.maximum.accumulate(bt[j], axis=0), axis=1)   # more CPUs or memory never hurt
    flat = bt.reshape(-1)
    bp = rng.integers(0, 1000, flat.size).astype(np.uint32)
    bp[flat == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, flat, bp)
    ref = rng.uniform(0.5, 2.0, J).astype(np.float32)
    G = int(rng.integers(J // 4, 2 * J + 1)) if big else int(rng.integers(0, 3 * g_max + 1))
    cl = workloads.Cluster(G, int(rng.integers(G if big else 0, 12 * max(G, 1))), float(rng.choice([0.0, 16.0, 200.0, 1e6])))
    cur_seg, cur_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    floor_seg, floor_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    left = G
    for j in rng.permutation(J).tolist():
        ok = np.flatnonzero(bt[j, 0, n_mem - 1] > 0)
        if rng.uniform() < 0.3:
            floor_seg[j], floor_c[j] = int(rng.choice(ok)), int(rng.integers(0, n_cpu))
        if rng.uniform() < 0.5:
            fit = ok[(ok + 1 <= left) & (ok >= floor_seg[j])] if rng.uniform() < 0.9 else ok[ok + 1 <= left]
            if fit.size:
                cur_seg[j], cur_c[j] = int(rng.choice(fit)), int(rng.integers(0, n_cpu))
                left -= cur_seg[j] + 1
    state = (rng.uniform(size=J) < 0.1).astype(np.uint8)
    state[rng.uniform(size=J) < 0.1] = 2                    # jobs that keep exactly what they hold
    coef = np.tile(workloads.tiny().coef[:1], (J, 1))
    coef[:, 16] = ref
    ints = np.tile(np.array([[1, math.lcm(*range(1, g_max + 1)), 1]], np.uint32), (J, 1))   # as table_for builds its table
    wl = workloads.Workload("drawn", coef, ints, workloads.Bounds(g_max=g_max, tp_max=1), grid, workloads.Env(), cl)
    return wl, tb, flat, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state


def test_random_rounds_on_drawn_values(gpu, orc):
    n_moves = n_priv = 0
    for seed in range(400):
        rng = np.random.default_rng(95000 + seed)
        wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = random_round(rng, orc)
        use_floor = seed % 4 != 0
        use_state = seed % 3 != 0
        want = orc.reschedule(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct, cur_seg, cur_c,
                              floor_seg if use_floor else None, floor_c if use_floor else None, state=state if use_state else None)
        run = gpu(wl)
        run.enumerate()
        assert np.array_equal(run.table_numpy()["seg_g"], tb.seg_g)
        got = on_gpu(run, bt, bp, ct, wl.cluster, cur_seg, cur_c, floor_seg if use_floor else None,
                     floor_c if use_floor else None, state if use_state else None)
        run.close()
        same(got, want)
        n_moves += want[2]
        n_priv += int(use_floor and np.any((floor_seg >= 0) & (cur_seg < floor_seg)))
    print(f"400 rounds, {n_moves} steps committed, {n_priv} rounds with privileged jobs")
    assert n_moves > 1500 and n_priv > 100


def test_states_outside_their_ranges(gpu, orc):
    """What a caller may get wrong without an error: a held GPU count or CPU level the job does not have (the job then
    holds nothing), a floor that is no index of its list (no floor), a floor's CPU level beyond the grid (clamped), a
    state byte other than 0 (2: keeps what it holds; anything else: takes no part), jobs that hold more than the cluster has.  Both sides read them alike."""
    n_moves = 0
    for seed in range(60):
        rng = np.random.default_rng(97000 + seed)
        wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = random_round(rng, orc)
        J, g_max, n_cpu = wl.n_jobs, wl.bounds.g_max, len(wl.grid.cpu_levels)
        for j in range(J):
            u = rng.uniform()
            if u < 0.10: cur_seg[j] = g_max + int(rng.integers(0, 3))
            elif u < 0.20: cur_c[j] = n_cpu + int(rng.integers(0, 3))
            elif u < 0.30: floor_seg[j] = g_max + int(rng.integers(0, 100))
            elif u < 0.40: floor_c[j] = n_cpu + int(rng.integers(0, 1000))
            elif u < 0.45: state[j] = int(rng.choice([2, 3, 7, 255]))
            elif u < 0.50: cur_seg[j], floor_seg[j] = -5, -7
        cl = wl.cluster if seed % 3 else workloads.Cluster(wl.cluster.G // 3, wl.cluster.C // 3, wl.cluster.host_mem_gb)
        want = orc.reschedule(wl.coef[:, 16], tb, wl.grid, cl, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state=state)
        run = gpu(wl)
        run.enumerate()
        got = on_gpu(run, bt, bp, ct, cl, cur_seg, cur_c, floor_seg, floor_c, state)
        run.close()
        same(got, want)
        n_moves += want[2]
    assert n_moves > 100


def test_larger_drawn_rounds(gpu, orc):
    """Rounds of hundreds to thousands of jobs with hundreds of committed steps each: a thread of the kernel then owns
    several jobs, the privileged list and the search for the next job to serve run over many wavefronts."""
    n_moves = 0
    for seed, J in enumerate([300, 1000, 1024, 1025, 2049, 3000] * 3):
        rng = np.random.default_rng(96000 + seed)
        wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = random_round(rng, orc, J, int(rng.integers(2, 23)))
        want = orc.reschedule(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state=state)
        run = gpu(wl)
        run.enumerate()
        assert np.array_equal(run.table_numpy()["seg_g"], tb.seg_g)
        got = on_gpu(run, bt, bp, ct, wl.cluster, cur_seg, cur_c, floor_seg, floor_c, state)
        run.close()
        same(got, want)
        n_moves += want[2]
    print(f"18 rounds, {n_moves} steps committed")
    assert n_moves > 3000


def test_the_largest_round(gpu, orc):
    """12,288 jobs, the most a round takes: every thread of the kernel owns twelve, the give-slopes fill 96 KiB of LDS."""
    rng = np.random.default_rng(96500)
    wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = random_round(rng, orc, 12288, 3)
    want = orc.reschedule(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state=state)
    run = gpu(wl)
    run.enumerate()
    got = on_gpu(run, bt, bp, ct, wl.cluster, cur_seg, cur_c, floor_seg, floor_c, state)
    run.close()
    same(got, want)
    print(f"12,288 jobs, {want[2]} steps committed")
    assert want[2] > 500


def many_amounts_round(rng, orc, J):
    """A round whose jobs have 174 GPU counts each (the divisors of a global batch of 720,720 up to 4,096 GPUs, data
    parallel only): drawn values on some of them, a random present state with floors and jobs that take no part."""
    bounds = workloads.Bounds(g_max=4096, tp_max=1)
    ints = np.tile(np.array([[1, 720720, 1]], np.uint32), (J, 1))
    tb = orc.enumerate_plans(ints, bounds)
    ns = int(tb.seg_off[1])
    assert ns == 174 and np.all(np.diff(tb.seg_off) == ns)
    seg_g = np.asarray(tb.seg_g[:ns], dtype=np.int64)
    n_cpu, n_mem = int(rng.integers(1, 5)), int(rng.integers(1, 4))
    grid = workloads.Grid(np.sort(rng.choice(np.arange(1, 9), n_cpu, replace=False)).astype(np.uint32), int(rng.integers(0, 2)),
                          np.sort(rng.choice(np.array([0, 4, 16, 64], np.float32), n_mem, replace=False)).astype(np.float32),
                          int(rng.integers(0, 2)))
    bt = np.zeros((J, n_cpu, n_mem, ns), np.float32)
    for j in range(J):
        valid = np.unique(np.concatenate([[0], rng.choice(np.arange(ns), int(rng.integers(3, 60)))]))
        base = np.zeros(ns)
        base[valid] = np.cumsum(np.sort(rng.uniform(0.2, 2.0, len(valid)))[::-1] * rng.uniform(0.5, 1.5, len(valid)))
        base = np.round(base * 16) / 16
        for c in range(n_cpu):
            for m in range(n_mem):
                v = base * (1 + 0.25 * c * rng.uniform(0, 1)) * (1.0 if m == n_mem - 1 else rng.choice([0.0, 0.8, 1.0]))
                bt[j, c, m] = np.round(v * 16) / 16
        bt[j] = np.maximum.accumulate(np.maximum.accumulate(bt[j], axis=0), axis=1)
    flat = bt.reshape(-1)
    bp = rng.integers(0, 1000, flat.size).astype(np.uint32)
    bp[flat == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, flat, bp)
    ref = rng.uniform(0.5, 2.0, J).astype(np.float32)
    G = int(rng.integers(64, 4097))
    cl = workloads.Cluster(G, int(rng.integers(G, 12 * G)), float(rng.choice([0.0, 16.0, 200.0, 1e6])))
    cur_seg, cur_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    floor_seg, floor_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    left = G
    for j in rng.permutation(J).tolist():
        ok = np.flatnonzero(bt[j, 0, n_mem - 1] > 0)
        if rng.uniform() < 0.3:
            floor_seg[j], floor_c[j] = int(rng.choice(ok[:max(1, len(ok) // 3)])), int(rng.integers(0, n_cpu))
        if rng.uniform() < 0.6:
            fit = ok[(seg_g[ok] <= left // 2) & (ok >= floor_seg[j])]
            if fit.size:
                cur_seg[j], cur_c[j] = int(rng.choice(fit)), int(rng.integers(0, n_cpu))
                left -= int(seg_g[cur_seg[j]])
    state = (rng.uniform(size=J) < 0.1).astype(np.uint8)
    state[rng.uniform(size=J) < 0.1] = 2
    coef = np.tile(workloads.tiny().coef[:1], (J, 1))
    coef[:, 16] = ref
    wl = workloads.Workload("many amounts", coef, ints, bounds, grid, workloads.Env(), cl)
    return wl, tb, flat, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state


def test_jobs_with_more_amounts_than_a_wavefront_has_lanes(gpu, orc):
    """174 GPU counts per job: the steps of such a job are searched 64 amounts at a time, not from one register row."""
    n_moves = n_shrunk = 0
    for seed in range(40):
        rng = np.random.default_rng(98000 + seed)
        wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = many_amounts_round(rng, orc, int(rng.integers(3, 30)))
        want = orc.reschedule(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state=state)
        run = gpu(wl)
        run.enumerate()
        assert np.array_equal(run.table_numpy()["seg_g"], tb.seg_g)
        got = on_gpu(run, bt, bp, ct, wl.cluster, cur_seg, cur_c, floor_seg, floor_c, state)
        run.close()
        same(got, want)
        n_moves += want[2]
        held = np.where(cur_seg >= 0, np.asarray(tb.seg_g[:174])[np.maximum(cur_seg, 0)], 0)
        n_shrunk += int(np.sum((want[0]["g"] < held) & (state == 0)))
    print(f"40 rounds, {n_moves} steps committed, {n_shrunk} jobs hold less afterwards")
    assert n_moves > 150 and n_shrunk > 20


@pytest.mark.parametrize("name", ["paper_scale", "what_if", "stress"])
def test_generated_rounds_from_a_running_state(gpu, orc, name):
    """The state a from-scratch round leaves, then the cluster loses a tenth of its GPUs and CPUs, a tenth of the
    jobs leave and their slots are new arrivals, some jobs are guaranteed: the loop on the library's own curves,
    given to both sides."""
    import paper_2408_08586_amd as rk
    wl = {"paper_scale": workloads.paper_scale, "what_if": lambda: workloads.what_if(7), "stress": workloads.stress}[name]()
    J = wl.n_jobs
    rng = np.random.default_rng(J)
    run = gpu(wl)
    run.enumerate()
    bt, bp, ct, _, _, n = run.fused()
    bt, bp, ct = run.host(bt, n).copy(), run.host(bp, n).view(np.uint32).copy(), run.host(ct, n).copy()
    tn = run.table_numpy()
    tb = orc.Table(tn["triple_off"], tn["triples"], tn["seg_off"], tn["seg_g"], tn["seg_first"])
    a0, _, _ = orc.greedy(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct)
    cur_seg, cur_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    levels = np.asarray(wl.grid.cpu_levels)
    for j in np.flatnonzero(a0["g"] > 0).tolist():
        seg_g = tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]]
        cur_seg[j] = int(np.flatnonzero(seg_g == a0["g"][j])[0])
        per = a0["c"][j] // a0["g"][j] if wl.grid.cpu_mode else a0["c"][j]
        cur_c[j] = int(np.flatnonzero(levels == per)[0])
    gone = rng.uniform(size=J) < 0.1
    cur_seg[gone] = -1                                                       # left; the slot is a new arrival
    floor_seg, floor_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    ns = np.diff(tb.seg_off)
    guaranteed = (rng.uniform(size=J) < 0.05) & (ns > 0)
    floor_seg[guaranteed] = np.minimum(rng.integers(0, 3, guaranteed.sum()), ns[guaranteed] - 1)
    floor_seg[(cur_seg >= 0) & (floor_seg > cur_seg)] = -1                  # running jobs sit at or above their floor
    state = (rng.uniform(size=J) < 0.02).astype(np.uint8)
    cl = workloads.Cluster(int(wl.cluster.G * 0.9), int(wl.cluster.C * 0.9), wl.cluster.host_mem_gb)
    # the jobs that stayed hold more than the smaller cluster has only if the greedy had filled it; make room first
    held = sum(int(tb.seg_g[tb.seg_off[j] + cur_seg[j]]) for j in np.flatnonzero((cur_seg >= 0) & (state == 0)))
    if held > cl.G:
        cl = workloads.Cluster(held, cl.C, cl.host_mem_gb)
    want = orc.reschedule(wl.coef[:, 16], tb, wl.grid, cl, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state=state)
    got = on_gpu(run, bt, bp, ct, cl, cur_seg, cur_c, floor_seg, floor_c, state)
    same(got, want)
    a = got[0]
    print(f"{name}: {int((a0['g'] > 0).sum())} jobs ran, {int(gone.sum())} slots changed hands, {got[2]} steps committed, "
          f"{int((a['g'] > 0).sum())} jobs run now")
    assert got[2] > 0 and a["g"].sum() <= cl.G
    run.close()


def test_many_rounds_at_once(gpu, orc):
    """rk_reschedule_rounds: what-if rounds over the same jobs, a workgroup each - other capacities from one state,
    and other states (jobs that left, other floors) round by round; every round is the oracle's loop for its inputs."""
    import torch
    import paper_2408_08586_amd as rk
    for seed, (J, n_rounds, per_round) in enumerate([(40, 7, False), (300, 64, True), (1500, 33, True), (1, 3, False)]):
        rng = np.random.default_rng(98000 + seed)
        wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = random_round(rng, orc, J, int(rng.integers(2, 17)))
        base = wl.cluster
        clusters = [workloads.Cluster(int(base.G * u), int(base.C * u), base.host_mem_gb)
                    for u in rng.uniform(0.5, 1.5, n_rounds)]
        if per_round:                                        # every round its own state: some jobs have left, floors differ
            seg = np.tile(cur_seg, (n_rounds, 1))
            seg[rng.uniform(size=seg.shape) < 0.1] = -1
            fl = np.tile(floor_seg, (n_rounds, 1))
            fl[rng.uniform(size=fl.shape) < 0.2] = -1
            lv, fc, stt = np.tile(cur_c, (n_rounds, 1)), np.tile(floor_c, (n_rounds, 1)), np.tile(state, (n_rounds, 1))
        else:
            seg, fl, lv, fc, stt = cur_seg[None], floor_seg[None], cur_c[None], floor_c[None], state[None]
        run = gpu(wl)
        run.enumerate()
        dev = run.device
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32).reshape(-1)).to(dev)
        u8 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8).reshape(-1)).to(dev)
        assign = rk.new_assign(n_rounds * J, dev)
        totals = run.f32(n_rounds)
        stats = torch.zeros(4 * n_rounds, dtype=torch.int32, device=dev)
        rk.rk_reschedule_rounds(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, [rk.make_cluster(c) for c in clusters],
                                run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct), i32(seg), run.dev_u32(lv.reshape(-1)), assign,
                                totals, state_stride=J if per_round else 0, state=u8(stt), floor_seg=i32(fl),
                                floor_c=run.dev_u32(fc.reshape(-1)), stats=stats)
        rk.rk_sync(run.ctx)
        got_a = rk.assign_to_numpy(assign).reshape(n_rounds, J)
        got_t, got_s = totals.cpu().numpy()[:n_rounds], stats.cpu().numpy().reshape(n_rounds, 4)
        n_moves = 0
        for r in range(n_rounds):
            k = r if per_round else 0
            want = orc.reschedule(wl.coef[:, 16], tb, wl.grid, clusters[r], bt, bp, ct, seg[k], lv[k], fl[k], fc[k], state=stt[k])
            same((got_a[r], float(got_t[r]), int(got_s[r, 0])), want)
            n_moves += want[2]
        # one round through the same entry point is rk_reschedule
        one = on_gpu(run, bt, bp, ct, clusters[0], seg[0], lv[0], fl[0], fc[0], stt[0])
        assert np.array_equal(one[0], got_a[0]) and one[2] == got_s[0, 0]
        print(f"{n_rounds} rounds of {J} jobs: {n_moves} steps committed")
        run.close()


def test_argument_errors(gpu, orc):
    import paper_2408_08586_amd as rk
    wl = workloads.tiny()
    run = gpu(wl)
    run.enumerate()
    bt, bp, ct, _, _, n = run.fused()
    J = wl.n_jobs
    assign, total = rk.new_assign(J, run.device), run.f32(1)
    with pytest.raises(rk.RkError) as e:
        rk.rk_reschedule(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, bt, bp, ct, None, None, assign, total)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    # nobody holds anything, no floors: every job is a newcomer
    cur = run.torch.full((J,), -1, dtype=run.torch.int32, device=run.device)
    rk.rk_reschedule(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, bt, bp, ct, cur, run.i32(J).zero_(), assign,
                     total)
    rk.rk_sync(run.ctx)
    a = rk.assign_to_numpy(assign)
    assert 0 < a["g"].sum() <= wl.cluster.G
    run.close()
