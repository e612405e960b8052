"""GPU parity of rk_reschedule_nodes (Algorithm 1's Schedule with ScheduleJob
searching node by node) against the oracle's ork_reschedule_nodes_f32 on shared
float32 inputs: records, the new placement part by part, totals and the number
of committed steps must be identical; a state that is no placement on the
nodes must be refused by both."""
import numpy as np
import pytest

import workloads
from test_gpu_reschedule import random_round
from test_oracle_reschedule_nodes import first_fit

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def on_gpu(run, bt, bp, ct, nodes, cur_seg, cur_c, prev, floor_seg, floor_c, state):
    import torch
    import paper_2408_08586_amd as rk
    J = run.wl.n_jobs
    dev = run.device
    i32 = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    u8 = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(dev)
    p_off = p_ent = None
    n_prev = 0
    if prev is not None:
        p_off = torch.from_numpy(np.ascontiguousarray(prev[0], dtype=np.uint32).view(np.int32).copy()).to(dev)
        ent = np.ascontiguousarray(prev[1], dtype=rk.PLACE_DTYPE)
        n_prev = int(ent.size)
        p_ent = torch.from_numpy((ent if ent.size else np.zeros(1, rk.PLACE_DTYPE)).view(np.uint8).copy()).to(dev)
    n_nodes, gpn, cpn, mem = nodes
    cap = n_nodes * gpn
    assign, total = rk.new_assign(J, dev), run.f32(1)
    off = torch.full((J + 1,), -1, dtype=torch.int32, device=dev)
    ent = rk.new_place_entries(cap, dev)
    stats = torch.full((5,), -1, dtype=torch.int32, device=dev)
    rk.rk_reschedule_nodes(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, rk.rk_nodes(n_nodes, gpn, cpn, mem),
                           run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct), i32(cur_seg), run.dev_u32(cur_c), assign, off,
                           ent, cap, total, prev_off=p_off, prev_entries=p_ent, n_prev_entries=n_prev, state=u8(state),
                           floor_seg=i32(floor_seg), floor_c=None if floor_c is None else run.dev_u32(floor_c), stats=stats)
    rk.rk_sync(run.ctx)
    off = rk.u32(off)
    stats = stats.cpu().numpy()
    return rk.assign_to_numpy(assign), off, rk.place_entries_to_numpy(ent, int(off[J])), float(total[0].item()), stats


def same(got, want):
    """want = the oracle's (records, offsets, entries, total, steps), or None for a state that is no placement."""
    g_a, g_off, g_ent, g_total, stats = got
    if want is None:
        assert stats[4] == 1 and not g_a["g"].any() and not g_off.any() and g_total == 0
        return
    w_a, w_off, w_ent, w_total, w_moves = want
    assert stats[4] == 0
    assert np.array_equal(g_a, w_a), np.flatnonzero(g_a != w_a)[:5]
    assert np.array_equal(g_off, w_off)
    assert np.array_equal(g_ent, w_ent), np.flatnonzero(g_ent != w_ent)[:5]
    assert g_total == pytest.approx(w_total, rel=1e-6, abs=1e-12)
    assert stats[0] == w_moves


def node_round(rng, orc, J=None, g_max=None, roomy=None, gpn=None, n_nodes=None):
    """A drawn round (as for the loop over totals) with CPU levels per GPU, nodes that hold the cluster's GPUs, and the
    jobs that hold something laid out by first fit (a job that finds no room holds nothing)."""
    wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = random_round(rng, orc, J, g_max)
    grid = workloads.Grid(wl.grid.cpu_levels, 1, wl.grid.mem_levels_gb, wl.grid.mem_mode)
    ct, _, _ = orc.curves(tb, grid, bt, bp)
    wl = workloads.Workload("drawn", wl.coef, wl.ints, wl.bounds, grid, wl.env, wl.cluster)
    J = wl.n_jobs
    gpn = int(rng.choice([1, 2, 4, 8])) if gpn is None else gpn
    n_nodes = max(1, -(-wl.cluster.G // gpn)) if n_nodes is None else n_nodes
    top = int(grid.cpu_levels[-1])
    roomy = rng.uniform() < 0.5 if roomy is None else roomy
    cpn = gpn * top if roomy else int(rng.integers(gpn, gpn * top + 1))
    mem = float(rng.choice([8.0, 64.0, 1e6]))
    free_g, free_c = [gpn] * n_nodes, [cpn] * n_nodes
    off, ent = [0], []
    cur_seg[(state != 0) & (state != 2)] = -1                # (they hold nothing, also when the states are not passed)
    for j in range(J):
        if cur_seg[j] >= 0:
            parts = first_fit(free_g, free_c, int(cur_seg[j]) + 1, int(grid.cpu_levels[cur_c[j]]))
            if parts is None:
                cur_seg[j] = -1
            else:
                ent += [(n, k, int(grid.cpu_levels[cur_c[j]]) * k, 0.0) for n, k in sorted(parts.items())]
        off.append(len(ent))
    prev = (np.array(off, np.uint32), np.array(ent, orc.PLACE_DTYPE) if ent else np.zeros(0, orc.PLACE_DTYPE))
    return wl, tb, bt, bp, ct, (n_nodes, gpn, cpn, mem), cur_seg, cur_c, prev, floor_seg, floor_c, state


def run_both(gpu, orc, case, use_floor=True, use_state=True):
    wl, tb, bt, bp, ct, nodes, cur_seg, cur_c, prev, floor_seg, floor_c, state = case
    fs, fc, st = (floor_seg, floor_c) if use_floor else (None, None), None, state if use_state else None
    fs, fc = fs
    want = orc.reschedule_nodes(wl.coef[:, 16], tb, wl.grid, *nodes, bt, bp, ct, cur_seg, cur_c, prev, fs, fc, state=st)
    run = gpu(wl)
    run.enumerate()
    assert np.array_equal(run.table_numpy()["seg_g"], tb.seg_g)
    got = on_gpu(run, bt, bp, ct, nodes, cur_seg, cur_c, prev, fs, fc, st)
    run.close()
    same(got, want)
    return want


def test_random_rounds_on_drawn_values(gpu, orc):
    n_moves = n_spread = n_dropped = 0
    for seed in range(400):
        rng = np.random.default_rng(81000 + seed)
        case = node_round(rng, orc)
        print("seed", 81000 + seed, "jobs", case[0].n_jobs, "nodes", case[5], flush=True)
        want = run_both(gpu, orc, case, use_floor=seed % 4 != 0, use_state=seed % 3 != 0)
        assert want is not None
        a, off, ent, _, moves = want
        n_moves += moves
        n_spread += int(np.any(np.diff(off.astype(np.int64)) > 1))
        n_dropped += int(np.any((a["g"] == 0) & (case[6] >= 0)))
    print(f"400 rounds, {n_moves} steps committed, {n_spread} rounds with a job on several nodes, {n_dropped} with a job that left")
    assert n_moves > 1500 and n_spread > 100


def test_larger_drawn_rounds(gpu, orc):
    n_moves = 0
    for seed, J in enumerate([300, 1000, 1024, 1025, 2049, 3000] * 2):
        rng = np.random.default_rng(82000 + seed)
        case = node_round(rng, orc, J, int(rng.integers(2, 23)))
        print("seed", 82000 + seed, "jobs", J, "nodes", case[5], flush=True)
        want = run_both(gpu, orc, case)
        n_moves += want[4]
    print(f"12 rounds, {n_moves} steps committed")
    assert n_moves > 1000


def test_jobs_with_more_amounts_than_a_wavefront_has_lanes(gpu, orc):
    """174 GPU counts per job (see the same test of the loop over totals), on nodes of 8 GPUs."""
    from test_gpu_reschedule import many_amounts_round
    n_moves = n_spread = 0
    for seed in range(25):
        rng = np.random.default_rng(83000 + seed)
        wl, tb, bt, bp, ct, cur_seg, cur_c, floor_seg, floor_c, state = many_amounts_round(rng, orc, int(rng.integers(3, 30)))
        grid = workloads.Grid(wl.grid.cpu_levels, 1, wl.grid.mem_levels_gb, wl.grid.mem_mode)
        ct, _, _ = orc.curves(tb, grid, bt, bp)
        wl = workloads.Workload("many amounts", wl.coef, wl.ints, wl.bounds, grid, wl.env, wl.cluster)
        seg_g = np.asarray(tb.seg_g[:174], dtype=np.int64)
        gpn, top = 8, int(grid.cpu_levels[-1])
        n_nodes = -(-wl.cluster.G // gpn)
        cpn = gpn * top if seed % 2 else int(rng.integers(gpn, gpn * top + 1))
        mem = float(rng.choice([8.0, 64.0, 1e6]))
        free_g, free_c = [gpn] * n_nodes, [cpn] * n_nodes
        off, ent = [0], []
        cur_seg[(state != 0) & (state != 2)] = -1
        for j in range(wl.n_jobs):
            if cur_seg[j] >= 0:
                parts = first_fit(free_g, free_c, int(seg_g[cur_seg[j]]), int(grid.cpu_levels[cur_c[j]]))
                if parts is None:
                    cur_seg[j] = -1
                else:
                    ent += [(n, k, int(grid.cpu_levels[cur_c[j]]) * k, 0.0) for n, k in sorted(parts.items())]
            off.append(len(ent))
        prev = (np.array(off, np.uint32), np.array(ent, orc.PLACE_DTYPE) if ent else np.zeros(0, orc.PLACE_DTYPE))
        print("seed", 83000 + seed, "jobs", wl.n_jobs, "nodes", n_nodes, flush=True)
        want = run_both(gpu, orc, (wl, tb, bt, bp, ct, (n_nodes, gpn, cpn, mem), cur_seg, cur_c, prev, floor_seg, floor_c, state))
        assert want is not None
        n_moves += want[4]
        n_spread += int(np.any(np.diff(want[1].astype(np.int64)) > 1))
    print(f"25 rounds, {n_moves} steps committed, {n_spread} rounds with a job on several nodes")
    assert n_moves > 100 and n_spread > 15


def test_shapes_at_the_limits(gpu, orc):
    """The most nodes the library takes (four per thread of the kernel), nodes of more GPUs than a wavefront has lanes,
    the most jobs a round may have, and the smallest cluster there is."""
    import time
    for seed, (J, g_max, gpn, n_nodes) in enumerate([(2000, 4, 1, 4096), (500, 22, 128, 8), (12288, 3, 8, 512), (1, 2, 1, 1),
                                                      (700, 16, 3, 1365)]):
        rng = np.random.default_rng(84000 + seed)
        case = node_round(rng, orc, J, g_max, gpn=gpn, n_nodes=n_nodes)
        t0 = time.time()
        want = run_both(gpu, orc, case)
        print("seed", 84000 + seed, "jobs", J, "nodes", case[5], "steps", want[4], f"{time.time() - t0:.1f} s", flush=True)
        assert want is not None


def test_states_that_are_no_placement(gpu, orc):
    n_bad = 0
    for seed in range(40):
        rng = np.random.default_rng(83000 + seed)
        case = list(node_round(rng, orc, roomy=True))
        off, ent = case[8][0].copy(), case[8][1].copy()
        kind = seed % 5
        if len(ent) == 0:
            continue
        i = int(rng.integers(0, len(ent)))
        if kind == 0: ent["g"][i] += 1                        # parts that do not add up (and CPUs that do not match)
        elif kind == 1: ent["node"][i] = case[5][0] + int(rng.integers(0, 3))     # a node the cluster does not have
        elif kind == 2: ent["c"][i] += 1                      # CPUs that are not level * GPUs
        elif kind == 3: off[1:] = off[1:][::-1]               # offsets that do not ascend (unless all jobs are alike)
        elif kind == 4: case[5] = (case[5][0], case[5][1], max(1, case[5][2] // 8), case[5][3])   # nodes with too few CPUs
        case[8] = (off, ent)
        print("seed", 83000 + seed, "kind", kind, flush=True)
        want = run_both(gpu, orc, tuple(case))
        n_bad += want is None
    assert n_bad > 20


@pytest.mark.parametrize("name", ["what_if", "stress"])
def test_generated_rounds_from_a_running_state(gpu, orc, name):
    """The state a from-scratch round leaves, laid out on the nodes by first fit; then a tenth of the jobs leave and
    their slots are new arrivals, some jobs are guaranteed: the loop over the nodes on the library's own curves, given
    to both sides.  What comes out is a placement that rk_place_plans keeps part by part."""
    import time
    import paper_2408_08586_amd as rk
    from test_gpu_placed import place_on_gpu
    wl = {"what_if": lambda: workloads.what_if(7), "stress": workloads.stress}[name]()
    assert wl.grid.cpu_mode == 1
    J = wl.n_jobs
    rng = np.random.default_rng(J + 1)
    run = gpu(wl)
    run.enumerate()
    bt, bp, ct, _, _, n = run.fused()
    bt, bp, ct = run.host(bt, n).copy(), run.host(bp, n).view(np.uint32).copy(), run.host(ct, n).copy()
    tn = run.table_numpy()
    tb = orc.Table(tn["triple_off"], tn["triples"], tn["seg_off"], tn["seg_g"], tn["seg_first"])
    a0, _, _ = orc.greedy(wl.coef[:, 16], tb, wl.grid, wl.cluster, bt, bp, ct)
    gpn = wl.env.gpus_per_node
    n_nodes = wl.cluster.G // gpn
    nodes = (n_nodes, gpn, int(wl.grid.cpu_levels[-1]) * gpn, wl.cluster.host_mem_gb / n_nodes)
    off0, ent0, status0 = orc.place(a0, *nodes)
    cur_seg, cur_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    levels = np.asarray(wl.grid.cpu_levels)
    for j in np.flatnonzero(status0 == 1).tolist():
        seg_g = tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]]
        cur_seg[j] = int(np.flatnonzero(seg_g == a0["g"][j])[0])
        cur_c[j] = int(np.flatnonzero(levels == a0["c"][j] // a0["g"][j])[0])
    gone = rng.uniform(size=J) < 0.1
    cur_seg[gone] = -1                                                       # left; the slot is a new arrival
    floor_seg, floor_c = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    ns = np.diff(tb.seg_off)
    guaranteed = (rng.uniform(size=J) < 0.05) & (ns > 0)
    floor_seg[guaranteed] = np.minimum(rng.integers(0, 3, guaranteed.sum()), ns[guaranteed] - 1)
    floor_seg[(cur_seg >= 0) & (floor_seg > cur_seg)] = -1                  # running jobs sit at or above their floor
    state = (rng.uniform(size=J) < 0.02).astype(np.uint8)
    cur_seg[state != 0] = -1
    prev = (off0, ent0)
    t0 = time.time()
    want = orc.reschedule_nodes(wl.coef[:, 16], tb, wl.grid, *nodes, bt, bp, ct, cur_seg, cur_c, prev, floor_seg, floor_c,
                                state=state)
    t1 = time.time()
    got = on_gpu(run, bt, bp, ct, nodes, cur_seg, cur_c, prev, floor_seg, floor_c, state)
    same(got, want)
    a, off, ent, total, stats = got
    print(f"{name}: {int((status0 == 1).sum())} jobs ran on {n_nodes} nodes, {int(gone.sum())} slots changed hands, "
          f"{stats[0]} steps committed ({stats[1]} jobs served in full, {stats[2]} shrinks, {stats[3]} steps taken back), "
          f"{int((a['g'] > 0).sum())} jobs run now, {int((np.diff(off.astype(np.int64)) > 1).sum())} on several nodes; "
          f"oracle {t1 - t0:.1f} s", flush=True)
    assert stats[0] > 0
    used = np.zeros(n_nodes, np.int64)
    np.add.at(used, ent["node"], ent["g"])
    assert used.max() <= gpn
    # GetBestPlan(j, placement).  The oracle's placement that feeds the plan, given this placement as the earlier one,
    # keeps every part and chooses the plans for the actual splits; so does rk_place_plans, and rk_best_plan_placed
    # chooses them without placing anything
    from types import SimpleNamespace
    from test_gpu_placed import compare
    w_placed = orc.place_plans(wl.coef, wl.ints, wl.bounds, tb, wl.grid, wl.env, bt, a, *nodes, min_seg=floor_seg, prev=(off, ent))
    assert np.array_equal(w_placed[1], off) and np.array_equal(w_placed[2], ent)
    got_pp = place_on_gpu(run, bt, a, floor_seg, *nodes, prev=(off, ent))
    n_band = compare(orc, wl, tb, w_placed, got_pp)
    assert got_pp[5].in_order == 1
    import torch
    dev = run.device
    d_a = torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).copy()).to(dev)
    d_off = torch.from_numpy(off.view(np.int32).copy()).to(dev)
    d_ent = torch.from_numpy((ent if ent.size else np.zeros(1, rk.PLACE_DTYPE)).view(np.uint8).copy()).to(dev)
    placed, total2 = rk.new_assign(J, dev), run.f32(1)
    rk.rk_best_plan_placed(run.ctx, run.jobs, run.table.c, run.grid, run.env, d_a, d_off, d_ent, placed, total2)
    rk.rk_sync(run.ctx)
    on = (a["g"] > 0)
    res = SimpleNamespace(n_entries=len(ent), n_placed=int(on.sum()), n_failed=0)
    compare(orc, wl, tb, w_placed, (rk.assign_to_numpy(placed), off, ent, on.astype(np.uint32), float(total2[0].item()), res))
    # the whole round in one call, from the job descriptors: the same records, placement and plans
    a1, p1, total1 = rk.new_assign(J, dev), rk.new_assign(J, dev), run.f32(1)
    off1 = torch.full((J + 1,), -1, dtype=torch.int32, device=dev)
    ent1 = rk.new_place_entries(n_nodes * gpn, dev)
    st1 = torch.full((5,), -1, dtype=torch.int32, device=dev)
    i32 = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    rk.rk_schedule_round_nodes(run.ctx, run.jobs, rk.make_bounds(wl.bounds), run.grid, run.env, rk.rk_nodes(*nodes), i32(cur_seg),
                               run.dev_u32(cur_c), a1, p1, off1, ent1, n_nodes * gpn, total1,
                               prev_off=torch.from_numpy(off0.view(np.int32).copy()).to(dev),
                               prev_entries=torch.from_numpy((ent0 if ent0.size else np.zeros(1, rk.PLACE_DTYPE)).view(np.uint8).copy()).to(dev),
                               n_prev_entries=len(ent0), state=torch.from_numpy(state).to(dev), floor_seg=i32(floor_seg),
                               floor_c=run.dev_u32(floor_c), stats=st1)
    rk.rk_sync(run.ctx)
    assert np.array_equal(rk.assign_to_numpy(a1), a) and np.array_equal(rk.u32(off1), off)
    assert np.array_equal(rk.place_entries_to_numpy(ent1, int(off[J])), ent) and st1.cpu().numpy().tolist() == stats.tolist()
    assert np.array_equal(rk.assign_to_numpy(p1), rk.assign_to_numpy(placed)) and float(total1[0].item()) == float(total2[0].item())
    changed = int(((rk.assign_to_numpy(placed)["plan"] != a["plan"]) & on).sum())
    print(f"{name}: the actual splits change the plan of {changed} of {int(on.sum())} jobs ({n_band} inside the tie band)", flush=True)
    run.close()


def test_argument_errors(gpu, orc):
    import paper_2408_08586_amd as rk
    rng = np.random.default_rng(5)
    wl, tb, bt, bp, ct, nodes, cur_seg, cur_c, prev, floor_seg, floor_c, state = node_round(rng, orc)
    run = gpu(wl)
    run.enumerate()
    J = wl.n_jobs
    dev = run.device
    assign, total = rk.new_assign(J, dev), run.f32(1)
    off = run.i32(J + 1)
    n_nodes, gpn, cpn, mem = nodes
    ent = rk.new_place_entries(n_nodes * gpn, dev)
    cur = run.torch.full((J,), -1, dtype=run.torch.int32, device=dev)
    args = (run.dev_f32(bt), run.dev_u32(bp), run.dev_f32(ct), cur, run.i32(J).zero_(), assign, off, ent)

    def call(grid=run.grid, nd=rk.rk_nodes(n_nodes, gpn, cpn, mem), cap=n_nodes * gpn, **kw):
        rk.rk_reschedule_nodes(run.ctx, run.jobs.ref_thr, run.table.c, grid, nd, *args, cap, total, **kw)

    with pytest.raises(rk.RkError) as e:
        call(grid=rk.make_grid(workloads.Grid(wl.grid.cpu_levels, 0, wl.grid.mem_levels_gb, wl.grid.mem_mode)))
    assert e.value.code == rk.RK_ERR_UNSUPPORTED              # CPU levels of the job, not per GPU
    with pytest.raises(rk.RkError) as e:
        call(cap=n_nodes * gpn - 1)
    assert e.value.code == rk.RK_ERR_CAPACITY
    with pytest.raises(rk.RkError) as e:
        call(nd=rk.rk_nodes(0, gpn, cpn, mem))
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    with pytest.raises(rk.RkError) as e:
        call(prev_off=off)                                   # offsets without entries
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    # nobody holds anything and there is no earlier placement: every job is a newcomer
    call()
    rk.rk_sync(run.ctx)
    a = rk.assign_to_numpy(assign)
    assert 0 <= a["g"].sum() <= n_nodes * gpn
    want = orc.reschedule_nodes(wl.coef[:, 16], tb, wl.grid, *nodes, bt, bp, ct, np.full(J, -1), np.zeros(J), None)
    assert np.array_equal(a, want[0])
    run.close()


def test_tables_without_jobs_or_without_plans(gpu, orc):
    """Zero jobs, and jobs none of which has a plan (no segment: the value arrays are empty and may be null), through the
    entry points of the loops: nothing is scheduled, nothing is read that is not there."""
    import torch
    import paper_2408_08586_amd as rk
    base = workloads.tiny()
    grid = workloads.Grid(np.array([1, 2], np.uint32), 1, np.array([0.0, 8.0], np.float32), 0)
    for name, coef, ints in (("empty", base.coef[:0], base.ints[:0]),
                             ("noplans", base.coef[:3], np.array([[5, 7, 2], [0, 8, 1], [8, 0, 1]], np.uint32))):
        wl = workloads.Workload(name, coef, ints, base.bounds, grid, base.env, base.cluster)
        J = wl.n_jobs
        run = gpu(wl)
        t = run.enumerate()
        assert t.n_segs == 0
        dev = run.device
        nodes = rk.rk_nodes(2, 4, 16, 64.0)
        seg = torch.full((max(J, 1),), -1, dtype=torch.int32, device=dev)
        lvl = torch.zeros(max(J, 1), dtype=torch.int32, device=dev)
        assign, placed, total = rk.new_assign(max(J, 1), dev), rk.new_assign(max(J, 1), dev), run.f32(1)
        off = torch.full((J + 1,), -1, dtype=torch.int32, device=dev)
        ent = rk.new_place_entries(8, dev)
        stats = torch.full((5,), -1, dtype=torch.int32, device=dev)
        rk.rk_reschedule_nodes(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, nodes, None, None, None, seg, lvl, assign, off,
                               ent, 8, total, stats=stats)
        rk.rk_sync(run.ctx)
        assert not rk.u32(off).any() and float(total[0].item()) == 0.0 and stats.cpu().numpy().tolist() == [0, 0, 0, 0, 0]
        assert not rk.assign_to_numpy(assign)["g"][:J].any()
        rk.rk_best_plan_placed(run.ctx, run.jobs, run.table.c, run.grid, run.env, assign, off, ent, placed, total)
        rk.rk_schedule_round_nodes(run.ctx, run.jobs, rk.make_bounds(wl.bounds), run.grid, run.env, nodes, seg, lvl, assign, placed,
                                   off, ent, 8, total, stats=stats)
        rk.rk_sync(run.ctx)
        assert not rk.u32(off).any() and float(total[0].item()) == 0.0 and not rk.assign_to_numpy(placed)["g"][:J].any()
        totals = run.f32(3)
        many = rk.new_assign(3 * max(J, 1), dev)
        rk.rk_reschedule_rounds(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, [rk.make_cluster(base.cluster)] * 3, None, None,
                                None, seg, lvl, many, totals)
        rk.rk_sync(run.ctx)
        assert not totals.cpu().numpy()[:3].any() and not rk.assign_to_numpy(many)["g"][:3 * J].any()
        z = np.zeros(max(J, 1), np.uint32)
        fs, fc = torch.zeros(max(J, 1), dtype=torch.int32, device=dev), torch.zeros(max(J, 1), dtype=torch.int32, device=dev)
        so = torch.zeros(max(J, 1), dtype=torch.uint8, device=dev)
        rk.rk_privileged(run.ctx, run.table.c, run.grid, rk.Sla(z + 1, z, [4], [4], device=dev), seg, lvl, seg, lvl, fs, fc, so)
        rk.rk_sync(run.ctx)
        if J:                                                # guaranteed jobs without a minimum demand wait
            assert so.cpu().numpy()[:J].tolist() == [1] * J and (fs.cpu().numpy()[:J] == -1).all()
        run.close()
