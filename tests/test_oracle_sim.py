"""Pins for the oracle's rounds with frozen jobs and its discrete-time
simulation (paper Sec. 5.2 "Incorporating reconfiguration penalty": reconfigure
only if (T - N*delta)/T > 0.97; Sec. 7.4: discrete-time simulator)."""
import numpy as np
import pytest

import workloads
from test_oracle_policy import one_job_table  # noqa: F401  (same tiny tables)


def tiny_round(orc, curves, state, cur_seg, cur_c, G, C=10 ** 6, host=1e9, n_cpu=2):
    """curves[j][s] = best throughput of job j at 1, 2, 4, 8 GPUs (every CPU level alike)."""
    J = len(curves)
    ints = np.tile(np.array([[8, 8, 1]], np.uint32), (J, 1))
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=8))
    grid = workloads.Grid(np.arange(1, n_cpu + 1, dtype=np.uint32), 0, np.array([1.0], np.float32), 0)
    bt = np.zeros((J, n_cpu, 1, 4), np.float32)
    for j, cv in enumerate(curves):
        bt[j, :, 0, :] = np.asarray(cv, np.float32)[None, :]
    bt = bt.reshape(-1)
    bp = np.arange(bt.size, dtype=np.uint32)
    ct, _, _ = orc.curves(tb, grid, bt, bp)
    ref = np.ones(J, np.float32)
    return orc.frozen_round(ref, tb, grid, workloads.Cluster(G, C, host), bt, bp, ct, state, cur_seg, cur_c), (tb, grid, bt, bp, ct, ref)


def test_frozen_round_hand_cases(orc):
    steep, flat = [4.0, 8.0, 12.0, 17.0], [1.0, 1.1, 1.2, 1.3]
    # all jobs normal: the greedy (the steep job takes everything)
    (a, total, _), _ = tiny_round(orc, [flat, steep], [0, 0], [-1, -1], [0, 0], G=8)
    assert a["g"].tolist() == [0, 8]
    # the flat job is frozen at 4 GPUs, CPU level 1: it keeps exactly that, the steep job gets the rest
    (a, total, _), _ = tiny_round(orc, [flat, steep], [2, 0], [2, -1], [1, 0], G=8)
    assert a["g"].tolist() == [4, 4] and a["c"][0] == 2
    assert total == pytest.approx(1.2 + 12.0)
    # a frozen job does not grow even when resources are plentiful, nor gain CPUs
    (a, _, _), _ = tiny_round(orc, [steep, flat], [2, 0], [0, -1], [0, 0], G=64)
    assert a["g"].tolist() == [1, 8] and a["c"][0] == 1
    # a job that takes no part gets nothing, whatever its slope
    (a, _, _), _ = tiny_round(orc, [steep, flat], [1, 0], [-1, -1], [0, 0], G=8)
    assert a["g"].tolist() == [0, 8]
    # frozen jobs holding more than the cluster has: nothing is left for the others
    (a, _, _), _ = tiny_round(orc, [flat, flat, steep], [2, 2, 0], [3, 2, -1], [0, 0, 0], G=10)
    assert a["g"].tolist() == [8, 4, 0]
    # CPUs of frozen jobs are charged: 2 CPUs in all, the frozen job holds both
    (a, _, _), _ = tiny_round(orc, [flat, steep], [2, 0], [0, -1], [1, 0], G=8, C=2)
    assert a["g"].tolist() == [1, 0]


def test_frozen_round_without_states_is_the_plain_greedy(orc):
    wl = workloads.paper_scale()
    r = orc.schedule_round(wl, n_threads=4)
    J = wl.n_jobs
    a, total, gap = orc.frozen_round(wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"],
                                     r["curve_thr"], np.zeros(J, np.uint8), np.full(J, -1, np.int32), np.zeros(J, np.uint32))
    assert np.array_equal(a, r["assign"]) and total == r["total"] and gap == r["min_gap"]


def lone_job(orc, work, arrival, delta=50.0, dt=60.0, n_ticks=40, policy="greedy"):
    curve = [2.0, 3.5, 6.0, 8.0]
    _, (tb, grid, bt, bp, ct, ref) = tiny_round(orc, [curve], [0], [-1], [0], G=4)
    return orc.simulator.simulate(ref, tb, grid, workloads.Cluster(4, 100, 1e9), bt, bp, ct, [arrival], [work], [delta], dt,
                                  n_ticks, policy=policy)


@pytest.mark.parametrize("policy", ["greedy", "loop"])
def test_lone_job_finishes_at_the_closed_form_time(orc, policy):
    import functools
    lone = functools.partial(lone_job, policy=policy)
    # arrives at 130 s: first seen by the tick at 180 s; 4 GPUs give 6 samples/s (the loop gets there in three steps
    # of one round: 1, 2, 4 GPUs)
    out = lone(orc, work=6.0 * 1000.0, arrival=130.0)
    assert out["finish"][0] == pytest.approx(180.0 + 1000.0, rel=1e-15)
    assert out["n_reconf"][0] == 0 and out["progress"][0] == 6000.0
    assert out["held"][0] == 60.0 * 17                       # ticks at 180 ... 1140 s
    assert out["gpus_in_use"].tolist()[:3] == [0, 0, 0] and set(out["gpus_in_use"][3:20]) == {4} and out["gpus_in_use"][20] == 0
    # arrival exactly on a tick counts for that tick; work that ends exactly with a tick
    out = lone(orc, work=6.0 * 120.0, arrival=120.0)
    assert out["finish"][0] == 240.0
    # never finishing inside the horizon
    out = lone(orc, work=1e9, arrival=0.0)
    assert out["finish"][0] == -1.0 and out["progress"][0] == pytest.approx(6.0 * 60.0 * 40)


def two_jobs(orc, gate, delta_a, n_ticks=60, trace=True):
    """Job A alone takes all 8 GPUs; job B arrives at 300 s and is worth half of them."""
    a_curve, b_curve = [1.0, 2.0, 4.0, 6.0], [1.5, 3.0, 5.0, 5.5]
    _, (tb, grid, bt, bp, ct, ref) = tiny_round(orc, [a_curve, b_curve], [0, 0], [-1, -1], [0, 0], G=8)
    out = orc.simulator.simulate(ref, tb, grid, workloads.Cluster(8, 100, 1e9), bt, bp, ct, [0.0, 300.0], [1e9, 1e9],
                                 [delta_a, 10.0], 60.0, n_ticks, gate=gate, trace=trace)
    return out


def test_gate_freezes_until_the_reconfiguration_is_cheap_enough(orc):
    # without B, A holds 8 GPUs; with B the greedy gives both 4 (A: 4, B: 5 beats A: 6, B: 0 ...)
    out = two_jobs(orc, gate=0.97, delta_a=30.0)
    g_a = [int(h["g"][0]) for h in out["history"]]
    g_b = [int(h["g"][1]) for h in out["history"]]
    # A may move once T - delta > 0.97 T, i.e. T > 1000 s: T = 1020 s after 17 ticks, seen by the tick with k = 17
    first_change = next(k for k, g in enumerate(g_a) if g != 8)
    assert first_change == 17
    assert g_a[:17] == [8] * 17 and g_a[17] == 4
    assert g_b[:5] == [0] * 5 and g_b[5:17] == [0] * 12 and g_b[17] == 4      # B waits while A is frozen on all GPUs
    assert out["n_reconf"][0] == 1 and out["n_reconf"][1] == 0
    assert out["frozen"][:17].tolist() == [0] + [1] * 16                      # A is not running at the very first tick
    # the reconfiguration costs A 30 s of the tick in which it happens
    assert out["progress"][0] == pytest.approx(6.0 * 60 * 17 + 4.0 * 30 + 4.0 * 60 * (60 - 18))
    # a gate of 1 can never be passed, a gate of minus infinity always
    assert two_jobs(orc, gate=1.0, delta_a=30.0)["n_reconf"].tolist() == [0, 0]
    free = two_jobs(orc, gate=-np.inf, delta_a=30.0)
    assert [int(h["g"][0]) for h in free["history"]][:7] == [8] * 5 + [4, 4] and free["frozen"].sum() == 0
    # a checkpoint-resume cost longer than a tick is paid over several ticks
    slow = two_jobs(orc, gate=-np.inf, delta_a=150.0)
    assert slow["progress"][0] == pytest.approx(6.0 * 60 * 5 + 4.0 * 30 + 4.0 * 60 * (60 - 8))


def test_simulation_conserves_what_it_should(orc):
    wl = workloads.paper_scale()
    r = orc.schedule_round(wl, n_threads=4)
    tr = workloads.trace(wl.n_jobs, horizon_s=2 * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * 4
    args = (wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"], r["curve_thr"], tr.arrival, work,
            tr.delta, 60.0, 300)
    out = orc.simulator.simulate(*args, trace=True)
    fin = out["finish"] >= 0
    assert 10 < fin.sum() < wl.n_jobs
    assert np.all(out["gpus_in_use"] <= wl.cluster.G)
    assert np.all(out["finish"][fin] > tr.arrival[fin]) and np.all(out["progress"][fin] == work[fin])
    assert np.all(out["progress"][~fin] < work[~fin])
    assert out["n_reconf"].sum() > 0 and out["frozen"].sum() > 0
    # no job runs before it arrives or after it has finished
    for k, h in enumerate(out["history"]):
        t = 60.0 * k
        assert np.all(h["g"][tr.arrival > t] == 0)
        assert np.all(h["g"][fin & (out["finish"] <= t)] == 0)
    # progress never exceeds the best throughput times the time held
    best = np.array([r["best_thr"][20 * 0:].max()])       # a loose global bound
    assert np.all(out["progress"] <= best * out["held"] + 1e-6)
    # a stricter gate can only reduce reconfigurations to zero; with no gate none is frozen
    assert orc.simulator.simulate(*args, gate=1.0)["n_reconf"].sum() == 0
    assert orc.simulator.simulate(*args, gate=-np.inf)["frozen"].sum() == 0


def test_the_loop_as_the_policy_of_the_simulation(orc):
    """Algorithm 1's loop every tick instead of the from-scratch greedy: running jobs keep what they hold unless a job
    with a higher slope takes it, and a job the gate freezes is not asked at all."""
    a_curve, b_curve = [1.0, 1.8, 2.4, 2.8], [1.5, 3.0, 5.0, 5.5]
    _, (tb, grid, bt, bp, ct, ref) = tiny_round(orc, [a_curve, b_curve], [0, 0], [-1, -1], [0, 0], G=8)

    def run(gate, delta_a=30.0, policy="loop"):
        return orc.simulator.simulate(ref, tb, grid, workloads.Cluster(8, 100, 1e9), bt, bp, ct, [0.0, 300.0], [1e9, 1e9],
                                      [delta_a, 10.0], 60.0, 60, gate=gate, trace=True, policy=policy)
    # A alone climbs to 8 GPUs; B arrives at 300 s.  Its first GPU is worth 1.5 and makes A give four (0.4 lost), the
    # next three are free by then; the step to 8 (0.125 per GPU) is not worth A's 0.3 per GPU: 4 + 4
    out = run(-np.inf)
    g_a, g_b = [int(h["g"][0]) for h in out["history"]], [int(h["g"][1]) for h in out["history"]]
    assert g_a[:5] == [8] * 5 and g_a[5:] == [4] * 55 and g_b[:5] == [0] * 5 and g_b[5:] == [4] * 55
    assert out["n_reconf"].tolist() == [1, 0]
    # with the gate A is frozen until T > 1000 s (the tick with k = 17), and a frozen job gives nothing
    out = run(0.97)
    g_a, g_b = [int(h["g"][0]) for h in out["history"]], [int(h["g"][1]) for h in out["history"]]
    assert g_a[:17] == [8] * 17 and g_a[17:] == [4] * 43 and g_b[:17] == [0] * 17 and g_b[17:] == [4] * 43
    assert out["frozen"][:17].tolist() == [0] + [1] * 16
    assert out["progress"][0] == pytest.approx(2.8 * 60 * 17 + 2.4 * 30 + 2.4 * 60 * (60 - 18))
    # where the two policies part: B's first GPU would cost A more than it brings (A gives four at once and loses 2.0,
    # B gains 1.5), so the loop leaves A alone for good, while a round from scratch shares the cluster
    _, (tb2, grid2, bt2, bp2, ct2, ref2) = tiny_round(orc, [[1.0, 2.0, 4.0, 6.0], b_curve], [0, 0], [-1, -1], [0, 0], G=8)
    args = (ref2, tb2, grid2, workloads.Cluster(8, 100, 1e9), bt2, bp2, ct2, [0.0, 300.0], [1e9, 1e9], [30.0, 10.0], 60.0, 20)
    loop = orc.simulator.simulate(*args, gate=-np.inf, trace=True, policy="loop")
    scratch = orc.simulator.simulate(*args, gate=-np.inf, trace=True)
    assert [int(h["g"][1]) for h in loop["history"]] == [0] * 20
    assert [int(h["g"][1]) for h in scratch["history"]][5:] == [4] * 15


def test_simulation_with_the_loop_conserves_what_it_should(orc):
    wl = workloads.paper_scale()
    r = orc.schedule_round(wl, n_threads=4)
    tr = workloads.trace(wl.n_jobs, horizon_s=2 * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * 4
    args = (wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"], r["curve_thr"], tr.arrival, work,
            tr.delta, 60.0, 300)
    out = orc.simulator.simulate(*args, trace=True, policy="loop")
    fin = out["finish"] >= 0
    assert 10 < fin.sum() < wl.n_jobs
    assert np.all(out["gpus_in_use"] <= wl.cluster.G)
    assert np.all(out["finish"][fin] > tr.arrival[fin]) and np.all(out["progress"][fin] == work[fin])
    assert np.all(out["progress"][~fin] < work[~fin])
    for k, h in enumerate(out["history"]):
        t = 60.0 * k
        assert np.all(h["g"][tr.arrival > t] == 0)
        assert np.all(h["g"][fin & (out["finish"] <= t)] == 0)
    assert orc.simulator.simulate(*args, gate=1.0, policy="loop")["n_reconf"].sum() == 0
    assert orc.simulator.simulate(*args, gate=-np.inf, policy="loop")["frozen"].sum() == 0
    # running jobs keep what they hold: fewer reconfigurations than rounds from scratch make on the same trace
    scratch = orc.simulator.simulate(*args, gate=-np.inf)
    loop = orc.simulator.simulate(*args, gate=-np.inf, policy="loop")
    print("reconfigurations without a gate: from scratch", int(scratch["n_reconf"].sum()), "loop", int(loop["n_reconf"].sum()))
    assert loop["n_reconf"].sum() < scratch["n_reconf"].sum()


def test_simulation_over_nodes(orc):
    """The loop with ScheduleJob searching node by node as the round of every tick, from the placement the last tick
    left: one node that holds the whole cluster gives the trajectories of the loop over totals; on real nodes no node
    ever holds more than it has and every job's parts add up to what it holds."""
    wl = workloads.large()
    r = orc.schedule_round(wl, n_threads=8)
    tr = workloads.trace(wl.n_jobs, horizon_s=2 * 3600.0)
    work = workloads.job_lengths_s(tr.u_duration) * wl.coef[:, 16] * 2.0
    args = (wl.coef[:, 16], r["table"], wl.grid, wl.cluster, r["best_thr"], r["best_plan"], r["curve_thr"], tr.arrival, work,
            tr.delta, 120.0, 40)
    loop = orc.simulator.simulate(*args, policy="loop")
    one = orc.simulator.simulate(*args, policy="nodes", nodes=(1, wl.cluster.G, wl.cluster.C, wl.cluster.host_mem_gb))
    for k in ("finish", "n_reconf", "progress", "held", "gpus_in_use", "frozen"):
        assert np.array_equal(loop[k], one[k]), k
    assert np.allclose(loop["totals"], one["totals"], rtol=1e-12)
    nodes = (128, 8, 128, 2048.0)
    out = orc.simulator.simulate(*args, policy="nodes", nodes=nodes, trace=True)
    fin = out["finish"] >= 0
    assert fin.sum() > 100 and out["n_reconf"].sum() > 0 and out["frozen"].sum() > 0
    levels = np.asarray(wl.grid.cpu_levels)
    spread = 0
    for k, (h, (off, ent)) in enumerate(zip(out["history"], out["placements"])):
        used_g, used_c = np.zeros(nodes[0], np.int64), np.zeros(nodes[0], np.int64)
        np.add.at(used_g, ent["node"], ent["g"])
        np.add.at(used_c, ent["node"], ent["c"])
        assert used_g.max(initial=0) <= nodes[1] and used_c.max(initial=0) <= nodes[2]
        per_job = np.add.reduceat(np.concatenate([ent["g"], [0]]), np.minimum(off[:-1], len(ent)))
        per_job[np.diff(off.astype(np.int64)) == 0] = 0
        assert np.array_equal(per_job, h["g"])
        spread += int((np.diff(off.astype(np.int64)) > 1).sum())
        t = 120.0 * k
        assert np.all(h["g"][tr.arrival > t] == 0)
    assert spread > 0
    print(f"over nodes: {int(fin.sum())} jobs finish, {int(out['n_reconf'].sum())} reconfigurations "
          f"(loop over totals: {int((loop['finish'] >= 0).sum())}, {int(loop['n_reconf'].sum())})")
