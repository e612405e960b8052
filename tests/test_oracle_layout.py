"""Pins for the oracle's candidate layout and for the per-GPU modes of the
allocation grid.

`eval_jobs` is walked index by index, (job, CPU level, memory tier, triple,
option), and every entry is compared with the pinned one-candidate evaluation
called with a CPU count and a host-memory size that are written out here from
the definitions (Table 1: c is the job's CPUs; Sec. 4.2: T_opt =
k_opt_off * P / (d * c); a level of a per-GPU grid stands for level * g CPUs,
a tier for GiB * g).  The greedy gets hand cases in which exactly those
products decide the result."""
import itertools

import numpy as np
import pytest

import workloads

GIB32 = np.float32(2 ** 30)


def small_jobs():
    """Four jobs of the paper-scale mix, on GPUs small enough that offloaded plans matter."""
    base = workloads.paper_scale()
    pick = [0, 7, 21, 40]
    return base.coef[pick].copy(), base.ints[pick].copy()


@pytest.mark.parametrize("cpu_mode,mem_mode", list(itertools.product((0, 1), (0, 1))))
def test_eval_jobs_index_by_index(orc, cpu_mode, mem_mode):
    coef, ints = small_jobs()
    bounds = workloads.Bounds(g_max=8, tp_max=4, pp_max=4)
    cpu_levels = np.array([1, 3, 8], np.uint32)                      # three CPU levels ...
    mem_levels = np.array([0.0, 6.0, 48.0, 512.0], np.float32)       # ... four tiers: a transposed layout cannot pass
    grid = workloads.Grid(cpu_levels, cpu_mode, mem_levels, mem_mode)
    env = workloads.Env(gpu_mem_cap=12e9, gpus_per_node=4)
    tb = orc.enumerate_plans(ints, bounds)
    jb, je = 1, 4                                                    # a range that does not start at job 0
    thr, reason = orc.eval_jobs(coef, ints, bounds, tb, grid, env, jb, je)
    n_cpu, n_mem = len(cpu_levels), len(mem_levels)
    k = 0
    seen_host_fail = seen_cpu_effect = 0
    for j in range(jb, je):
        t0, t1 = int(tb.triple_off[j]), int(tb.triple_off[j + 1])
        for ci in range(n_cpu):
            for mi in range(n_mem):
                for tl in range(t1 - t0):
                    d, t, p, v = (int(x) for x in tb.triples[t0 + tl])
                    g = d * t * p
                    c = int(cpu_levels[ci]) * g if cpu_mode else int(cpu_levels[ci])
                    host = mem_levels[mi] * GIB32                    # float32 products, as the header states
                    if mem_mode:
                        host = host * np.float32(g)
                    for o in range(16):
                        z, gc, off = o >> 2, (o >> 1) & 1, o & 1
                        want_reason, x = orc.eval_one(coef[j], ints[j], bounds, env, d, t, p, z, gc, off, c,
                                                      float(host), v=v)
                        assert reason[k] == want_reason, (j, ci, mi, tl, o)
                        assert thr[k] == (0.0 if want_reason else x["thr"]), (j, ci, mi, tl, o)
                        seen_host_fail += bool(want_reason & 4)
                        if off and not want_reason and ci:
                            # the same plan one CPU level lower, at this entry's own tier
                            lower = k - n_mem * (t1 - t0) * 16
                            seen_cpu_effect += bool(reason[lower] == 0 and thr[lower] < thr[k])
                        k += 1
    assert k == thr.size == reason.size
    # the case is not a trivial one: host memory does bind somewhere, CPUs do change offloaded plans
    assert seen_host_fail > 50 and seen_cpu_effect > 50


def test_per_gpu_modes_change_what_they_should(orc):
    """The same level vector read per job and per GPU: entries of one-GPU plans
    coincide, entries of wider plans see g times the CPUs and g times the host memory."""
    coef, ints = small_jobs()
    bounds = workloads.Bounds(g_max=4, tp_max=2, pp_max=2)
    env = workloads.Env(gpu_mem_cap=12e9, gpus_per_node=4)
    tb = orc.enumerate_plans(ints, bounds)
    cpu, mem = np.array([2, 5], np.uint32), np.array([4.0, 20.0], np.float32)
    out = {}
    for cm, mm in itertools.product((0, 1), (0, 1)):
        out[cm, mm] = orc.eval_jobs(coef, ints, bounds, tb, workloads.Grid(cpu, cm, mem, mm), env)
    g_of = []
    for j in range(len(ints)):
        tr = tb.triples[tb.triple_off[j]:tb.triple_off[j + 1], :3].prod(axis=1)
        g_of.append(np.tile(np.repeat(tr, 16), 4))
    g_of = np.concatenate(g_of)
    one = g_of == 1
    for key in out:
        assert np.array_equal(out[key][0][one], out[0, 0][0][one])
        assert np.array_equal(out[key][1][one], out[0, 0][1][one])
    wide = ~one
    # per-GPU CPUs: never slower, somewhere faster; per-GPU memory: never less feasible, somewhere more
    ok = (out[0, 0][1] == 0) & wide
    assert (out[1, 0][0][ok] >= out[0, 0][0][ok]).all() and (out[1, 0][0][ok] > out[0, 0][0][ok]).any()
    assert ((out[0, 1][1] & 4) <= (out[0, 0][1] & 4)).all()
    assert ((out[0, 1][1] & 4) < (out[0, 0][1] & 4)).any()


def one_job_table(orc, g_max, n_jobs=1):
    """Jobs whose every GPU count 1..g_max is valid with exactly one triple (tp = pp = 1)."""
    import math
    lcm = 1
    for v in range(1, g_max + 1):
        lcm = lcm * v // math.gcd(lcm, v)
    ints = np.tile(np.array([[1, lcm, 1]], np.uint32), (n_jobs, 1))
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=g_max, tp_max=1))
    assert tb.seg_g.tolist() == list(range(1, g_max + 1)) * n_jobs
    return tb


def test_greedy_cpus_per_gpu_limit_a_gpu_step(orc):
    # one job, linear in GPUs, CPU levels 2 and 3 per GPU, 7 CPUs in the cluster:
    # three GPUs cost 6 CPUs, four would cost 8; afterwards level 3 would cost 9
    tb = one_job_table(orc, 4)
    bt = np.array([[1.0, 2.0, 3.0, 4.0], [1.5, 3.0, 4.5, 6.0]], np.float32)          # [cpu level][segment]
    bp = np.arange(8, dtype=np.uint32)
    ref = np.ones(1, np.float32)
    per_gpu = workloads.Grid(np.array([2, 3], np.uint32), 1, np.array([1.0], np.float32), 0)
    ct, _, _ = orc.curves(tb, per_gpu, bt.reshape(-1), bp)
    a, total, _ = orc.greedy(ref, tb, per_gpu, workloads.Cluster(4, 7, 100.0), bt.reshape(-1), bp, ct)
    assert (a["g"][0], a["c"][0], a["thr"][0], a["plan"][0]) == (3, 6, 3.0, 2)
    # nine CPUs: the CPU pass can raise the three GPUs to level 3, which four GPUs at level 2 (8 CPUs) leave no room for
    a, total, _ = orc.greedy(ref, tb, per_gpu, workloads.Cluster(3, 9, 100.0), bt.reshape(-1), bp, ct)
    assert (a["g"][0], a["c"][0], a["thr"][0], a["plan"][0]) == (3, 9, 4.5, 6)
    a, total, _ = orc.greedy(ref, tb, per_gpu, workloads.Cluster(4, 9, 100.0), bt.reshape(-1), bp, ct)
    assert (a["g"][0], a["c"][0], a["thr"][0]) == (4, 8, 4.0)
    # the same numbers read as CPUs of the whole job: four GPUs with 2 CPUs, then 3
    per_job = workloads.Grid(np.array([2, 3], np.uint32), 0, np.array([1.0], np.float32), 0)
    a, total, _ = orc.greedy(ref, tb, per_job, workloads.Cluster(4, 7, 100.0), bt.reshape(-1), bp, ct)
    assert (a["g"][0], a["c"][0], a["thr"][0], a["plan"][0]) == (4, 3, 6.0, 7)


def test_greedy_cpu_pass_gain_is_per_added_cpu_of_the_job(orc):
    # two jobs hold 1 and 4 GPUs (the only counts they gain from); level 1 -> 2 per GPU costs the first job 1 CPU
    # and the second 4: the second job gains twice as much throughput, which is half the first job's gain per CPU
    tb = one_job_table(orc, 4, n_jobs=2)
    grid = workloads.Grid(np.array([1, 2], np.uint32), 1, np.array([1.0], np.float32), 0)
    bt = np.array([[[5.0, 5.0, 5.0, 5.0], [6.0, 6.0, 6.0, 6.0]],
                   [[0.0, 0.0, 0.0, 8.0], [0.0, 0.0, 0.0, 10.0]]], np.float32)       # [job][cpu level][segment]
    bp = np.arange(16, dtype=np.uint32)
    bp[bt.reshape(-1) == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, bt.reshape(-1), bp)
    ref = np.ones(2, np.float32)
    # 5 GPUs; CPUs: 5 at level 1, 4 spare: job 0 takes 1 of them (slope 1), job 1 cannot have 4 any more
    a, _, _ = orc.greedy(ref, tb, grid, workloads.Cluster(5, 9, 100.0), bt.reshape(-1), bp, ct)
    assert a["g"].tolist() == [1, 4] and a["c"].tolist() == [2, 4] and a["thr"].tolist() == [6.0, 8.0]
    # 5 spare: both
    a, _, _ = orc.greedy(ref, tb, grid, workloads.Cluster(5, 10, 100.0), bt.reshape(-1), bp, ct)
    assert a["c"].tolist() == [2, 8] and a["thr"].tolist() == [6.0, 10.0]


def test_greedy_memory_per_gpu_costs_gib_times_g(orc):
    # tiers of 10 and 30 GiB per GPU; job 0 ends with 3 GPUs (tiers cost 30 / 90), job 1 with 2 (20 / 60)
    tb = one_job_table(orc, 3, n_jobs=2)
    grid = workloads.Grid(np.array([1], np.uint32), 0, np.array([10.0, 30.0], np.float32), 1)
    bt = np.array([[[1.0, 2.0, 3.0], [1.0, 2.0, 3.5]],                               # [job][tier][segment]
                   [[1.0, 1.75, 1.75], [1.0, 2.5, 2.5]]], np.float32)
    bp = np.arange(12, dtype=np.uint32)
    ct, _, _ = orc.curves(tb, grid, bt.reshape(-1), bp)
    ref = np.ones(2, np.float32)
    flat = bt.reshape(-1)
    # ample memory: both take the large tier, booked as GiB * g
    a, total, _ = orc.greedy(ref, tb, grid, workloads.Cluster(5, 100, 1000.0), flat, bp, ct)
    assert a["g"].tolist() == [3, 2] and a["mem_gb"].tolist() == [90.0, 60.0] and a["thr"].tolist() == [3.5, 2.5]
    # 100 GiB: job 0 takes 90, job 1 finds 10 left, less than its small tier's 20: dropped
    a, total, _ = orc.greedy(ref, tb, grid, workloads.Cluster(5, 100, 100.0), flat, bp, ct)
    assert a["mem_gb"].tolist() == [90.0, 0.0] and a["g"].tolist() == [3, 0] and total == pytest.approx(3.5)
    # 80 GiB: job 0 only fits the small tier (30), job 1 then has 50: small tier again (20)
    a, total, _ = orc.greedy(ref, tb, grid, workloads.Cluster(5, 100, 80.0), flat, bp, ct)
    assert a["mem_gb"].tolist() == [30.0, 20.0] and a["thr"].tolist() == [3.0, 1.75]
    assert a["plan"].tolist() == [2, 7]
    # the same tiers for the whole job: 80 GiB hold 30 + 30
    per_job = workloads.Grid(np.array([1], np.uint32), 0, np.array([10.0, 30.0], np.float32), 0)
    a, total, _ = orc.greedy(ref, tb, per_job, workloads.Cluster(5, 100, 80.0), flat, bp, ct)
    assert a["mem_gb"].tolist() == [30.0, 30.0] and a["thr"].tolist() == [3.5, 2.5]


def test_round_on_a_per_gpu_grid_books_what_it_grants(orc):
    """A generated round on a per-GPU grid in both dimensions: the records' CPUs and
    memory are level * g and GiB * g, the capacities hold, and the granted
    throughput is the candidate tensor's entry at (level, tier, plan)."""
    base = workloads.paper_scale()
    grid = workloads.Grid(np.array([1, 2, 4], np.uint32), 1, np.array([0.0, 8.0, 64.0], np.float32), 1)
    env = workloads.Env(gpu_mem_cap=4e9)                 # small GPUs: offloaded plans, which need CPUs and host memory, win
    wl = workloads.Workload("per_gpu", base.coef[:20], base.ints[:20], workloads.Bounds(g_max=16), grid, env,
                            workloads.Cluster(48, 120, 900.0))
    r = orc.schedule_round(wl, n_threads=4)
    a, tb = r["assign"], r["table"]
    assert a["g"].sum() <= 48 and a["c"].sum() <= 120 and a["mem_gb"].sum() <= 900.0
    used_tiers, used_levels = set(), set()
    for j in np.flatnonzero(a["g"] > 0):
        g = int(a["g"][j])
        assert a["c"][j] % g == 0 and a["c"][j] // g in (1, 2, 4)
        per = float(a["mem_gb"][j]) / g
        assert per in (0.0, 8.0, 64.0)
        ci, mi = (1, 2, 4).index(a["c"][j] // g), (0.0, 8.0, 64.0).index(per)
        used_tiers.add(mi)
        used_levels.add(ci)
        nt = int(tb.triple_off[j + 1] - tb.triple_off[j])
        k = 16 * 9 * int(tb.triple_off[j]) + ((ci * 3 + mi) * nt) * 16 + int(a["plan"][j])
        assert np.float32(r["thr"][k]) == a["thr"][j] and r["reason"][k] == 0
    assert len(used_tiers) >= 2 and len(used_levels) >= 2 and (a["g"] > 0).sum() >= 5
