"""Pins of the oracle's placement-aware plan choice (Sec. 5.2, Algorithm 1,
ScheduleJob: the plan is selected given the found placement; Sec. 4.1
"Modeling T_comm": the bottleneck bandwidth of a communication group; last
paragraph of Sec. 5.2: jobs over several nodes see the inter-node bandwidth).

The bandwidth classes of a node split and three iteration times are worked
by hand below; the packed rule of the candidate evaluation is the special
case of splits at node boundaries; generated rounds are checked with the
pinned first-fit placement and a brute-force search over the plans."""
import numpy as np
import pytest

import oracle as orc
import workloads
from workloads import COEF_FIELDS

GIB = float(2 ** 30)
BIG = 1e30


def make_job(**kw):
    vals = dict(elem_bytes=2, mem_state=1, mem_act=34, mem_act_gc=2, mem_const=GIB, ref_thr=1)
    vals.update(kw)
    coef = np.array([vals[n] for n in COEF_FIELDS], dtype=np.float32)
    ints = np.array([vals["layers"], vals["gbatch"], vals["mbatch"]], dtype=np.uint32)
    return coef, ints


# one billion 2-byte parameters, 24 layers, 32 samples of 512 tokens x 2048 hidden: b*s*h = 2^25; plain sums (k = 1)
HAND_JOB = dict(P_bytes=2e9, seq=512, hidden=2048, t_fwd_sample=0.02, k_bwd=2, k_sync=1, k_opt=1e-11, k_opt_off=1e-9,
                k_off=1, k_swap=1, k_const=0.05, layers=24, gbatch=32, mbatch=1)
HAND_ENV = workloads.Env(B_intra=400e9, B_inter=25e9, B_pcie=32e9, gpu_mem_cap=BIG, gpus_per_node=4)
PLAIN = workloads.Bounds(g_max=8, zero_mask=1, gc_mask=1, off_mask=1)       # only the option without ZeRO, GC, offload


def classes(d, t, p, parts, env=HAND_ENV):
    coef, ints = make_job(**HAND_JOB)
    ints = ints.copy()
    ints[1] = 5040                                                          # a batch every d divides
    _, x = orc.eval_one_placed(coef, ints, workloads.Bounds(g_max=64), env, d, t, p, 0, 0, 0, 1, BIG, parts)
    name = {float(np.float32(env.B_intra)): "intra", float(np.float32(env.B_inter)): "inter"}   # the bandwidths are float32
    return name[x["B_tp"]], name[x["B_dp"]], name[x["B_pp"]]


def test_bandwidth_classes_of_a_node_split():
    # (tensor, data, pipeline) groups: intra-node only if all ranks of every such group sit on one node; ranks fill
    # the job's GPU slots in placement order, tensor-parallel ranks adjacent, then data-parallel, then stages
    assert classes(2, 2, 1, [4]) == ("intra", "intra", "intra")
    assert classes(2, 2, 1, [3, 1]) == ("inter", "inter", "inter")          # ranks 2,3 of the second TP pair are apart
    assert classes(2, 2, 1, [2, 2]) == ("intra", "inter", "inter")          # each TP pair on a node, DP pairs across
    assert classes(2, 4, 1, [4, 4]) == ("intra", "inter", "inter")
    assert classes(2, 4, 1, [4, 2, 2]) == ("inter", "inter", "inter")       # the second TP group of four is split 2+2
    assert classes(1, 2, 4, [4, 4]) == ("intra", "intra", "inter")          # stages 0,1 on one node, 2,3 on the other
    assert classes(2, 2, 2, [4, 4]) == ("intra", "intra", "inter")          # a whole stage (t*d = 4 ranks) per node
    assert classes(2, 2, 2, [2, 6]) == ("intra", "inter", "inter")
    assert classes(4, 1, 2, [6, 2]) == ("intra", "inter", "inter")          # t = 1: no TP traffic, class irrelevant
    assert classes(1, 1, 8, [8]) == ("intra", "intra", "intra")
    assert classes(8, 1, 1, [1] * 8) == ("intra", "inter", "inter")


def test_packed_split_is_the_rule_of_the_candidate_evaluation():
    """A job laid over whole nodes from a node boundary on is what the candidate evaluation assumes: every term equal."""
    wl = workloads.paper_scale()
    env = workloads.Env(gpus_per_node=8)
    b = workloads.Bounds(g_max=64)
    tb = orc.enumerate_plans(wl.ints[:6], b)
    n = 0
    for j in range(6):
        for d, t, p, v in tb.triples[tb.triple_off[j]:tb.triple_off[j + 1]].tolist():
            g = d * t * p
            parts = [8] * (g // 8) + ([g % 8] if g % 8 else [])
            for o in (0, 7, 13):
                z, gc, off = o >> 2, (o >> 1) & 1, o & 1
                want = orc.eval_one(wl.coef[j], wl.ints[j], b, env, d, t, p, z, gc, off, 3, BIG, v=v)
                got = orc.eval_one_placed(wl.coef[j], wl.ints[j], b, env, d, t, p, z, gc, off, 3, BIG, parts, v=v)
                assert got == want, (j, d, t, p, o)
                n += 1
    assert n > 1000


def test_iteration_times_on_a_split_by_hand():
    coef, ints = make_job(**HAND_JOB)

    def t_iter(d, t, p, parts):
        reason, x = orc.eval_one_placed(coef, ints, PLAIN, HAND_ENV, d, t, p, 0, 0, 0, 1, BIG, parts)
        assert reason == 0
        return x

    # d=2, t=2: 16 accumulation steps of 0.01 s forward + 0.02 s backward, V_dp = 1e9, V_tp = 16 * 2^25 * 6 bytes,
    # optimizer 0.01 s, constant 0.05 s: T_iter = 0.54 + T_dp + T_tp
    x = t_iter(2, 2, 1, [4])
    assert x["V_dp"] == pytest.approx(1e9, rel=1e-7) and x["V_tp"] == pytest.approx(3221225472.0, rel=1e-7)
    assert x["T_iter"] == pytest.approx(0.54 + 0.0025 + 0.00805306368, rel=1e-6)
    assert t_iter(2, 2, 1, [3, 1])["T_iter"] == pytest.approx(0.54 + 0.04 + 0.12884901888, rel=1e-6)
    assert t_iter(2, 2, 1, [2, 2])["T_iter"] == pytest.approx(0.54 + 0.04 + 0.00805306368, rel=1e-6)
    # p=4: 35 slots of 0.005 s forward, twice that backward, V_pp = 16 * 2^25 bytes: T_iter = 0.58 + T_pp
    assert t_iter(1, 1, 4, [4])["T_iter"] == pytest.approx(0.58 + 0.00134217728, rel=1e-6)
    assert t_iter(1, 1, 4, [3, 1])["T_iter"] == pytest.approx(0.58 + 0.02147483648, rel=1e-6)
    # t=2, p=2: 33 slots of 0.005 s, V_tp = 16 * 2^25 * 12, V_pp = 4 * 2^25: T_iter = 0.55 + T_tp + T_pp
    assert t_iter(1, 2, 2, [2, 2])["T_iter"] == pytest.approx(0.55 + 0.01610612736 + 0.00536870912, rel=1e-6)
    assert t_iter(1, 2, 2, [3, 1])["T_iter"] == pytest.approx(0.55 + 0.25769803776 + 0.00536870912, rel=1e-6)


def hand_round(filler_g, asked=4, floor=None, n_nodes=2, per_gpu=False):
    """A filler job on `filler_g` GPUs of node 0, then the hand job asking for `asked` GPUs, on nodes of 4 GPUs.
    per_gpu: 2 CPUs and 10 GiB per GPU on nodes of 8 CPUs and 40 GiB, instead of 1 CPU and 64 GiB per job."""
    coef, ints = make_job(**HAND_JOB)
    fill_c, fill_i = make_job(**dict(HAND_JOB, layers=1, gbatch=6))
    coef2, ints2 = np.stack([fill_c, coef]), np.stack([fill_i, ints])
    tb = orc.enumerate_plans(ints2, PLAIN)
    grid = workloads.Grid(np.array([1], np.uint32), 0, np.array([64.0], np.float32), 0)
    if per_gpu:
        grid = workloads.Grid(np.array([2], np.uint32), 1, np.array([10.0], np.float32), 1)
    thr, _ = orc.eval_jobs(coef2, ints2, PLAIN, tb, grid, HAND_ENV)
    bt64, bp = orc.best_plan(tb, grid, thr)
    a = np.zeros(2, orc.ASSIGN_DTYPE)
    a["g"], a["c"], a["mem_gb"] = [filler_g, asked], [1 if filler_g else 0, 1], [64.0 if filler_g else 0.0, 64.0]
    if per_gpu:
        a["c"], a["mem_gb"] = [2 * filler_g, 2 * asked], [10.0 * filler_g, 10.0 * asked]
    counts = tb.seg_g[tb.seg_off[1]:tb.seg_off[2]].tolist()
    assert counts == [1, 2, 3, 4, 6, 8]                          # pipeline stages divide 24 layers, replicas divide 32 samples
    ms = None if floor is None else np.array([-1, counts.index(floor)], np.int32)     # floor: a GPU count of the job
    out, off, ent, st, total = orc.place_plans(coef2, ints2, PLAIN, tb, grid, HAND_ENV, bt64.astype(np.float32), a, n_nodes, 4,
                                               8, 40.0 if per_gpu else 1000.0, min_seg=ms)
    plan = None
    if out["plan"][1] != orc.NO_PLAN:
        plan = tuple(int(x) for x in tb.triples[tb.triple_off[1] + out["plan"][1] // 16][:3])
    return out, [int(e["g"]) for e in ent[off[1]:off[2]]], st.tolist(), plan, total


def test_a_split_flips_the_best_plan():
    # alone on a node: data x tensor parallel 2 x 2 is the best plan of four GPUs
    out, parts, st, plan, total = hand_round(0)
    assert parts == [4] and st == [0, 1] and plan == (2, 2, 1)
    assert out["thr"][1] == np.float32(32 / (0.54 + 0.0025 + 0.00805306368)) and total == pytest.approx(58.1233, rel=1e-5)
    # one GPU of node 0 is taken: first fit splits 3 + 1, every group crosses the nodes, the pipeline moves the least
    out, parts, st, plan, _ = hand_round(1)
    assert parts == [3, 1] and st == [1, 1] and plan == (1, 1, 4)
    assert out["thr"][1] == pytest.approx(32 / (0.58 + 0.02147483648), rel=1e-6)
    assert (out["g"][1], out["c"][1], out["mem_gb"][1]) == (4, 1, 64.0)
    # two are taken: 2 + 2 keeps tensor-parallel pairs together
    out, parts, st, plan, _ = hand_round(2)
    assert parts == [2, 2] and plan == (1, 2, 2)
    assert out["thr"][1] == pytest.approx(32 / (0.55 + 0.01610612736 + 0.00536870912), rel=1e-6)


def test_a_job_that_does_not_fit_takes_its_next_smaller_count():
    # three GPUs of node 0 are taken; eight are asked, five are free: six do not fit either, the job runs on four (1 + 3)
    out, parts, st, plan, _ = hand_round(3, asked=8)
    assert st == [1, 2] and parts == [1, 3] and out["g"][1] == 4 and plan == (1, 1, 4)
    assert out["thr"][1] == pytest.approx(32 / (0.58 + 0.02147483648), rel=1e-6)
    # not below its floor: with eight as the minimum it waits, with four it runs
    out, parts, st, plan, total = hand_round(3, asked=8, floor=8)
    assert st == [1, 3] and parts == [] and out["g"][1] == 0 and plan is None and out["thr"][1] == 0
    out, parts, st, plan, _ = hand_round(3, asked=8, floor=6)
    assert st == [1, 3] and out["g"][1] == 0
    out, parts, st, plan, _ = hand_round(3, asked=8, floor=4)
    assert st == [1, 2] and out["g"][1] == 4
    # amounts per GPU shrink with the count: 8 GPUs would hold 16 CPUs and 80 GiB, the 4 that fit hold 8 and 40 -
    # 1 GPU, 2 CPUs, 10 GiB beside the filler (3 GPUs, 6 CPUs, 30 GiB) and 3 GPUs, 6 CPUs, 30 GiB on the other node
    out, parts, st, plan, _ = hand_round(3, asked=8, per_gpu=True)
    assert st == [1, 2] and parts == [1, 3]
    assert (out["g"][1], out["c"][1], out["mem_gb"][1]) == (4, 8, 40.0) and plan == (1, 1, 4)
    # with room for all eight nothing changes: 1 + 4 + 3 over three nodes
    out, parts, st, plan, _ = hand_round(3, asked=8, n_nodes=3)
    assert st == [1, 1] and parts == [1, 4, 3] and out["g"][1] == 8


@pytest.mark.parametrize("cpn,mpn", [(64, 4096.0), (2, 4096.0), (64, 100.0)])
def test_generated_round_against_first_fit_and_brute_force(cpn, mpn):
    """paper_scale jobs limited to 6 GPUs each (15 of them run, on 1, 4, 5 or 6 GPUs) on 8 nodes x 8 GPUs with roomy,
    CPU-short and memory-short nodes."""
    import dataclasses
    wl = dataclasses.replace(workloads.paper_scale(), bounds=workloads.Bounds(g_max=6))
    r = orc.schedule_round(wl, n_threads=4)
    tb, grid = r["table"], wl.grid
    floors = np.full(wl.n_jobs, -1, np.int32)
    floors[::5] = 1                                              # some jobs may not go below their second count
    out, off, ent, st, total = orc.place_plans(wl.coef, wl.ints, wl.bounds, tb, grid, wl.env, r["best_thr"], r["assign"], 8, 8,
                                               cpn, mpn, min_seg=floors)
    # 1. the amounts that were placed, given to the pinned first fit, give the same parts
    p_off, p_ent, p_st = orc.place(out, 8, 8, cpn, mpn)
    assert np.array_equal(p_off, off) and np.array_equal(p_ent, ent)
    assert np.array_equal(p_st == 1, (st == 1) | (st == 2)) and np.array_equal(p_st == 0, (st == 0) | (st == 3))
    rows = len(grid.cpu_levels) * len(grid.mem_levels_gb)
    n_multi = n_changed = n_retried = 0
    for j in range(wl.n_jobs):
        a = r["assign"][j]
        if a["g"] == 0:
            assert st[j] == 0
            continue
        seg_g = tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]].tolist()
        ns = len(seg_g)
        ci = int(np.flatnonzero(grid.cpu_levels == a["c"])[0])
        bt = r["best_thr"][rows * int(tb.seg_off[j]):rows * int(tb.seg_off[j + 1])].reshape(rows, ns)[ci]
        s0, s_min = seg_g.index(a["g"]), max(int(floors[j]), 0)
        s_got = seg_g.index(out["g"][j]) if out["g"][j] else -1
        assert st[j] == (1 if s_got == s0 else 2 if s_got >= 0 else 3)
        assert s_got == -1 or s_got >= s_min
        # 2. every larger count the job was entitled to try does not fit at its turn (pinned first fit on a prefix)
        for s in range(s0, max(s_got, s_min - 1), -1):
            if s < s_min or not bt[s] > 0:
                continue
            trial = out[:j + 1].copy()
            trial[j] = (seg_g[s], a["c"], a["mem_gb"], 0, 0)
            assert orc.place(trial, 8, 8, cpn, mpn)[2][j] == 2, (j, s)
        if s_got < 0:
            continue
        n_retried += st[j] == 2
        # 3. the plan: brute force over the plans of the placed count on the actual split
        parts = ent["g"][off[j]:off[j + 1]].tolist()
        n_multi += len(parts) > 1
        g = seg_g[s_got]
        best, arg = 0.0, None
        tr = tb.triples[tb.triple_off[j]:tb.triple_off[j + 1]]
        for tl in np.flatnonzero(tr[:, :3].prod(axis=1) == g).tolist():
            d, t, p, v = (int(x) for x in tr[tl])
            for o in range(16):
                reason, x = orc.eval_one_placed(wl.coef[j], wl.ints[j], wl.bounds, wl.env, d, t, p, o >> 2, (o >> 1) & 1, o & 1,
                                                int(a["c"]), float(a["mem_gb"]) * GIB, parts, v=v)
                if reason == 0 and x["thr"] > best:
                    best, arg = x["thr"], tl * 16 + o
        assert out["plan"][j] == arg and out["thr"][j] == np.float32(best)
        assert (out["c"][j], out["mem_gb"][j]) == (a["c"], a["mem_gb"])       # absolute CPU levels and tiers here
        n_changed += out["plan"][j] != a["plan"] and st[j] == 1
    assert total == pytest.approx(float((out["thr"].astype(np.float64) / wl.coef[:, 16]).sum()), rel=1e-12)
    assert n_multi >= 2
    if cpn == 2:
        assert n_retried + int((st == 3).sum()) >= 1
    print(f"cpn={cpn} mpn={mpn}: {int(((st == 1) | (st == 2)).sum())} placed, {n_multi} over several nodes, {n_changed} plans "
          f"changed by the split, {n_retried} with fewer GPUs, {int((st == 3).sum())} not placed")


# ---------------------------------------------------------------- jobs that stay where they are
def stay_jobs(n):
    """n copies of the hand job (counts 1, 2, 3, 4, 6, 8; 1 CPU and 64 GiB per job) with their maxima on a one-row grid."""
    coef, ints = make_job(**HAND_JOB)
    coef_n, ints_n = np.stack([coef] * n), np.stack([ints] * n)
    tb = orc.enumerate_plans(ints_n, PLAIN)
    grid = workloads.Grid(np.array([1], np.uint32), 0, np.array([64.0], np.float32), 0)
    thr, _ = orc.eval_jobs(coef_n, ints_n, PLAIN, tb, grid, HAND_ENV)
    bt = orc.best_plan(tb, grid, thr)[0].astype(np.float32)
    return coef_n, ints_n, tb, grid, bt


def stay_round(jobs, gs, prev=None, n_nodes=2, cpn=8):
    coef, ints, tb, grid, bt = jobs
    a = np.zeros(len(gs), orc.ASSIGN_DTYPE)
    a["g"] = gs
    a["c"] = [1 if g else 0 for g in gs]
    a["mem_gb"] = [64.0 if g else 0.0 for g in gs]
    out, off, ent, st, total = orc.place_plans(coef, ints, PLAIN, tb, grid, HAND_ENV, bt, a, n_nodes, 4, cpn, 1000.0, prev=prev)
    parts = [[(int(e["node"]), int(e["g"])) for e in ent[off[j]:off[j + 1]]] for j in range(len(gs))]
    return out, off, ent, st.tolist(), parts


def test_running_jobs_stay_on_their_nodes():
    jobs = stay_jobs(4)
    # first round: A takes 3 GPUs of node 0, B 1 + 3, C the last GPU of node 1; D is not there yet
    out1, off1, ent1, st1, parts1 = stay_round(jobs, [3, 4, 1, 0])
    assert parts1 == [[(0, 3)], [(0, 1), (1, 3)], [(1, 1)], []] and st1 == [1, 1, 1, 0]
    # A leaves, D arrives with 3 GPUs.  Laid out anew B would move to node 0; with the earlier placement B and C stay
    # and D takes the three GPUs that A left
    _, _, _, st_new, parts_new = stay_round(jobs, [0, 4, 1, 3])
    assert parts_new == [[], [(0, 4)], [(1, 1)], [(1, 3)]]
    out2, _, _, st2, parts2 = stay_round(jobs, [0, 4, 1, 3], prev=(off1, ent1))
    assert parts2 == [[], [(0, 1), (1, 3)], [(1, 1)], [(0, 3)]] and st2 == [0, 1, 1, 1]
    # B's plan is the one of its split 1 + 3 (every group crosses the nodes: four pipeline stages), as in round one
    assert out2["plan"][1] == out1["plan"][1] and out2["thr"][1] == out1["thr"][1]
    assert out2["thr"][1] == pytest.approx(32 / (0.58 + 0.02147483648), rel=1e-6)


def test_a_newcomer_with_a_lower_index_does_not_take_a_kept_jobs_gpus():
    jobs = stay_jobs(2)
    _, off1, ent1, _, parts1 = stay_round(jobs, [0, 4])
    assert parts1 == [[], [(0, 4)]]
    # job 0 arrives and asks for 4: in index order from empty nodes it would take node 0; job 1 is booked first
    _, _, _, st2, parts2 = stay_round(jobs, [4, 4], prev=(off1, ent1))
    assert parts2 == [[(1, 4)], [(0, 4)]] and st2 == [1, 1]
    # and falls back to a smaller count when what is left is less than it asks for
    _, _, _, st3, parts3 = stay_round(jobs, [8, 4], prev=(off1, ent1))
    assert parts3 == [[(1, 4)], [(0, 4)]] and st3 == [2, 1]


def test_a_job_whose_amounts_changed_is_placed_again():
    jobs = stay_jobs(3)
    _, off1, ent1, _, parts1 = stay_round(jobs, [2, 3, 2])
    assert parts1 == [[(0, 2)], [(0, 2), (1, 1)], [(1, 2)]]
    # job 1 shrinks to 2 GPUs: its parts are released, jobs 0 and 2 stay, job 1 first-fits into what is free (node 0)
    _, _, _, st2, parts2 = stay_round(jobs, [2, 2, 2], prev=(off1, ent1))
    assert parts2 == [[(0, 2)], [(0, 2)], [(1, 2)]] and st2 == [1, 1, 1]
    # job 0 grows to 4: released and placed again in its turn, after the kept jobs were booked: node 0 has 2 free,
    # node 1 has 1 free -> 3 GPUs at most: it falls back to 3
    out3, _, _, st3, parts3 = stay_round(jobs, [4, 3, 2], prev=(off1, ent1))
    assert parts3 == [[(0, 2), (1, 1)], [(0, 2), (1, 1)], [(1, 2)]] and st3 == [2, 1, 1] and out3["g"][0] == 3
    # the same GPUs with another CPU amount is a change as well (the parts' CPUs would differ)
    coef, ints, tb, grid, bt = jobs
    a = np.zeros(3, orc.ASSIGN_DTYPE)
    a["g"], a["c"], a["mem_gb"] = [2, 3, 2], [1, 1, 1], [64.0, 64.0, 64.0]
    ent_c = ent1.copy()
    ent_c["c"][off1[1]] += 1                                         # job 1's first part claims one CPU more than first fit books
    out, off, ent, st, _ = orc.place_plans(coef, ints, PLAIN, tb, grid, HAND_ENV, bt, a, 2, 4, 8, 1000.0, prev=(off1, ent_c))
    assert [(int(e["node"]), int(e["g"])) for e in ent[off[1]:off[2]]] == [(0, 2), (1, 1)] and st.tolist() == [1, 1, 1]
    assert int(ent["c"][off[1]]) + int(ent["c"][off[1] + 1]) == 1    # placed again with what first fit books


def test_a_job_that_grew_is_not_kept_on_its_smaller_parts():
    """One CPU per GPU and no host memory: the parts of 3 GPUs are exactly the first parts that 4 GPUs would get, so
    only the GPU total tells that the job has changed."""
    coef, ints, tb, _, _ = stay_jobs(2)
    grid = workloads.Grid(np.array([1], np.uint32), 1, np.array([0.0], np.float32), 1)
    thr, _ = orc.eval_jobs(coef, ints, PLAIN, tb, grid, HAND_ENV)
    bt = orc.best_plan(tb, grid, thr)[0].astype(np.float32)

    def round_(gs, prev=None):
        a = np.zeros(2, orc.ASSIGN_DTYPE)
        a["g"], a["c"] = gs, gs
        out, off, ent, st, _ = orc.place_plans(coef, ints, PLAIN, tb, grid, HAND_ENV, bt, a, 2, 4, 8, 1000.0, prev=prev)
        return off, ent, st.tolist(), [[(int(e["node"]), int(e["g"]), int(e["c"])) for e in ent[off[j]:off[j + 1]]] for j in range(2)]

    off1, ent1, st1, parts1 = round_([2, 3])
    assert parts1 == [[(0, 2, 2)], [(0, 2, 2), (1, 1, 1)]]
    _, _, st2, parts2 = round_([2, 4], prev=(off1, ent1))
    assert parts2 == [[(0, 2, 2)], [(0, 2, 2), (1, 2, 2)]] and st2 == [1, 1]


def test_an_earlier_placement_that_does_not_fit_is_refused():
    jobs = stay_jobs(2)
    _, off1, ent1, _, _ = stay_round(jobs, [4, 4])
    both_on_node_0 = ent1.copy()
    both_on_node_0["node"][:] = 0
    with pytest.raises(AssertionError):
        stay_round(jobs, [4, 4], prev=(off1, both_on_node_0))
    off_node = ent1.copy()
    off_node["node"][1] = 7                                          # a node the cluster does not have: the job does not stay
    _, _, _, st, parts = stay_round(jobs, [4, 4], prev=(off1, off_node))
    assert parts == [[(0, 4)], [(1, 4)]] and st == [1, 1]


def test_generated_rounds_with_an_earlier_placement():
    """paper_scale jobs of at most 6 GPUs on 8 nodes x 8 GPUs: a round, then a quarter of the running jobs leave, the
    others keep their amounts, newcomers take the free slots of the job list.  Every job that kept its amounts keeps
    its parts, nothing exceeds a node, the newcomers are placed by first fit into what the kept jobs leave."""
    import dataclasses
    wl = dataclasses.replace(workloads.paper_scale(), bounds=workloads.Bounds(g_max=6))
    r = orc.schedule_round(wl, n_threads=4)
    tb, grid = r["table"], wl.grid
    args = (wl.coef, wl.ints, wl.bounds, tb, grid, wl.env, r["best_thr"])
    a1 = r["assign"]
    out1, off1, ent1, st1, _ = orc.place_plans(*args, a1, 8, 8, 64, 4096.0)
    running = np.flatnonzero(st1 == 1)
    assert running.size >= 10
    n_kept = n_new = 0
    for seed in range(20):
        rng = np.random.default_rng(seed)
        a2 = out1.copy()                                             # what the jobs hold after round one
        leave = running[rng.uniform(size=running.size) < 0.25]
        a2[leave] = (0, 0, 0.0, orc.NO_PLAN, 0.0)
        idle = np.flatnonzero(a2["g"] == 0)
        arrive = idle[rng.uniform(size=idle.size) < 0.3]
        for j in arrive:                                             # a newcomer asks for what the round gave some running job
            src = int(rng.choice(running))
            seg_g = tb.seg_g[tb.seg_off[j]:tb.seg_off[j + 1]]
            rows = len(grid.cpu_levels) * len(grid.mem_levels_gb)
            row0 = r["best_thr"][rows * int(tb.seg_off[j]):][:seg_g.size]       # lowest CPU level, first tier
            ok = [s for s in range(seg_g.size) if row0[s] > 0]
            if not ok:
                continue
            s = int(rng.choice(ok))
            a2[j] = (int(seg_g[s]), int(grid.cpu_levels[0]), float(grid.mem_levels_gb[0]), 0, 0.0)
        out2, off2, ent2, st2, _ = orc.place_plans(*args, a2, 8, 8, 64, 4096.0, prev=(off1, ent1))
        stay = np.flatnonzero((a2["g"] > 0) & (a2["g"] == out1["g"]) & (a2["c"] == out1["c"]) & (a2["mem_gb"] == out1["mem_gb"])
                              & (st1 > 0))
        for j in stay:
            assert np.array_equal(ent2[off2[j]:off2[j + 1]], ent1[off1[j]:off1[j + 1]]) and st2[j] == 1
        n_kept += stay.size
        used_g = np.bincount(ent2["node"], weights=ent2["g"], minlength=8)
        used_c = np.bincount(ent2["node"], weights=ent2["c"], minlength=8)
        assert used_g.max() <= 8 and used_c.max() <= 64
        # the others, given to the pinned first fit on nodes that hold the kept parts already, get the same parts:
        # replay them one by one in index order
        freeG = np.full(8, 8, np.int64)
        for j in stay:
            for e in ent1[off1[j]:off1[j + 1]]:
                freeG[e["node"]] -= int(e["g"])
        for j in np.flatnonzero((a2["g"] > 0) & ~np.isin(np.arange(wl.n_jobs), stay)):
            n_new += 1
            if st2[j] == 3:
                continue
            g = int(out2["g"][j])
            need, want = g, []
            for n in range(8):                                       # GPUs bind alone here (64 CPUs, 4 TiB per node)
                k = int(min(freeG[n], need))
                if k:
                    want.append((n, k))
                    need -= k
                if need == 0:
                    break
            assert need == 0 and [(int(e["node"]), int(e["g"])) for e in ent2[off2[j]:off2[j + 1]]] == want
            for n, k in want:
                freeG[n] -= k
    assert n_kept > 100 and n_new > 30
