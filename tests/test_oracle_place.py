"""Pins of the oracle's node-level placement (Sec. 5.2, Algorithm 1, ScheduleJob:
a job walks the nodes in order and takes what is free on each): cases worked by
hand, the closed form when only GPUs bind (jobs laid end to end on the nodes'
GPU slots), and a checker that replays any result and verifies the first-fit
property part by part."""
import numpy as np
import pytest

import oracle as orc


def jobs(g, c, mem):
    a = np.zeros(len(g), orc.ASSIGN_DTYPE)
    a["g"], a["c"], a["mem_gb"] = g, c, mem
    return a


def parts(off, ent, j):
    return [(int(e["node"]), int(e["g"]), int(e["c"]), float(e["mem_gb"])) for e in ent[off[j]:off[j + 1]]]


def test_hand_case_two_nodes():
    # 2 nodes x 4 GPUs; jobs of 3, 2 and 3 GPUs end to end: 3 | 1+1 | 3
    off, ent, st = orc.place(jobs([3, 2, 3], [6, 4, 3], [3.0, 8.0, 1.5]), 2, 4, 100, 100.0)
    assert st.tolist() == [1, 1, 1] and off.tolist() == [0, 1, 3, 4]
    assert parts(off, ent, 0) == [(0, 3, 6, 3.0)]
    assert parts(off, ent, 1) == [(0, 1, 2, 4.0), (1, 1, 2, 4.0)]
    assert parts(off, ent, 2) == [(1, 3, 3, 1.5)]


def test_cpus_of_a_split_job_add_up():
    # 5 CPUs over three parts of one GPU each: floor(5/3), floor(10/3) - 1, 5 - 3
    off, ent, st = orc.place(jobs([3], [5], [0.0]), 3, 1, 8, 1.0)
    assert [p[2] for p in parts(off, ent, 0)] == [1, 2, 2]


def test_cpus_bind_and_a_later_job_fills_the_hole():
    # node 0 loses all 8 CPUs to job 0 (4 per GPU) but keeps 2 GPUs; job 1 needs CPUs and moves on, job 2 needs none
    off, ent, st = orc.place(jobs([2, 2, 2], [8, 2, 0], [0.0, 0.0, 0.0]), 2, 4, 8, 1.0)
    assert st.tolist() == [1, 1, 1]
    assert parts(off, ent, 0) == [(0, 2, 8, 0.0)]
    assert parts(off, ent, 1) == [(1, 2, 2, 0.0)]
    assert parts(off, ent, 2) == [(0, 2, 0, 0.0)]


def test_part_of_a_node_when_cpus_are_short():
    # job 0 leaves 3 CPUs on node 0; job 1 (2 CPUs per GPU) gets one GPU there and three on node 1
    off, ent, st = orc.place(jobs([1, 4], [5, 8], [0.0, 0.0]), 2, 8, 8, 1.0)
    assert parts(off, ent, 1) == [(0, 1, 2, 0.0), (1, 3, 6, 0.0)]


def test_memory_binds():
    # 2.5 GiB per GPU, 6 GiB per node: two GPUs per node
    off, ent, st = orc.place(jobs([4], [0], [10.0]), 3, 4, 8, 6.0)
    assert parts(off, ent, 0) == [(0, 2, 0, 5.0), (1, 2, 0, 5.0)]


def test_a_job_that_does_not_fit_leaves_the_nodes_alone():
    off, ent, st = orc.place(jobs([3, 2, 1, 0], [0, 0, 0, 0], [0.0] * 4), 2, 2, 4, 1.0)
    assert st.tolist() == [1, 2, 1, 0]
    assert parts(off, ent, 0) == [(0, 2, 0, 0.0), (1, 1, 0, 0.0)]
    assert parts(off, ent, 1) == [] and parts(off, ent, 3) == []
    assert parts(off, ent, 2) == [(1, 1, 0, 0.0)]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_only_gpus_bind_jobs_lie_end_to_end(seed):
    """With CPUs and memory to spare, first fit in node order is the jobs laid end
    to end on the GPU slots: job j covers slots [S_j, S_j + g_j), S = prefix sum."""
    rng = np.random.default_rng(seed)
    n_nodes, gpn = 40, 8
    g = rng.choice([0, 0, 1, 2, 3, 4, 8, 12, 16, 24], size=60).astype(np.uint32)
    while g.sum() > n_nodes * gpn:
        g[rng.integers(len(g))] = 0
    c = (g * rng.integers(0, 5, size=len(g))).astype(np.uint32) + rng.integers(0, 3, size=len(g)).astype(np.uint32) * (g > 0)
    off, ent, st = orc.place(jobs(g, c, np.zeros(len(g))), n_nodes, gpn, 10 ** 6, 1.0)
    start = np.concatenate([[0], np.cumsum(g)[:-1]])
    for j in range(len(g)):
        if g[j] == 0:
            assert st[j] == 0 and off[j] == off[j + 1]
            continue
        slots = np.arange(start[j], start[j] + g[j])
        nodes, counts = np.unique(slots // gpn, return_counts=True)
        cum = np.cumsum(counts)
        cpus = (int(c[j]) * cum) // int(g[j])
        cpus = np.diff(np.concatenate([[0], cpus]))
        got = parts(off, ent, j)
        assert st[j] == 1
        assert [p[0] for p in got] == nodes.tolist() and [p[1] for p in got] == counts.tolist()
        assert [p[2] for p in got] == cpus.tolist()


def check_first_fit(assign, n_nodes, gpn, cpn, mpn, off, ent, st):
    """Replays a placement and verifies it part by part (a checker, not a second
    implementation of the search): capacities hold, every placed job has all its
    GPUs and CPUs, nodes ascend, no part could have been one GPU larger, a node
    that was passed over could not give a single GPU, and a job that was not
    placed could not have been."""
    f32 = np.float32
    freeG = np.full(n_nodes, gpn, np.int64)
    freeC = np.full(n_nodes, cpn, np.int64)
    freeM = np.full(n_nodes, mpn, np.float32)

    def fits(j, n, k):
        g, c, mem = int(assign["g"][j]), int(assign["c"][j]), f32(assign["mem_gb"][j])
        return k <= freeG[n] and -(-c * k // g) <= freeC[n] and f32(f32(mem * f32(k)) / f32(g)) <= freeM[n]

    for j in range(len(assign)):
        g = int(assign["g"][j])
        got = parts(off, ent, j)
        if g == 0:
            assert st[j] == 0 and not got
            continue
        if st[j] == 2:
            assert not got
            assert sum(max([k for k in range(0, min(g, int(freeG[n])) + 1) if k == 0 or fits(j, n, k)]) for n in range(n_nodes)) < g
            continue
        assert st[j] == 1
        assert sum(p[1] for p in got) == g and sum(p[2] for p in got) == int(assign["c"][j])
        assert [p[0] for p in got] == sorted(set(p[0] for p in got))
        used = {p[0]: p for p in got}
        left = g
        for n in range(got[-1][0] + 1):
            k = used[n][1] if n in used else 0
            assert k == 0 or fits(j, n, k)
            if k < left:                                   # more was wanted here
                assert not fits(j, n, k + 1)
            left -= k
        for n, k, c, m in got:
            assert m == f32(f32(f32(assign["mem_gb"][j]) * f32(k)) / f32(g))
            freeG[n] -= k
            freeC[n] -= c
            freeM[n] = f32(freeM[n] - f32(m))
        assert (freeG >= 0).all() and (freeC >= 0).all() and (freeM >= 0).all()


def random_round(seed):
    rng = np.random.default_rng(100 + seed)
    n_nodes, gpn, cpn, mpn = 24, 8, int(rng.choice([16, 32, 96])), float(rng.choice([64.0, 256.0, 1600.0]))
    J = 40
    g = rng.choice([0, 1, 1, 2, 2, 3, 4, 6, 8, 16], size=J).astype(np.uint32)
    c = (g * rng.choice([1, 2, 4, 8, 16], size=J)).astype(np.uint32)
    c[rng.random(J) < 0.3] += 1
    c[g == 0] = 0
    mem = (g * rng.choice([0.0, 8.0, 37.5, 120.0], size=J)).astype(np.float32)
    return jobs(g, c, mem), n_nodes, gpn, cpn, mpn


@pytest.mark.parametrize("seed", range(6))
def test_random_rounds_pass_the_checker(seed):
    a, n_nodes, gpn, cpn, mpn = random_round(seed)
    off, ent, st = orc.place(a, n_nodes, gpn, cpn, mpn)
    check_first_fit(a, n_nodes, gpn, cpn, mpn, off, ent, st)


def test_random_rounds_cover_skipped_nodes_splits_and_failures():
    failed = split = skipped = 0
    for seed in range(6):
        a, n_nodes, gpn, cpn, mpn = random_round(seed)
        off, ent, st = orc.place(a, n_nodes, gpn, cpn, mpn)
        failed += int((st == 2).sum())
        for j in range(len(a)):
            nodes = ent["node"][off[j]:off[j + 1]].astype(int)
            split += len(nodes) > 1
            skipped += len(nodes) > 1 and bool((np.diff(nodes) > 1).any())
    assert failed >= 3 and split >= 10 and skipped >= 2


def test_checker_rejects_a_wrong_placement():
    a = jobs([2, 2, 2], [8, 2, 0], [0.0, 0.0, 0.0])
    off, ent, st = orc.place(a, 2, 4, 8, 1.0)
    check_first_fit(a, 2, 4, 8, 1.0, off, ent, st)
    bad = ent.copy()
    bad[2]["node"] = 1                                     # job 2 skips the hole on node 0
    with pytest.raises(AssertionError):
        check_first_fit(a, 2, 4, 8, 1.0, off, bad, st)
