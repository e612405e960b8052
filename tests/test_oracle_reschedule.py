"""Pins of the oracle's Schedule loop (Sec. 5.2, Algorithm 1: privileged jobs
first, the others by slope; ScheduleJob takes what is free and shrinks the
job with the lowest slope while the new job's slope is higher or the new job
is below its minimum demand).  Hand cases for every rule, the exhaustive
optimum and the from-scratch greedy on concave curves, invariants on random
rounds - and the measured answer to whether the from-scratch greedy is where
this loop stops (it is on concave curves, it is not in general)."""
import itertools
import math

import numpy as np
import pytest

import workloads


def table_for(orc, J, g_max):
    lcm = 1
    for v in range(1, g_max + 1):
        lcm = lcm * v // math.gcd(lcm, v)
    ints = np.tile(np.array([[1, lcm, 1]], np.uint32), (J, 1))
    tb = orc.enumerate_plans(ints, workloads.Bounds(g_max=g_max, tp_max=1))
    assert tb.seg_g.tolist() == list(range(1, g_max + 1)) * J        # every count 1..g_max is a segment
    return tb


def loop(orc, pts, G, hold, floors=None, ref=None, C=10 ** 6, host=1e9, state=None, cpu=None):
    """pts[j][g-1] = best throughput with g GPUs (0 = not a valid count); hold[j] = GPUs held now (0 = queued);
    floors[j] = minimum GPUs (0 = none).  cpu = (levels, mode, values[j][level][g-1], held level[j], floor level[j])."""
    J, g_max = len(pts), len(pts[0])
    tb = table_for(orc, J, g_max)
    if cpu is None:
        grid = workloads.Grid(np.array([1], np.uint32), 0, np.array([1.0], np.float32), 0)
        bt = np.array(pts, np.float32).reshape(J, 1, g_max)
        cur_c, floor_c = np.zeros(J, np.uint32), np.zeros(J, np.uint32)
    else:
        levels, mode, vals, cur_c, floor_c = cpu
        grid = workloads.Grid(np.array(levels, np.uint32), mode, np.array([1.0], np.float32), 0)
        bt = np.array(vals, np.float32)
    bp = np.arange(bt.size, dtype=np.uint32)
    bp[bt.reshape(-1) == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, bt.reshape(-1), bp)
    ref = np.ones(J, np.float32) if ref is None else np.asarray(ref, np.float32)
    floors = [0] * J if floors is None else floors
    a, total, moves = orc.reschedule(ref, tb, grid, workloads.Cluster(G, C, host), bt.reshape(-1), bp, ct,
                                     [h - 1 for h in hold], cur_c, [f - 1 for f in floors], floor_c, state=state)
    return a, total, moves


STEEP, FLAT = [1.0, 1.9, 2.7, 3.4], [1.0, 1.1, 1.15, 1.18]


def test_a_higher_slope_takes_from_the_lowest():
    import oracle as orc
    # the flat job holds all four GPUs, the steep one arrives: it takes them one by one while its gain per GPU
    # (1.0, 0.9, 0.8) exceeds what the flat job loses (0.03, 0.05, 0.1); the fourth would cost the flat job 1.0 for 0.7
    a, total, moves = loop(orc, [FLAT, STEEP], 4, [4, 0])
    assert a["g"].tolist() == [1, 3] and moves == 3 and total == pytest.approx(1.0 + 2.7)
    # the other way round the result is the same split
    a, _, moves = loop(orc, [FLAT, STEEP], 4, [0, 4])
    assert a["g"].tolist() == [1, 3] and moves == 1
    # a running job keeps what it holds when nobody's slope is higher: 5 - 3 = 2 per GPU against the newcomer's 1
    a, _, moves = loop(orc, [[3.0, 5.0], [1.0, 1.5]], 2, [2, 0])
    assert a["g"].tolist() == [2, 0] and moves == 0
    # equal slopes do not move anything either (the rule asks for a higher one)
    a, _, moves = loop(orc, [[3.0, 4.0], [1.0, 1.5]], 2, [2, 0])
    assert a["g"].tolist() == [2, 0] and moves == 0


def test_a_job_below_its_minimum_takes_at_a_loss():
    import oracle as orc
    # the newcomer is guaranteed one GPU: the running job gives it although the total falls from 5 to 4
    a, total, _ = loop(orc, [[3.0, 5.0], [1.0, 1.5]], 2, [2, 0], floors=[0, 1])
    assert a["g"].tolist() == [1, 1] and total == pytest.approx(4.0)
    # ... but not from a job that is at its own minimum
    a, _, moves = loop(orc, [[3.0, 5.0], [1.0, 1.5]], 2, [2, 0], floors=[2, 1])
    assert a["g"].tolist() == [2, 0] and moves == 0
    # ... and beyond its minimum it competes by slope like anyone else: 0.5 < 2
    a, _, _ = loop(orc, [[3.0, 5.0, 7.0], [1.0, 1.5, 2.0]], 3, [3, 0], floors=[0, 1])
    assert a["g"].tolist() == [2, 1]
    # a best-effort job can be preempted altogether, a guaranteed one stops at its minimum
    a, _, _ = loop(orc, [[1.0], [0.5]], 1, [1, 0], floors=[0, 1])
    assert a["g"].tolist() == [0, 1]
    # two GPUs are the newcomer's minimum and only one can be had: it waits and nothing moves
    a, _, moves = loop(orc, [[3.0, 5.0], [1.0, 1.5]], 2, [2, 0], floors=[1, 2])
    assert a["g"].tolist() == [2, 0] and moves == 0
    # privileged jobs go first, in job order, whatever their slopes: job 2 finds the last GPU gone
    a, _, _ = loop(orc, [[0.1], [5.0], [9.0]], 2, [0, 0, 0], floors=[1, 1, 1])
    assert a["g"].tolist() == [1, 1, 0]


def test_the_unit_is_the_distance_to_the_next_useful_amount():
    import oracle as orc
    four = [1.0, 0.0, 0.0, 4.0]                      # valid on 1 and 4 GPUs only: the curve is flat in between
    # job 0 needs three more: one is free, one the other job gives for 0.5 < 1, its last would cost 1.0, not less
    # than job 0 gains per GPU: the whole step is taken back
    a, _, moves = loop(orc, [four, [1.0, 1.5, 0, 0]], 4, [1, 2])
    assert a["g"].tolist() == [1, 2] and moves == 0
    # with one more free GPU the step goes through
    a, _, moves = loop(orc, [four, [1.0, 1.5, 0, 0]], 5, [1, 2])
    assert a["g"].tolist() == [4, 1] and moves == 1
    # a job that holds more than it uses gives the surplus first, at no loss
    a, _, _ = loop(orc, [[1.0, 2.0, 0.0, 0.0], [0.2, 0, 0, 0], [1.0, 1.9, 0, 0]], 4, [3, 1, 0])
    assert a["g"].tolist() == [2, 0, 2]              # one surplus GPU of job 0, then job 1's only one (0.2 < 0.9)
    # a step down can free more than is needed: job 1 steps from 3 to 1 GPU (slope 0.6 < 1) and loses 1.2, more than
    # job 0 gains with its one GPU: not taken
    a, _, moves = loop(orc, [[1.0, 0, 0], [2.0, 0.0, 3.2]], 3, [0, 3])
    assert a["g"].tolist() == [0, 3] and moves == 0
    a, _, moves = loop(orc, [[1.3, 0, 0], [2.0, 0.0, 3.2]], 3, [0, 3])
    assert a["g"].tolist() == [1, 1] and moves == 1


def test_the_lowest_slope_is_per_unit_given():
    import oracle as orc
    # all five GPUs are held: job 0 would give two for 1.0 (0.5 each), job 1 one for 0.8.  The lowest slope is job 0's;
    # the newcomer's gain of 0.9 does not cover the 1.0 job 0 would lose: nothing moves (job 1's GPU is never asked for)
    a, _, moves = loop(orc, [[2.0, 0.0, 3.0], [1.0, 1.8, 0.0], [0.9, 0.0, 0.0]], 5, [3, 2, 0])
    assert a["g"].tolist() == [3, 2, 0] and moves == 0
    # with a gain of 1.1 it does, and the second freed GPU stays free (nobody has a use for it)
    a, _, moves = loop(orc, [[2.0, 0.0, 3.0], [1.0, 1.8, 0.0], [1.1, 0.0, 0.0]], 5, [3, 2, 0])
    assert a["g"].tolist() == [1, 2, 1] and moves == 1
    # a victim stops at its minimum: its curve says one GPU is as good as two (1.0 against 0.9), it is guaranteed
    # two, so it gives two of its four, not three
    a, _, moves = loop(orc, [[1.0, 0.9, 0.0, 4.0], [0.5, 0.6, 0.0, 0.0]], 4, [4, 0], floors=[2, 2])
    assert a["g"].tolist() == [2, 2] and a["thr"].tolist() == [np.float32(0.9), np.float32(0.6)]
    assert moves == 1                                         # (it did not give three and take one back)
    # the same per CPU: levels of 1 and 2 CPUs per GPU, all 7 CPUs held; job 0 (two GPUs) would give two CPUs for 1.0,
    # job 1 one for 0.8; job 2's extra CPU is worth 0.9
    vals = [[[0.0, 3.0], [0.0, 4.0]], [[1.0, 0.0], [1.8, 0.0]], [[1.0, 0.0], [1.9, 0.0]]]
    cpu = ([1, 2], 1, vals, np.array([1, 1, 0], np.uint32), np.zeros(3, np.uint32))
    a, _, moves = loop(orc, [[0.0, 3.0], [1.0, 0.0], [1.0, 0.0]], 4, [2, 1, 1], C=7, cpu=cpu)
    assert a["c"].tolist() == [4, 2, 1] and moves == 0
    vals[2][1][0] = 2.1                                       # worth 1.1: job 0 steps down, one CPU stays free
    a, _, moves = loop(orc, [[0.0, 3.0], [1.0, 0.0], [1.0, 0.0]], 4, [2, 1, 1], C=7, cpu=cpu)
    assert a["c"].tolist() == [2, 2, 2] and moves == 1


def test_jobs_are_taken_by_slope():
    import oracle as orc
    # the order decides here: job 0 (slope 1.0 for its first GPU) goes first and ends with both GPUs; job 1's best step
    # (both GPUs, 0.95 each) would need job 0's first GPU, worth 1.0.  Served the other way round, job 1 would keep both
    a, total, _ = loop(orc, [[1.0, 1.5], [0.9, 1.9]], 2, [0, 0])
    assert a["g"].tolist() == [2, 0] and total == pytest.approx(1.5)
    # one free GPU, two queued jobs: the steeper one is served first and the other cannot take it away
    a, _, _ = loop(orc, [[1.0], [2.0]], 1, [0, 0])
    assert a["g"].tolist() == [0, 1]
    # the reference throughput normalises the slopes
    a, _, _ = loop(orc, [[1.0], [2.0]], 1, [0, 0], ref=[0.25, 1.0])
    assert a["g"].tolist() == [1, 0]
    # a job that takes no part neither gets nor gives
    a, _, _ = loop(orc, [[1.0], [2.0]], 1, [0, 0], state=[0, 1])
    assert a["g"].tolist() == [1, 0]


def test_a_job_that_keeps_what_it_holds():
    import oracle as orc
    # state 2: the flat job keeps its four GPUs whatever the newcomer's slope (without the state it would give three)
    a, _, moves = loop(orc, [FLAT, STEEP], 4, [4, 0], state=[2, 0])
    assert a["g"].tolist() == [4, 0] and moves == 0
    # ... it does not grow either, with a GPU free and a step worth taking
    a, _, moves = loop(orc, [STEEP, FLAT], 4, [1, 0], state=[2, 0])
    assert a["g"].tolist() == [1, 3] and moves == 3
    # ... what it holds is not there for the others: three of four GPUs held, one left
    a, _, _ = loop(orc, [FLAT, STEEP], 4, [3, 0], state=[2, 0])
    assert a["g"].tolist() == [3, 1]
    # ... not even for a job below its minimum
    a, _, _ = loop(orc, [FLAT, STEEP], 4, [4, 0], floors=[0, 2], state=[2, 0])
    assert a["g"].tolist() == [4, 0]
    # any other state byte: the job takes no part and holds nothing
    a, _, _ = loop(orc, [FLAT, STEEP], 4, [4, 0], state=[3, 0])
    assert a["g"].tolist() == [0, 4]


def test_cpus_after_gpus():
    import oracle as orc
    # one GPU each; CPU levels 1, 2, 4 for the job; values [job][level][g-1]
    vals = [[[1.0], [1.5], [1.6]], [[1.0], [3.0], [3.2]]]
    cpu = ([1, 2, 4], 0, vals, np.array([0, 0], np.uint32), np.zeros(2, np.uint32))
    # 5 CPUs: both start on 1; job 1's second CPU is worth 2, job 0's 0.5, then one CPU is left and level 4 needs two
    a, total, _ = loop(orc, [[1.0], [1.0]], 2, [1, 1], C=5, cpu=cpu)
    assert a["c"].tolist() == [2, 2] and a["thr"].tolist() == [1.5, 3.0]
    # job 0 holds level 4 (4 CPUs) of 5, job 1 level 1: job 1's step to 2 CPUs (slope 2) takes from job 0, whose
    # fourth and third CPU are worth 0.05 each
    cpu = ([1, 2, 4], 0, vals, np.array([2, 0], np.uint32), np.zeros(2, np.uint32))
    a, _, _ = loop(orc, [[1.0], [1.0]], 2, [1, 1], C=5, cpu=cpu)
    assert a["c"].tolist() == [2, 2]
    # a GPU step must find its CPUs: per-GPU level of 2 CPUs, 3 CPUs in all: the second GPU is out of reach
    per_gpu = ([2], 1, [[[1.0, 2.0]]], np.zeros(1, np.uint32), np.zeros(1, np.uint32))
    a, _, _ = loop(orc, [[1.0, 2.0]], 2, [0], C=3, cpu=per_gpu)
    assert a["g"].tolist() == [1] and a["c"].tolist() == [2]


def exhaustive_best(values, G):
    J = len(values)
    best = 0.0
    for alloc in itertools.product(range(G + 1), repeat=J):
        if sum(alloc) <= G:
            best = max(best, sum(values[j][alloc[j]] for j in range(J)))
    return best


def test_concave_curves_end_at_the_optimum_and_at_the_greedy():
    """Where the from-scratch greedy is provably where unit transfers stop (concave curves), the loop agrees with it
    from an empty cluster and from any starting split, and both reach the exhaustive optimum."""
    import oracle as orc
    from test_oracle_selection import run_greedy_on
    rng = np.random.default_rng(41)
    for trial in range(25):
        J, G = 4, 7
        gains = np.sort(rng.uniform(0.1, 2.0, size=(J, G)).astype(np.float32), axis=1)[:, ::-1]
        pts = np.cumsum(gains.astype(np.float64), axis=1).astype(np.float32).tolist()
        g_assign, g_total, _ = run_greedy_on(orc, pts, G)
        opt = exhaustive_best([[0.0] + p for p in pts], G)
        assert g_total == pytest.approx(opt, rel=1e-6)
        for start in range(3):
            hold = [0] * J
            if start:
                cuts = np.sort(rng.integers(0, G + 1, size=J - 1))
                hold = np.diff(np.concatenate([[0], cuts, [G]])).astype(int).tolist()
            a, total, _ = loop(orc, pts, G, hold)
            assert total == pytest.approx(opt, rel=1e-6), (trial, start)
            assert a["g"].tolist() == g_assign["g"].tolist(), (trial, start)


def random_case(rng):
    J, G = int(rng.integers(2, 7)), int(rng.integers(3, 17))
    pts, floors = [], []
    for _ in range(J):
        valid = sorted(set([1] + rng.choice([1, 2, 3, 4, 6, 8, 12, 16], int(rng.integers(1, 5))).tolist()))
        valid = [x for x in valid if x <= G]
        v = np.cumsum(np.sort(rng.uniform(0.2, 2.0, len(valid)))[::-1] * rng.uniform(0.5, 1.5, len(valid)))
        row = np.zeros(G, np.float32)
        row[np.array(valid) - 1] = v
        pts.append(row.tolist())
        floors.append(int(rng.choice(valid)) if rng.uniform() < 0.25 else 0)
    return J, G, pts, floors


def test_invariants_on_random_rounds():
    import oracle as orc
    rng = np.random.default_rng(77)
    n = 0
    for trial in range(300):
        J, G, pts, floors = random_case(rng)
        if sum(floors) > G:
            continue
        # a starting state: some jobs hold a valid count (at or above their floor), within the cluster
        hold = [0] * J
        left = G
        for j in rng.permutation(J).tolist():
            if rng.uniform() < 0.5:
                ok = [g + 1 for g in range(G) if pts[j][g] > 0 and g + 1 <= left and g + 1 >= floors[j]]
                if ok:
                    hold[j] = int(rng.choice(ok))
                    left -= hold[j]
        state = (rng.uniform(size=J) < 0.15).astype(np.uint8)
        hold = [0 if state[j] else hold[j] for j in range(J)]
        a, total, moves = loop(orc, pts, G, hold, floors=floors, state=state)
        g = a["g"].astype(int)
        assert g.sum() <= G
        curve = [np.maximum.accumulate(np.array([0.0] + p)) for p in pts]
        before = sum(curve[j][hold[j]] for j in range(J))
        privileged = False
        for j in range(J):
            if state[j]:
                assert g[j] == 0
                continue
            if g[j]:
                assert pts[j][g[j] - 1] > 0 or curve[j][g[j]] == curve[j][g[j] - 1]      # a valid count (or a held surplus)
            if floors[j] and hold[j] >= floors[j]:
                assert g[j] >= floors[j]                      # never shrunk below its minimum
            if floors[j] and hold[j] < floors[j]:
                privileged = True
                assert g[j] >= floors[j] or g[j] == hold[j]   # reaches its minimum or stays as it was
        if not privileged:
            assert total >= before * (1 - 1e-6)               # every committed step raised the total
        n += 1
    assert n > 200


def test_the_from_scratch_greedy_is_not_where_the_loop_stops_in_general():
    """On curves with flats (valid GPU counts only) the loop from an empty cluster and the from-scratch greedy part
    ways in a good share of the rounds, in either direction: the greedy interleaves the jobs' steps by slope and never
    takes anything back, the loop serves the jobs one after the other and shrinks.  The counts are what this seeded
    sample gives; they are here so that a change of either rule shows."""
    import oracle as orc
    from test_oracle_selection import run_greedy_on
    rng = np.random.default_rng(5)
    same = better = worse = n = 0
    for trial in range(300):
        J, G, pts, floors = random_case(rng)
        g_assign, g_total, _ = run_greedy_on(orc, pts, G)
        a, total, _ = loop(orc, pts, G, [0] * J)
        n += 1
        same += a["g"].tolist() == g_assign["g"].tolist()
        better += total > g_total * (1 + 1e-6)
        worse += total < g_total * (1 - 1e-6)
    print(f"{n} rounds: same allocation {same}, loop's total higher {better}, lower {worse}")
    assert same < n and better + worse > 0
    assert same > 0.5 * n
