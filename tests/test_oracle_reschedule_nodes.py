"""Pins of the oracle's Schedule loop with the node-by-node search of ScheduleJob
(Sec. 5.2, Algorithm 1: on each node the job takes what is free and then shrinks
the job with the lowest slope among those on that node).  The loop over the
cluster's totals is its special case of one node that holds everything; hand
cases pin what the nodes add: the order free -> victims of this node -> next
node, victims restricted to the node, which parts a shrunk job gives up, CPUs
that come with a GPU on its node, CPU steps on every node of a job, roll-back,
memory per node, and the states that are no placement."""
import numpy as np
import pytest

import workloads
from test_oracle_reschedule import random_case, table_for

STEEP, FLAT = [1.0, 1.9, 2.7, 3.4], [1.0, 1.1, 1.15, 1.18]


def first_fit(free_g, free_c, g, per_gpu):
    """Parts {node: k} for g GPUs with per_gpu CPUs each, or None; books them."""
    parts, lack = {}, g
    fg, fc = list(free_g), list(free_c)
    for n in range(len(fg)):
        k = min(lack, fg[n], fc[n] // per_gpu)
        if k:
            parts[n] = k
            fg[n] -= k
            fc[n] -= k * per_gpu
            lack -= k
    if lack:
        return None
    free_g[:], free_c[:] = fg, fc
    return parts


def nodes_loop(orc, vals, nodes, where, levels=(1,), cur_c=None, floors=None, floor_c=None, ref=None, tiers=(1.0,),
               mem_mode=0, state=None, prev="from where"):
    """vals[j][level][tier][g-1] (or [j][g-1] for one level and one tier) = best throughput, 0 = no plan;
    nodes = (n, GPUs, CPUs, GiB) per node; where[j] = {node: GPUs held there}."""
    vals = np.array(vals, np.float32)
    J, g_max = vals.shape[0], vals.shape[-1]
    if vals.ndim == 2:
        vals = vals.reshape(J, 1, 1, g_max)
    assert vals.shape == (J, len(levels), len(tiers), g_max)
    tb = table_for(orc, J, g_max)
    grid = workloads.Grid(np.array(levels, np.uint32), 1, np.array(tiers, np.float32), mem_mode)
    bt = vals.reshape(-1)
    bp = np.arange(bt.size, dtype=np.uint32)
    bp[bt == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, bt, bp)
    cur_c = np.zeros(J, np.uint32) if cur_c is None else np.asarray(cur_c, np.uint32)
    hold = [sum(w.values()) for w in where]
    if prev == "from where":
        off, ent = [0], []
        for j, w in enumerate(where):
            for n in sorted(w):
                ent.append((n, w[n], levels[int(cur_c[j])] * w[n], 0.0))
            off.append(len(ent))
        prev = (np.array(off, np.uint32), np.array(ent, orc.PLACE_DTYPE) if ent else np.zeros(0, orc.PLACE_DTYPE))
    ref = np.ones(J, np.float32) if ref is None else np.asarray(ref, np.float32)
    floors = [0] * J if floors is None else floors
    floor_c = np.zeros(J, np.uint32) if floor_c is None else np.asarray(floor_c, np.uint32)
    res = orc.reschedule_nodes(ref, tb, grid, *nodes, bt, bp, ct, [h - 1 for h in hold], cur_c, prev,
                               [f - 1 for f in floors], floor_c, state=state)
    if res is None:
        return None
    a, off, ent, total, moves = res
    parts = [{int(e["node"]): int(e["g"]) for e in ent[off[j]:off[j + 1]]} for j in range(J)]
    for j in range(J):                                       # the records and the parts say the same
        assert sum(parts[j].values()) == a["g"][j]
        assert sum(int(e["c"]) for e in ent[off[j]:off[j + 1]]) == a["c"][j]
        assert [int(e["node"]) for e in ent[off[j]:off[j + 1]]] == sorted(parts[j])
    return a, parts, total, moves


def test_free_first_then_the_jobs_of_this_node_then_the_next_node():
    import oracle as orc
    # two nodes of two GPUs; the flat job fills node 0, node 1 is empty, the steep job arrives.  Its first GPU comes
    # from the flat job (0.1 lost for 1.0) although node 1 is free: the search is at node 0 first.  Its second would
    # cost the flat job its last GPU (1.0 for 0.9): not permitted, so the search goes on to node 1.
    a, parts, total, moves = nodes_loop(orc, [FLAT, STEEP], (2, 2, 99, 1e6), [{0: 2}, {}])
    assert parts == [{0: 1}, {0: 1, 1: 2}] and moves == 3 and total == pytest.approx(1.0 + 2.7)
    # with the empty node first its two GPUs are taken first; the third (0.8) is still worth the flat job's second (0.1)
    a, parts, _, _ = nodes_loop(orc, [FLAT, STEEP], (2, 2, 99, 1e6), [{1: 2}, {}])
    assert parts == [{1: 1}, {0: 2, 1: 1}]


def test_the_job_to_shrink_is_one_of_this_node():
    import oracle as orc
    # job 1 has the lowest slope of the cluster (0.2) but sits on node 1; the newcomer (0.6) meets job 0 (0.5) on node 0
    vals = [[0.5], [0.2], [0.6]]
    a, parts, _, moves = nodes_loop(orc, vals, (2, 1, 99, 1e6), [{0: 1}, {1: 1}, {}])
    # ... and takes its GPU; job 0, queued now, finds job 1 on node 1 when its own turn comes (0.5 against 0.2)
    assert parts == [{1: 1}, {}, {0: 1}] and moves == 2
    # the loop over totals takes from the lowest slope anywhere
    tb = table_for(orc, 3, 1)
    grid = workloads.Grid(np.array([1], np.uint32), 1, np.array([1.0], np.float32), 0)
    bt = np.array(vals, np.float32).reshape(-1)
    bp = np.arange(3, dtype=np.uint32)
    ct, _, _ = orc.curves(tb, grid, bt, bp)
    t, _, _ = orc.reschedule(np.ones(3, np.float32), tb, grid, workloads.Cluster(2, 99, 1e6), bt, bp, ct, [0, 0, -1],
                             np.zeros(3, np.uint32))
    assert t["g"].tolist() == [1, 0, 1]
    # a job of this node that may not be shrunk ends the search here, whatever sits elsewhere
    a, parts, _, moves = nodes_loop(orc, [[0.7], [0.2], [0.6]], (2, 1, 99, 1e6), [{0: 1}, {1: 1}, {}])
    assert parts == [{0: 1}, {}, {1: 1}] and moves == 1       # node 0: 0.7 stays; node 1: 0.2 goes


def test_a_job_that_keeps_what_it_holds_is_not_asked():
    import oracle as orc
    # the flat job fills node 0 and must not be touched (state 2): the newcomer takes the two GPUs of node 1 and stops
    a, parts, _, moves = nodes_loop(orc, [FLAT, STEEP], (2, 2, 99, 1e6), [{0: 2}, {}], state=[2, 0])
    assert parts == [{0: 2}, {1: 2}] and moves == 2


def test_a_shrunk_job_gives_this_node_first_then_its_last_parts():
    import oracle as orc
    # job 0 runs on 4 GPUs over three nodes and has plans for 1 and 4 only: it can only give three at once (0.3 lost)
    wide = [1.0, 0.0, 0.0, 1.3]
    a, parts, _, _ = nodes_loop(orc, [wide, STEEP], (3, 2, 99, 1e6), [{0: 1, 1: 2, 2: 1}, {}])
    # the newcomer's first GPU is the free one of node 0; its second makes job 0 give its GPU there, the one on node 2
    # and one of node 1 (last part first); the newcomer then finds its third on node 1 and its fourth on node 2
    assert parts == [{1: 1}, {0: 2, 1: 1, 2: 1}]
    assert a["thr"].tolist() == pytest.approx([1.0, 3.4])


def test_a_gpu_comes_with_its_cpus_on_its_node():
    import oracle as orc
    # 2 CPUs per GPU, 3 CPUs per node: a node's second GPU has no CPUs, so the job spreads over both nodes
    a, parts, _, _ = nodes_loop(orc, [[1.0, 2.0]], (2, 2, 3, 1e6), [{}], levels=(2,))
    assert parts == [{0: 1, 1: 1}] and a["c"].tolist() == [4]
    # a shrunk job frees its CPUs with its GPUs.  The flat job holds both GPUs of the node at 1 CPU each; the newcomer is
    # guaranteed one GPU at 2 CPUs per GPU.  With 3 CPUs on the node one GPU of the flat job is enough (1 free + 1 freed)
    vals = [[[FLAT[:2]], [FLAT[:2]]], [[[1.0, 0]], [[1.0, 0]]]]
    a, parts, _, _ = nodes_loop(orc, vals, (1, 2, 3, 1e6), [{0: 2}, {}], levels=(1, 2), floors=[0, 1], floor_c=[0, 1])
    assert parts == [{0: 1}, {0: 1}] and a["c"].tolist() == [1, 2]
    # with 2 CPUs on the node the freed GPU has only one CPU: the flat job is asked again and leaves
    a, parts, _, _ = nodes_loop(orc, vals, (1, 2, 2, 1e6), [{0: 2}, {}], levels=(1, 2), floors=[0, 1], floor_c=[0, 1])
    assert parts == [{}, {0: 1}] and a["c"].tolist() == [0, 2]


def test_a_cpu_step_is_taken_on_every_node_of_the_job():
    import oracle as orc
    # levels 1 and 2 CPUs per GPU, 3 CPUs per node.  Job 0 has a GPU on each node at level 0; job 1 has one on node 1
    # at level 1, so node 1 has no CPU free.  Job 0's step to level 1 is worth (3 - 2) / 2 = 0.5 per CPU.
    def vals(job1_top):
        return [[[[0, 2.0]], [[0, 3.0]]], [[[1.0, 0]], [[job1_top, 0]]]]
    where = [{0: 1, 1: 1}, {1: 1}]
    # job 1 would lose 0.8 for its CPU: it stays, and job 0 stays at level 0 on both nodes (node 0's CPUs are put back)
    a, parts, _, moves = nodes_loop(orc, vals(1.8), (2, 2, 3, 1e6), where, levels=(1, 2), cur_c=[0, 1])
    assert a["c"].tolist() == [2, 2] and moves == 0
    # job 1 would lose 0.2: it gives its level, job 0 goes up on both nodes
    a, parts, _, moves = nodes_loop(orc, vals(1.2), (2, 2, 3, 1e6), where, levels=(1, 2), cur_c=[0, 1])
    assert a["c"].tolist() == [4, 1] and a["thr"].tolist() == [3.0, 1.0] and moves == 1


def test_a_job_that_gives_a_cpu_level_gives_it_on_all_its_nodes():
    import oracle as orc
    # both jobs have a GPU on each node; job 1 runs at 2 CPUs per GPU and fills the nodes (3 CPUs each).  Job 0's step
    # to 2 CPUs per GPU meets it on node 0; the level it gives there also frees a CPU on node 1, where job 0 then
    # needs nobody (and nobody would be left to ask: job 1 is at the lowest level by then)
    vals = [[[[0, 2.0]], [[0, 3.0]]], [[[0, 1.0]], [[0, 1.4]]]]
    a, _, total, moves = nodes_loop(orc, vals, (2, 2, 3, 1e6), [{0: 1, 1: 1}, {0: 1, 1: 1}], levels=(1, 2), cur_c=[0, 1])
    assert a["c"].tolist() == [4, 2] and moves == 1 and total == pytest.approx(4.0)
    # a CPU step is weighed like a GPU step: job 1 holds three GPUs at 2 CPUs each and would give three CPUs (1.2 lost,
    # 0.4 each) where job 0 needs one (0.5 gained): permitted by slope, taken back by the sum
    def vals(top):
        return [[[[1.0, 0, 0]], [[1.5, 0, 0]]], [[[0, 0, 2.0]], [[0, 0, top]]]]
    a, _, _, moves = nodes_loop(orc, vals(3.2), (1, 4, 7, 1e6), [{0: 1}, {0: 3}], levels=(1, 2), cur_c=[0, 1])
    assert a["c"].tolist() == [1, 6] and moves == 0
    a, _, _, moves = nodes_loop(orc, vals(2.3), (1, 4, 7, 1e6), [{0: 1}, {0: 3}], levels=(1, 2), cur_c=[0, 1])
    assert a["c"].tolist() == [2, 3] and moves == 1


def test_a_step_that_costs_more_than_it_brings_is_taken_back():
    import oracle as orc
    # the newcomer needs two GPUs at once (1.5, 0.75 each); the only job on the node can give three at once (2.1 lost,
    # 0.7 each): permitted by slope, but the newcomer gains less than the other loses
    a, parts, total, moves = nodes_loop(orc, [[0.5, 0, 0, 2.6], [0, 1.5, 0, 0]], (1, 4, 99, 1e6), [{0: 4}, {}])
    assert parts == [{0: 4}, {}] and moves == 0 and total == pytest.approx(2.6)
    # one GPU fewer to lose and it goes through
    a, parts, _, moves = nodes_loop(orc, [[1.2, 0, 0, 2.6], [0, 1.5, 0, 0]], (1, 4, 99, 1e6), [{0: 4}, {}])
    assert parts == [{0: 1}, {0: 2}] and moves == 1


def test_a_job_below_its_minimum_takes_at_a_loss_on_the_node():
    import oracle as orc
    a, parts, _, _ = nodes_loop(orc, [[3.0, 5.0], [1.0, 1.5]], (1, 2, 99, 1e6), [{0: 2}, {}], floors=[0, 1])
    assert parts == [{0: 1}, {0: 1}]
    # a step to a floor with a higher CPU level raises the parts the job has: their CPUs must be free where they are
    vals = [[[[1.0, 0]], [[1.0, 2.0]]], [[[1.0, 0]], [[1.0, 0]]]]
    where = [{0: 1}, {0: 1}]
    a, parts, _, _ = nodes_loop(orc, vals, (2, 2, 3, 1e6), where, levels=(1, 2), cur_c=[0, 0], floors=[2, 0], floor_c=[1, 0])
    assert parts[0] == {0: 1, 1: 1} and a["c"].tolist()[0] == 4          # node 0: 1 + 1 used, one more is free
    a, parts, _, _ = nodes_loop(orc, vals, (2, 2, 3, 1e6), where, levels=(1, 2), cur_c=[0, 1], floors=[2, 0], floor_c=[1, 0])
    assert parts[0] == {0: 1} and a["c"].tolist()[0] == 1                # node 0: 1 + 2 used, nothing free: it stays


def test_memory_is_paid_per_node():
    import oracle as orc
    # tiers 0 and 64 GiB per job, 40 GiB per node.  Job 0 on two nodes pays 32 on each for the upper tier; job 1 on
    # node 0 then cannot pay 64 and keeps the lower tier; job 2 has no plan without memory and is dropped
    vals = [[[[0, 1.0], [0, 2.0]]], [[[1.0, 0], [3.0, 0]]], [[[0, 0], [1.0, 0]]]]
    a, parts, total, _ = nodes_loop(orc, vals, (2, 2, 99, 40.0), [{0: 1, 1: 1}, {0: 1}, {1: 1}], tiers=(0.0, 64.0))
    assert a["mem_gb"].tolist() == [64.0, 0.0, 0.0] and a["thr"].tolist() == [2.0, 1.0, 0.0]
    assert parts == [{0: 1, 1: 1}, {0: 1}, {}] and a["g"].tolist() == [2, 1, 0]
    # with 64 GiB per GPU the parts of a job pay 64 each
    a, _, _, _ = nodes_loop(orc, vals, (2, 2, 99, 100.0), [{0: 1, 1: 1}, {0: 1}, {1: 1}], tiers=(0.0, 64.0), mem_mode=1)
    assert a["mem_gb"].tolist() == [128.0, 0.0, 0.0]


def test_states_that_are_no_placement():
    import oracle as orc
    P = orc.PLACE_DTYPE
    good = (np.array([0, 2, 2], np.uint32), np.array([(0, 1, 1, 0), (1, 1, 1, 0)], P))
    assert nodes_loop(orc, [FLAT, STEEP], (2, 2, 99, 1e6), [{0: 1, 1: 1}, {}], prev=good) is not None

    def bad(entries, off=(0, 2, 2)):
        prev = (np.array(off, np.uint32), np.array(entries, P))
        return nodes_loop(orc, [FLAT, STEEP], (2, 2, 99, 1e6), [{0: 1, 1: 1}, {}], prev=prev)

    assert bad([(0, 1, 1, 0), (1, 2, 2, 0)]) is None          # three GPUs for a job that holds two
    assert bad([(0, 1, 1, 0), (2, 1, 1, 0)]) is None          # a node the cluster does not have
    assert bad([(1, 1, 1, 0), (0, 1, 1, 0)]) is None          # parts out of order
    assert bad([(0, 1, 1, 0), (0, 1, 1, 0)]) is None          # two parts on one node
    assert bad([(0, 1, 2, 0), (1, 1, 1, 0)]) is None          # CPUs that are not level * GPUs
    assert bad([(0, 2, 2, 0)], off=(0, 1, 1)) is not None     # (the same amount on one node is a placement)
    assert nodes_loop(orc, [FLAT, STEEP], (2, 2, 99, 1e6), [{0: 1, 1: 1}, {}], prev=None) is None
    # two jobs that together hold more than the node has
    over = (np.array([0, 1, 2], np.uint32), np.array([(0, 2, 2, 0), (0, 1, 1, 0)], P))
    assert nodes_loop(orc, [FLAT, STEEP], (2, 2, 99, 1e6), [{0: 2}, {0: 1}], prev=over) is None


def draw_state(rng, pts, floors, n_nodes, gpn, cpn, levels):
    """Some jobs hold a valid count at or above their floor, laid out by first fit."""
    J, G = len(pts), len(pts[0])
    free_g, free_c = [gpn] * n_nodes, [cpn] * n_nodes
    where, cur_c = [{} for _ in range(J)], np.zeros(J, np.uint32)
    for j in rng.permutation(J).tolist():
        if rng.uniform() < 0.6:
            ok = [g + 1 for g in range(G) if pts[j][g] > 0 and g + 1 >= floors[j]]
            if ok:
                lvl = int(rng.integers(0, len(levels)))
                parts = first_fit(free_g, free_c, int(rng.choice(ok)), levels[lvl])
                if parts:
                    where[j], cur_c[j] = parts, lvl
    return where, cur_c


def level_values(rng, pts, levels):
    """[job][level][tier 0][g-1]: more CPUs never hurt, sometimes help."""
    out = []
    for row in pts:
        rows, cur = [], np.array(row, np.float32)
        for _ in levels:
            rows.append([cur.tolist()])
            cur = (cur * np.float32(rng.choice([1.0, 1.0, 1.1, 1.4]))).astype(np.float32)
        out.append(rows)
    return out


def test_one_node_that_holds_everything_is_the_loop_over_totals():
    import oracle as orc
    rng = np.random.default_rng(20240)
    n = moved = 0
    for trial in range(300):
        J, G, pts, floors = random_case(rng)
        if sum(floors) > G:
            continue
        levels = (1, 2, 4)[:int(rng.integers(1, 4))]
        vals = level_values(rng, pts, levels)
        where, cur_c = draw_state(rng, pts, floors, 1, G, 10 ** 6, levels)
        floor_c = rng.integers(0, len(levels), J).astype(np.uint32)
        state = (rng.uniform(size=J) < 0.15).astype(np.uint8)
        where = [{} if state[j] else where[j] for j in range(J)]
        a, parts, total, moves = nodes_loop(orc, vals, (1, G, 10 ** 6, 1e9), where, levels=levels, cur_c=cur_c,
                                            floors=floors, floor_c=floor_c, state=state)
        tb = table_for(orc, J, G)
        grid = workloads.Grid(np.array(levels, np.uint32), 1, np.array([1.0], np.float32), 0)
        bt = np.array(vals, np.float32).reshape(-1)
        bp = np.arange(bt.size, dtype=np.uint32)
        bp[bt == 0] = orc.NO_PLAN
        ct, _, _ = orc.curves(tb, grid, bt, bp)
        hold = [sum(w.values()) for w in where]
        t, t_total, t_moves = orc.reschedule(np.ones(J, np.float32), tb, grid, workloads.Cluster(G, 10 ** 6, 1e9), bt, bp,
                                             ct, [h - 1 for h in hold], cur_c, [f - 1 for f in floors], floor_c, state=state)
        for f in ("g", "c", "plan", "thr"):
            assert a[f].tolist() == t[f].tolist(), (trial, f)
        assert moves == t_moves and total == pytest.approx(t_total, rel=1e-12)
        n += 1
        moved += moves > 0
    assert n > 200 and moved > 100


def test_invariants_on_random_rounds_over_nodes():
    import oracle as orc
    rng = np.random.default_rng(4711)
    n = moved = spread = 0
    for trial in range(300):
        J, G, pts, floors = random_case(rng)
        gpn = int(rng.choice([1, 2, 4]))
        n_nodes = -(-G // gpn)
        levels = (1, 2, 4)[:int(rng.integers(1, 4))]
        cpn = int(rng.integers(gpn, 4 * gpn + 1))
        vals = level_values(rng, pts, levels)
        floors = [f if f <= n_nodes * gpn else 0 for f in floors]
        where, cur_c = draw_state(rng, pts, floors, n_nodes, gpn, cpn, levels)
        floor_c = np.zeros(J, np.uint32)
        state = (rng.uniform(size=J) < 0.15).astype(np.uint8)
        where = [{} if state[j] else where[j] for j in range(J)]
        hold = [sum(w.values()) for w in where]
        a, parts, total, moves = nodes_loop(orc, vals, (n_nodes, gpn, cpn, 1e9), where, levels=levels, cur_c=cur_c,
                                            floors=floors, floor_c=floor_c, state=state)
        used_g, used_c = [0] * n_nodes, [0] * n_nodes
        for j in range(J):
            g = int(a["g"][j])
            if state[j]:
                assert g == 0
                continue
            if g:
                lvl = a["c"][j] // g
                assert lvl in levels and a["c"][j] == lvl * g
                for node, k in parts[j].items():
                    used_g[node] += k
                    used_c[node] += lvl * k
            if floors[j] and hold[j] >= floors[j]:
                assert g >= floors[j]                          # never shrunk below its minimum
            if floors[j] and hold[j] < floors[j]:
                assert g >= floors[j] or g == hold[j]          # reaches its minimum or stays as it was
            if moves == 0:
                assert parts[j] == where[j]                    # nothing committed: nobody moved
        assert max(used_g) <= gpn and max(used_c) <= cpn       # no node holds more than it has
        if not any(floors[j] and hold[j] < floors[j] and not state[j] for j in range(J)):
            # nobody had to be served at a loss: every committed step raised the total (memory is plentiful here)
            v = np.array(vals, np.float32)[:, :, 0, :]
            best = [np.maximum.accumulate(np.concatenate([[0.0], np.maximum.accumulate(v[j], axis=0)[cur_c[j]]])) for j in range(J)]
            before = sum(float(best[j][hold[j]]) for j in range(J))
            assert total >= before * (1 - 1e-6), (trial, total, before)
        n += 1
        moved += moves > 0
        spread += any(len(p) > 1 for p in parts)
    assert n == 300 and moved > 150 and spread > 50
