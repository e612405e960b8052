"""GPU parity of the node-level placement (paper Sec. 5.2, Algorithm 1,
ScheduleJob: a job walks the nodes in order and takes what is free on each)
against the CPU oracle: offsets, parts and status words must be identical,
whichever of the library's two stages produced them."""
import json
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def placer():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2408_08586_amd as rk

    class Placer:
        def __init__(self):
            self.ctx = rk.rk_create(0)

        def place(self, assign, n_nodes, gpn, cpn, mpn, cap=None):
            assign = np.ascontiguousarray(assign, dtype=rk.ASSIGN_DTYPE)
            J = assign.size
            dev = "cuda:0"
            d_assign = torch.from_numpy(assign.view(np.uint8).copy()).to(dev) if J else torch.zeros(4, dtype=torch.uint8, device=dev)
            cap = n_nodes * gpn if cap is None else cap
            off = torch.full((J + 1,), -1, dtype=torch.int32, device=dev)
            status = torch.full((max(J, 1),), -1, dtype=torch.int32, device=dev)
            ent = rk.new_place_entries(cap, dev)
            res = rk.rk_place(self.ctx, rk.rk_nodes(n_nodes, gpn, cpn, mpn), J, d_assign, off, ent, cap, status)
            return (rk.u32(off), rk.place_entries_to_numpy(ent, res.n_entries), rk.u32(status)[:J], res)

        def close(self):
            rk.rk_destroy(self.ctx)

    p = Placer()
    yield p
    p.close()


def jobs(orc, g, c, mem):
    a = np.zeros(len(g), orc.ASSIGN_DTYPE)
    a["g"], a["c"], a["mem_gb"] = g, c, mem
    return a


def same(orc, placer, a, n_nodes, gpn, cpn, mpn, in_order=None):
    w_off, w_ent, w_st = orc.place(a, n_nodes, gpn, cpn, mpn)
    off, ent, st, res = placer.place(a, n_nodes, gpn, cpn, mpn)
    assert np.array_equal(off, w_off)
    assert np.array_equal(st, w_st)
    assert res.n_entries == len(w_ent) and res.n_placed == int((w_st == 1).sum()) and res.n_failed == int((w_st == 2).sum())
    for f in ("node", "g", "c", "mem_gb"):
        assert np.array_equal(ent[f], w_ent[f]), f
    if in_order is not None:
        assert res.in_order == in_order
    return res


def test_hand_cases(orc, placer):
    same(orc, placer, jobs(orc, [3, 2, 3], [6, 4, 3], [3.0, 8.0, 1.5]), 2, 4, 100, 100.0, in_order=0)
    same(orc, placer, jobs(orc, [3], [5], [0.0]), 3, 1, 8, 1.0, in_order=0)
    same(orc, placer, jobs(orc, [2, 2, 2], [8, 2, 0], [0.0, 0.0, 0.0]), 2, 4, 8, 1.0, in_order=1)     # CPUs bind
    same(orc, placer, jobs(orc, [1, 4], [5, 8], [0.0, 0.0]), 2, 8, 8, 1.0, in_order=1)
    same(orc, placer, jobs(orc, [4], [0], [10.0]), 3, 4, 8, 6.0, in_order=1)                           # memory binds
    same(orc, placer, jobs(orc, [3, 2, 1, 0], [0, 0, 0, 0], [0.0] * 4), 2, 2, 4, 1.0, in_order=1)      # a job fails


@pytest.mark.parametrize("seed", range(8))
def test_random_small_rounds(orc, placer, seed):
    rng = np.random.default_rng(100 + seed)
    n_nodes, gpn, cpn, mpn = 24, 8, int(rng.choice([16, 32, 96, 4096])), float(rng.choice([64.0, 256.0, 1600.0, 1e6]))
    J = 40
    g = rng.choice([0, 1, 1, 2, 2, 3, 4, 6, 8, 16], size=J).astype(np.uint32)
    c = (g * rng.choice([1, 2, 4, 8, 16], size=J)).astype(np.uint32)
    c[rng.random(J) < 0.3] += 1
    c[g == 0] = 0
    mem = (g * rng.choice([0.0, 8.0, 37.5, 120.0], size=J)).astype(np.float32)
    same(orc, placer, jobs(orc, g, c, mem), n_nodes, gpn, cpn, mpn)


def stored_stress_assignment(orc):
    """The oracle's stored round on the stress workload: 143 of 10,000 jobs hold the 4,096 GPUs."""
    d = json.load(open(os.path.join(HERE, "golden", "stress_round.json")))
    a = np.zeros(d["n_jobs"], orc.ASSIGN_DTYPE)
    for j, g, c, mem, plan, thr in d["scheduled"]:
        a[j] = (g, c, mem, plan, thr)
    return a


def test_stress_round_on_the_papers_node_shape(orc, placer):
    a = stored_stress_assignment(orc)
    assert int(a["g"].sum()) == 4096
    res = same(orc, placer, a, 512, 8, 128, 2048.0, in_order=0)       # roomy nodes: all jobs at once
    assert res.n_placed == 143 and res.n_failed == 0
    # the stored round asks for one CPU per GPU and no host memory; give its jobs 1-3 CPUs per GPU and 0-90 GiB per GPU
    jid = np.arange(a.size, dtype=np.uint32)
    b = a.copy()
    b["c"] = a["g"] * (1 + jid % 3)
    b["mem_gb"] = a["g"].astype(np.float32) * (30.0 * (jid % 4)).astype(np.float32)
    same(orc, placer, b, 512, 8, 128, 2048.0, in_order=0)
    res = same(orc, placer, b, 512, 8, 16, 2048.0, in_order=1)        # two CPUs per GPU on a node: CPUs bind
    print(f"stress round, 16 CPUs per node: {res.n_placed} placed, {res.n_failed} not placed, {res.n_entries} parts")
    same(orc, placer, b, 600, 8, 40, 500.0, in_order=1)               # spare nodes, memory binds
    same(orc, placer, b, 4096, 1, 16, 2048.0)                         # one GPU per node
    same(orc, placer, a, 100, 8, 128, 2048.0, in_order=1)             # too few nodes: later jobs fail


@pytest.mark.parametrize("n_jobs,n_nodes,fill", [(12000, 4096, 0.9), (5000, 1024, 1.3), (3333, 700, 0.5)])
def test_many_jobs_per_round(orc, placer, n_jobs, n_nodes, fill):
    """Several tiles of 1,024 jobs, parts crossing node borders everywhere; once
    with room to spare (all jobs at once) and once with CPUs or memory binding."""
    rng = np.random.default_rng(n_jobs)
    gpn = 8
    g = rng.choice([0, 0, 0, 1, 1, 2, 3, 4, 5, 8, 16, 40], size=n_jobs).astype(np.uint32)
    scale = fill * n_nodes * gpn / max(int(g.sum()), 1)
    g = np.where(rng.random(n_jobs) < scale, g, 0).astype(np.uint32)
    c = (g * rng.choice([1, 2, 4, 12], size=n_jobs)).astype(np.uint32) + (rng.random(n_jobs) < 0.2) * (g > 0)
    mem = (g * rng.choice([0.0, 16.0, 50.0], size=n_jobs)).astype(np.float32)
    a = jobs(orc, g, c.astype(np.uint32), mem)
    r0 = same(orc, placer, a, n_nodes, gpn, 200, 4096.0)
    assert r0.in_order == (1 if int(g.sum()) > n_nodes * gpn else 0)
    r1 = same(orc, placer, a, n_nodes, gpn, 48, 300.0, in_order=1)
    print(f"{n_jobs} jobs on {n_nodes} nodes: {r0.n_placed}/{r0.n_failed} placed/failed roomy, {r1.n_placed}/{r1.n_failed} tight")


def test_buffers_that_are_not_16_byte_aligned_and_no_result(orc, placer):
    """The library reads and writes eight jobs at a time with 16-byte accesses when the
    caller's buffers allow it; buffers that start 4 bytes off take the plain path.
    Without a result struct the call does not wait."""
    import torch
    import paper_2408_08586_amd as rk
    rng = np.random.default_rng(5)
    J, n_nodes, gpn = 3001, 300, 8
    g = np.where(rng.random(J) < 0.15, rng.choice([1, 2, 4, 8, 24], size=J), 0).astype(np.uint32)
    a = jobs(orc, g, g * 2, (g * 10).astype(np.float32))
    w_off, w_ent, w_st = orc.place(a, n_nodes, gpn, 96, 1600.0)
    dev = "cuda:0"
    raw = torch.zeros(4 + a.nbytes, dtype=torch.uint8, device=dev)
    raw[4:] = torch.from_numpy(a.view(np.uint8).copy()).to(dev)
    off = torch.full((J + 2,), -1, dtype=torch.int32, device=dev)
    status = torch.full((J + 1,), -1, dtype=torch.int32, device=dev)
    cap = n_nodes * gpn
    ent = rk.new_place_entries(cap, dev)
    assert raw[4:].data_ptr() % 16 == 4 and off[1:].data_ptr() % 16 == 4
    res = rk.rk_place(placer.ctx, rk.rk_nodes(n_nodes, gpn, 96, 1600.0), J, raw[4:], off[1:], ent, cap, status[1:],
                      want_result=False)
    assert res is None
    rk.rk_sync(placer.ctx)
    assert np.array_equal(rk.u32(off)[1:], w_off) and np.array_equal(rk.u32(status)[1:], w_st)
    got = rk.place_entries_to_numpy(ent, len(w_ent))
    for f in ("node", "g", "c", "mem_gb"):
        assert np.array_equal(got[f], w_ent[f]), f
    assert rk.u32(off)[0] == 0xFFFFFFFF and rk.u32(status)[0] == 0xFFFFFFFF      # nothing before the buffers is touched


def test_edge_cases(orc, placer):
    import paper_2408_08586_amd as rk
    same(orc, placer, jobs(orc, [], [], []), 4, 8, 96, 1600.0, in_order=0)                   # no jobs
    same(orc, placer, jobs(orc, [0, 0, 0], [0, 0, 0], [0.0] * 3), 4, 8, 96, 1600.0, in_order=0)
    same(orc, placer, jobs(orc, [40, 8], [40, 8], [0.0, 0.0]), 4, 8, 96, 1600.0, in_order=1)  # larger than the cluster
    same(orc, placer, jobs(orc, [8], [8], [1600.0]), 1, 8, 96, 1600.0, in_order=1)            # memory exactly full
    same(orc, placer, jobs(orc, [8], [96], [100.0]), 1, 8, 96, 1600.0, in_order=0)            # CPUs exactly full
    same(orc, placer, jobs(orc, [4, 4], [0, 0], [0.0, 0.0]), 1, 8, 0, 0.0, in_order=0)        # nodes without CPUs or memory
    # amounts beyond 16 bits (the library switches to 64-bit products): 81,920 CPUs, 70,000 GPUs
    same(orc, placer, jobs(orc, [5, 2048, 3], [10, 81920, 7], [0.0, 4096.0, 1.0]), 300, 8, 400, 64.0, in_order=0)
    same(orc, placer, jobs(orc, [5, 2048, 3], [10, 81920, 7], [0.0, 4096.0, 1.0]), 300, 8, 300, 64.0, in_order=1)
    same(orc, placer, jobs(orc, [3, 70000, 9], [3, 140001, 9], [0.0, 7.0e4, 0.0]), 4096, 32, 100, 64.0, in_order=0)
    same(orc, placer, jobs(orc, [3, 70000, 9], [3, 140001, 9], [0.0, 7.0e4, 0.0]), 4096, 32, 60, 64.0, in_order=1)
    with pytest.raises(rk.RkError) as e:
        placer.place(jobs(orc, [1], [1], [0.0]), 4, 8, 96, 1600.0, cap=31)
    assert e.value.code == rk.RK_ERR_CAPACITY
    with pytest.raises(rk.RkError) as e:
        placer.place(jobs(orc, [1], [1], [0.0]), 5000, 8, 96, 1600.0)
    assert e.value.code == rk.RK_ERR_UNSUPPORTED
