"""rk_allocate_static, the allocation entry point that allocates nothing, through the C ABI against rk_allocate:
bit-identical records and totals on two calls in a row, the second on a smaller input, with no change in the
device's free memory across the calls; a round beyond its limit is refused."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


def curves_of(run, jb=0, je=None):
    run.enumerate()
    bt, bp, ct, _, _, n = run.fused(jb, je)
    return bt, bp, ct


def both(rk, run, cluster, bt, bp, ct, jb, je, fresh_ctx):
    """(records, total) of rk_allocate and of rk_allocate_static; the latter on a context that never allocated for it."""
    import torch
    n = je - jb
    a_ref, t_ref = rk.new_assign(n, run.device), run.f32(1)
    rk.rk_allocate(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, cluster, jb, je, bt, bp, ct, a_ref, t_ref)
    rk.rk_sync(run.ctx)
    a_new, t_new = rk.new_assign(n, run.device), run.f32(1)
    t_new.fill_(-1.0)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    rk.rk_allocate_static(fresh_ctx, run.jobs.ref_thr, run.table.c, run.grid, cluster, jb, je, bt, bp, ct, a_new, t_new)
    rk.rk_sync(fresh_ctx)
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated or freed during the call"
    return (rk.assign_to_numpy(a_ref), float(t_ref[0].item())), (rk.assign_to_numpy(a_new), float(t_new[0].item()))


def test_static_scratch_allocation_matches_rk_allocate():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    import paper_2408_08586_amd as rk
    from gpu_harness import DeviceRun
    fresh = rk.rk_create(0)                       # never used by any other entry point: owns no buffer
    # first call: the 10,000-job round (multi-workgroup kernels, histograms)
    wl = workloads.stress()
    run = DeviceRun(wl)
    bt, bp, ct = curves_of(run)
    ref, new = both(rk, run, run.cluster, bt, bp, ct, 0, wl.n_jobs, fresh)
    assert np.array_equal(ref[0], new[0]) and ref[1] == new[1]
    assert (ref[0]["g"] > 0).sum() > 100
    # second call, smaller: a job range of the same table under a scarce cluster (the single-workgroup kernels)
    jb, je = 4100, 4700
    bt2, bp2, ct2 = curves_of(run, jb, je)
    small = rk.make_cluster(workloads.Cluster(300, 700, 2000.0))
    ref2, new2 = both(rk, run, small, bt2, bp2, ct2, jb, je, fresh)
    assert np.array_equal(ref2[0], new2[0]) and ref2[1] == new2[1]
    assert 0 < (ref2[0]["g"] > 0).sum() < je - jb
    # and the large one again after the small one: nothing of the earlier calls is left in the way
    ref3, new3 = both(rk, run, run.cluster, bt, bp, ct, 0, wl.n_jobs, fresh)
    assert np.array_equal(ref[0], new3[0]) and ref[1] == new3[1]
    run.close()
    # a round beyond the limit is refused with a clear error and nothing is written
    wide = workloads.Grid(np.arange(1, 65, dtype=np.uint32), 1, np.array([64.0], np.float32), 0)
    big = workloads.stress(n_jobs=12288)
    big = workloads.Workload("too_many_steps", big.coef, big.ints, workloads.Bounds(g_max=64), wide, big.env, big.cluster)
    run = DeviceRun(big)
    bt, bp, ct = curves_of(run)
    assert big.n_jobs * 64 > rk.RK_STATIC_MAX_STEPS
    a, t = rk.new_assign(big.n_jobs, run.device), run.f32(1)
    with pytest.raises(rk.RkError) as e:
        rk.rk_allocate_static(fresh, run.jobs.ref_thr, run.table.c, run.grid, run.cluster, 0, big.n_jobs, bt, bp, ct, a, t)
    assert e.value.code == rk.RK_ERR_UNSUPPORTED and "rk_allocate_static takes up to" in str(e.value)
    # the same round within the limit on a job range
    ref4, new4 = both(rk, run, run.cluster, *curves_of(run, 0, 8000), 0, 8000, fresh)
    assert np.array_equal(ref4[0], new4[0]) and ref4[1] == new4[1]
    run.close()
    rk.rk_destroy(fresh)
