"""GPU parity of rk_eval_best_plan (evaluation and best plan in one pass, the candidate tensor written once and not
read back): its four outputs must be, bit for bit, what rk_eval_candidates and then rk_best_plan give; those are
compared with the oracle in test_gpu_parity.py and test_gpu_full_size.py, and once more here on the outputs of the
one-pass call itself."""
import dataclasses

import numpy as np
import pytest

import workloads
from test_gpu_parity import check_best_in_band, check_thr
from test_gpu_random_workloads import draw_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def same_as_two_calls(run, jb=0, je=None, want_feas=True):
    thr, feas, n = run.eval(jb, je, want_feas=want_feas)
    bt, bp, ns = run.best(thr, jb, je)
    t2, f2, b2, p2, n2, ns2 = run.eval_best(jb, je, want_feas=want_feas)
    assert (n2, ns2) == (n, ns)
    assert np.array_equal(run.host(t2, n).view(np.uint32), run.host(thr, n).view(np.uint32))
    if want_feas:
        assert np.array_equal(run.host(f2, n), run.host(feas, n))
    assert np.array_equal(run.host(b2, ns).view(np.uint32), run.host(bt, ns).view(np.uint32))
    assert np.array_equal(run.host(p2, ns), run.host(bp, ns))
    return t2, f2, b2, p2, n, ns


@pytest.mark.parametrize("name", ["tiny", "paper_scale", "large"])
def test_named_configurations(gpu, orc, name):
    wl = getattr(workloads, name)()
    r = orc.schedule_round(wl, n_threads=16)
    run = gpu(wl)
    run.enumerate()
    thr, feas, bt, bp, n, ns = same_as_two_calls(run)
    check_thr(run.host(thr, n), run.host(feas, n), r["thr"], r["reason"])
    o_bt, o_bp = orc.best_plan(r["table"], wl.grid, r["thr"])
    check_best_in_band(r["table"], run.n_rows, 0, wl.n_jobs, r["thr"], o_bt, o_bp, run.host(bt, ns),
                       run.host(bp, ns).view(np.uint32))
    # job ranges and the call without the feasibility bytes
    J = wl.n_jobs
    for jb, je in ((0, 1), (J // 3, J - 1), (J - 1, J), (2, 2)):
        same_as_two_calls(run, jb, je, want_feas=(jb % 2 == 0))
    run.close()


def test_random_workloads(gpu, orc):
    """Seeded random workloads: option masks, micro-batch shifts, both grid modes, jobs without plans, small GPU memory
    (many infeasible candidates), jobs with hundreds of GPU counts, rounds of hundreds of jobs."""
    base = workloads.paper_scale()
    done = 0
    for seed in range(260):
        rng = np.random.default_rng(98000 + seed)
        wl = draw_workload(rng, base, wide=seed % 4 == 1, mid=seed % 13 == 2)
        ot = orc.enumerate_plans(wl.ints, wl.bounds)
        if int(np.diff(ot.triple_off).max(initial=0)) > 2048:
            continue
        run = gpu(wl)
        run.enumerate()
        if ot.triple_off[-1] > 0:
            same_as_two_calls(run, want_feas=seed % 2 == 0)
            done += 1
        run.close()
    assert done > 200


def test_many_segments_and_tiers(gpu, orc):
    """Hundreds of GPU counts per job (every tile of 64 triples then touches many segments, up to one per triple) on 16
    and on 2 memory tiers: the CPU levels are split over several workgroups per tile so that their keys fit in LDS."""
    base = workloads.paper_scale()
    ints = np.array([[2, 21621600, 1], [1, 21621600, 1], [24, 64, 2], [2, 3603600, 2]], np.uint32)
    coef = base.coef[[60, 61, 62, 63]].copy()
    b = workloads.Bounds(g_max=20000, tp_max=2, pp_max=2)
    for n_mem in (16, 2):
        grid = workloads.Grid(np.array([1, 2, 6], np.uint32), 1, np.arange(n_mem, dtype=np.float32) * (16 // n_mem), 1)
        wl = workloads.Workload("many_segments", coef, ints, b, grid, workloads.Env(gpu_mem_cap=3e9),
                                workloads.Cluster(30000, 200000, 1500.0))
        run = gpu(wl)
        run.enumerate()
        assert int(np.diff(run.table_numpy()["seg_off"]).max()) > 64
        same_as_two_calls(run)
        same_as_two_calls(run, 1, 3, want_feas=False)
        run.close()


def test_argument_errors(gpu, orc):
    import paper_2408_08586_amd as rk
    wl = workloads.tiny()
    run = gpu(wl)
    run.enumerate()
    n, ns = run.table.n_candidates(run.n_rows), run.table.n_segments(run.n_rows)
    thr, bt, bp = run.f32(n), run.f32(ns), run.i32(ns)
    longer = run.f32(n + 4)
    call = lambda t=thr, b=bt, p=bp, jb=0, je=wl.n_jobs: rk.rk_eval_best_plan(run.ctx, run.jobs, run.table.c, run.grid, run.env,
                                                                             jb, je, t, b, p)
    for kwargs, code in (({"t": None}, rk.RK_ERR_INVALID_ARG), ({"b": None}, rk.RK_ERR_INVALID_ARG),
                         ({"p": None}, rk.RK_ERR_INVALID_ARG), ({"t": thr[:n - 16]}, rk.RK_ERR_CAPACITY),
                         ({"b": bt[:ns - 1]}, rk.RK_ERR_CAPACITY), ({"t": longer[1:]}, rk.RK_ERR_INVALID_ARG),
                         ({"jb": 3, "je": 2}, rk.RK_ERR_INVALID_ARG), ({"je": wl.n_jobs + 1}, rk.RK_ERR_INVALID_ARG)):
        with pytest.raises(rk.RkError) as e:
            call(**kwargs)
        assert e.value.code == code, kwargs
    call()
    rk.rk_sync(run.ctx)
    run.close()
