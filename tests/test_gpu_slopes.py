"""GPU parity of rk_curve_slopes against the oracle's ork_curve_slopes on shared float32 inputs: the slope table of
the resource sensitivity curves must be identical, entry by entry (it is float32 arithmetic in a fixed order)."""
import numpy as np
import pytest

import workloads
from test_gpu_reschedule import random_round

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


def slopes_on_gpu(run, bt, ct, n, jb=0, je=None):
    """bt, ct: device tensors in segment layout of [jb, je); n entries."""
    import torch
    import paper_2408_08586_amd as rk
    je = run.wl.n_jobs if je is None else je
    dev = run.device
    rows = len(run.wl.grid.cpu_levels) * len(run.wl.grid.mem_levels_gb)
    f32 = lambda k: torch.full((max(k, 1),), -9.0, dtype=torch.float32, device=dev)
    i32 = lambda k: torch.full((max(k, 1),), -9, dtype=torch.int32, device=dev)
    out = dict(gpu_slope=f32(n), gpu_next=i32(n), from0_slope=f32(rows * (je - jb)), from0_next=i32(rows * (je - jb)),
               cpu_slope=f32(n), cpu_next=i32(n))
    rk.rk_curve_slopes(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, jb, je, bt, ct, out["gpu_slope"], out["gpu_next"],
                       out["from0_slope"], out["from0_next"], out["cpu_slope"], out["cpu_next"])
    rk.rk_sync(run.ctx)
    sizes = dict(gpu_slope=n, gpu_next=n, cpu_slope=n, cpu_next=n, from0_slope=rows * (je - jb), from0_next=rows * (je - jb))
    return {k: v.cpu().numpy()[:sizes[k]] for k, v in out.items()}


def same(got, want):
    for k, w in want.items():
        g = got[k].view(w.dtype) if got[k].dtype != w.dtype else got[k]
        assert np.array_equal(g, w), (k, np.flatnonzero(g != w)[:5])


def test_drawn_tables(gpu, orc):
    n_steps = 0
    for seed in range(150):
        rng = np.random.default_rng(71000 + seed)
        wl, tb, bt, bp, ct, *_ = random_round(rng, orc, 500 if seed % 25 == 24 else None, 20 if seed % 25 == 24 else None)
        want = orc.curve_slopes(wl.coef[:, 16], tb, wl.grid, bt, ct)
        run = gpu(wl)
        run.enumerate()
        same(slopes_on_gpu(run, run.dev_f32(bt), run.dev_f32(ct), bt.size), want)
        n_steps += int((want["gpu_next"] >= 0).sum())
        run.close()
    assert n_steps > 10000


@pytest.mark.parametrize("name", ["paper_scale", "large", "stress"])
def test_generated_workloads_and_job_ranges(gpu, orc, name):
    """The library's own curves (fused path) of a generated workload, the whole table and a range of jobs in its middle."""
    wl = workloads.CONFIGS[name]()
    run = gpu(wl)
    run.enumerate()
    bt, bp, ct, _, _, n = run.fused()
    h_bt, h_ct = run.host(bt, n).copy(), run.host(ct, n).copy()
    tn = run.table_numpy()
    tb = orc.Table(tn["triple_off"], tn["triples"], tn["seg_off"], tn["seg_g"], tn["seg_first"])
    want = orc.curve_slopes(wl.coef[:, 16], tb, wl.grid, h_bt, h_ct)
    got = slopes_on_gpu(run, bt, ct, n)
    same(got, want)
    J = wl.n_jobs
    jb, je = J // 3, J // 3 + max(1, J // 7)
    rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
    a, b = rows * int(tb.seg_off[jb]), rows * int(tb.seg_off[je])
    part = slopes_on_gpu(run, bt[a:], ct[a:], b - a, jb, je)
    for k in ("gpu_slope", "gpu_next", "cpu_slope", "cpu_next"):
        assert np.array_equal(part[k], got[k][a:b]), k
    for k in ("from0_slope", "from0_next"):
        assert np.array_equal(part[k], got[k][rows * jb:rows * je]), k
    print(f"{name}: {n} entries, {int((want['gpu_next'] >= 0).sum())} with a GPU step, "
          f"{int((want['cpu_next'] < len(wl.grid.cpu_levels)).sum())} with a CPU step, steepest first step "
          f"{float(want['from0_slope'].max()):.3g} per GPU")
    run.close()


def test_argument_errors(gpu, orc):
    import paper_2408_08586_amd as rk
    wl = workloads.tiny()
    run = gpu(wl)
    run.enumerate()
    bt, bp, ct, _, _, n = run.fused()
    with pytest.raises(rk.RkError) as e:
        slopes_on_gpu(run, bt, ct, n - 1)
    assert e.value.code == rk.RK_ERR_CAPACITY
    f = run.f32(n)
    with pytest.raises(rk.RkError) as e:
        rk.rk_curve_slopes(run.ctx, run.jobs.ref_thr, run.table.c, run.grid, 0, wl.n_jobs, bt, ct, f, None, f, f, f, f)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    run.close()
