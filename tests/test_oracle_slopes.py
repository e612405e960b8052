"""Pins of the oracle's slope table of the resource sensitivity curves (Sec. 5.2: slopes per resource type; Fig. 6):
hand values, concave curves, and the Schedule loop of a lone job on a large empty cluster, whose steps walk the table."""
import numpy as np
import pytest

import workloads
from test_oracle_reschedule import table_for


def table_of(orc, vals, levels=(1,), mode=0, ref=None):
    """vals[j][level][g-1] (or [j][g-1]): best throughput with g GPUs at that CPU level, 0 = no plan."""
    vals = np.array(vals, np.float32)
    if vals.ndim == 2:
        vals = vals[:, None, :]
    J, n_cpu, g_max = vals.shape
    tb = table_for(orc, J, g_max)
    grid = workloads.Grid(np.array(levels, np.uint32), mode, np.array([1.0], np.float32), 0)
    bt = vals.reshape(-1)
    bp = np.arange(bt.size, dtype=np.uint32)
    bp[bt == 0] = orc.NO_PLAN
    ct, _, _ = orc.curves(tb, grid, bt, bp)
    ref = np.ones(J, np.float32) if ref is None else np.asarray(ref, np.float32)
    out = orc.curve_slopes(ref, tb, grid, bt, ct)
    shape = (J, n_cpu, g_max)
    return {k: (v.reshape(shape) if v.size == bt.size else v.reshape(J, n_cpu)) for k, v in out.items()}, (tb, grid, bt, bp, ct, ref)


def test_hand_values():
    import oracle as orc
    f32 = np.float32
    # a concave curve: always the next count, with falling slopes; from nothing the first GPU
    t, _ = table_of(orc, [[1.0, 1.9, 2.7, 3.4]])
    assert t["gpu_next"][0, 0].tolist() == [1, 2, 3, -1] and t["from0_next"][0, 0] == 0
    assert t["gpu_slope"][0, 0].tolist() == [f32(1.9) - f32(1.0), f32(2.7) - f32(1.9), f32(3.4) - f32(2.7), 0.0]
    assert t["from0_slope"][0, 0] == 1.0
    # counts without a plan are stepped over: from 1 GPU the only gain is at 4, worth 0.3 over three GPUs
    t, _ = table_of(orc, [[1.0, 0.0, 0.0, 1.3]])
    assert t["gpu_next"][0, 0].tolist() == [3, 3, 3, -1] and t["gpu_slope"][0, 0, 0] == (f32(1.3) - f32(1.0)) / f32(3.0)
    # the best reachable point, not the nearest: 4 GPUs give 1.0 per GPU, 2 GPUs 0.5; equal slopes: the smaller count
    t, _ = table_of(orc, [[0.5, 1.0, 0.0, 4.0], [1.0, 2.0, 3.0, 4.0]])
    assert t["from0_next"][:, 0].tolist() == [3, 0] and t["from0_slope"][0, 0] == 1.0
    # the reference throughput divides the slopes
    t, _ = table_of(orc, [[1.0, 1.9]], ref=[0.5])
    assert t["from0_slope"][0, 0] == 2.0
    # CPU steps: per CPU of the job (mode 0) or per GPU (mode 1, two GPUs: twice the CPUs)
    vals = [[[1.0, 2.0], [1.5, 2.0], [1.6, 3.0]]]
    t, _ = table_of(orc, vals, levels=(1, 2, 4))
    assert t["cpu_next"][0, :, 0].tolist() == [1, 2, 3] and t["cpu_slope"][0, 0, 0] == 0.5
    assert t["cpu_next"][0, :, 1].tolist() == [2, 2, 3] and t["cpu_slope"][0, 0, 1] == f32(1.0) / f32(3.0)
    t, _ = table_of(orc, vals, levels=(1, 2, 4), mode=1)
    assert t["cpu_slope"][0, 0, 1] == f32(1.0) / f32(6.0) and t["cpu_slope"][0, 1, 0] == (f32(1.6) - f32(1.5)) / f32(2.0)


def test_a_lone_job_walks_the_table():
    import oracle as orc
    rng = np.random.default_rng(5150)
    for trial in range(200):
        g_max, n_cpu = int(rng.integers(2, 17)), int(rng.integers(1, 4))
        base = np.zeros(g_max)
        valid = np.unique(np.concatenate([[1], rng.choice(np.arange(1, g_max + 1), int(rng.integers(1, 6)))]))
        base[valid - 1] = np.cumsum(rng.uniform(0.1, 2.0, len(valid)))
        vals = np.stack([base * (1 + 0.3 * c * rng.uniform()) for c in range(n_cpu)])
        levels = tuple(int(x) for x in np.cumsum(rng.integers(1, 4, n_cpu)))
        t, (tb, grid, bt, bp, ct, ref) = table_of(orc, [vals], levels=levels, mode=int(rng.integers(0, 2)))
        # GPUs at the lowest level: from nothing, then from count to count until the table says stop
        s = int(t["from0_next"][0, 0])
        while s >= 0 and t["gpu_next"][0, 0, s] >= 0:
            s = int(t["gpu_next"][0, 0, s])
        c = 0
        while s >= 0 and t["cpu_next"][0, c, s] < n_cpu:
            c = int(t["cpu_next"][0, c, s])
        a, _, _ = orc.reschedule(ref, tb, grid, workloads.Cluster(g_max, 10 ** 6, 1e9), bt, bp, ct, [-1], [0])
        assert a["g"][0] == (s + 1 if s >= 0 else 0), trial
        if s >= 0:
            assert a["c"][0] == (levels[c] * (s + 1) if grid.cpu_mode else levels[c]), trial
