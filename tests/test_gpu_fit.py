"""GPU parity of the model fitting (paper Sec. 4, "Continuous model fitting")
against the CPU oracle: the objective element by element, exact recovery of
exact data, and the minimum reached on noisy data."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from gpu_harness import DeviceRun
    return DeviceRun


class FitCase:
    """Models, their sample runs (plans from the oracle's enumeration) and the
    oracle's noise-free throughputs of these runs under the true parameters."""

    def __init__(self, orc, n_models, n_samples, sigma, g_max=64, n_offload=5):
        F = orc.fitting
        self.F = F
        self.wl = workloads.large().subset(np.arange(n_models))
        wl = self.wl
        self.tb = orc.enumerate_plans(wl.ints, workloads.Bounds(g_max=g_max))
        self.dr = workloads.fit_draws(n_models, n_samples, n_offload=n_offload)
        self.d, self.t, self.p = workloads.fit_sample_triples(self.dr, self.tb.triple_off, self.tb.triples)
        self.true = wl.coef[:, list(F.THETA_COLUMNS)].astype(np.float64)
        clean = np.stack([F.predict(wl.coef[j], wl.ints[j], wl.env, self.true[j], self.d[j], self.t[j], self.p[j],
                                    self.dr.option[j], self.dr.cpus[j]) for j in range(n_models)])
        assert np.all(clean > 0)
        self.y = (clean * np.exp(sigma * self.dr.noise_z)).astype(np.float32)      # what both sides are given
        self.theta0 = np.stack([F.project(self.true[j] * self.dr.start_factor[j]) for j in range(n_models)])
        # the job array the library starts from: true constants, perturbed fittable parameters (float32)
        self.coef0 = wl.coef.copy()
        self.coef0[:, list(F.THETA_COLUMNS)] = self.theta0.astype(np.float32)
        self.theta0 = self.coef0[:, list(F.THETA_COLUMNS)].astype(np.float64)      # as both sides see them
        self.n_models, self.n_samples = n_models, n_samples

    def run_args(self, j):
        return (self.d[j], self.t[j], self.p[j], self.dr.option[j], self.dr.cpus[j])

    def oracle_rmsle(self, j, theta):
        wl = self.wl
        return self.F.rmsle(self.F.predict(wl.coef[j], wl.ints[j], wl.env, theta, *self.run_args(j)), self.y[j].astype(np.float64))

    def fit_on_gpu(self, gpu, with_starts=True, refit_threshold=0.0, counts=None):
        import paper_2408_08586_amd as rk
        wl0 = workloads.Workload("fit", self.coef0, self.wl.ints, self.wl.bounds, self.wl.grid, self.wl.env, self.wl.cluster)
        run = gpu(wl0)
        J, S = self.n_models, self.n_samples
        counts = np.full(J, S) if counts is None else np.asarray(counts)
        off = np.concatenate([[0], np.cumsum(counts)])
        take = np.concatenate([np.arange(c) + j * S for j, c in enumerate(counts)]).astype(np.int64)
        flat = lambda a: np.ascontiguousarray(a).reshape(-1)[take]
        smp = rk.Samples(off, flat(rk.pack_triples(self.d, self.t, self.p)), flat(self.dr.option), flat(self.dr.cpus),
                         flat(self.y))
        res = rk.FitResult(J)
        rk.rk_fit_models(run.ctx, run.jobs, run.env, smp, res, max_iter=100, refit_threshold=refit_threshold,
                         start_offsets=self.dr.start_offsets if with_starts else None)
        rk.rk_sync(run.ctx)
        out = dict(theta=res.theta.cpu().numpy()[:J], params=res.params.cpu().numpy()[:, :J],
                   before=res.rmsle_before.cpu().numpy()[:J], after=res.rmsle_after.cpu().numpy()[:J],
                   iters=res.iters.cpu().numpy()[:J].view(np.uint32))
        run.close()
        return out


def test_objective_matches_the_oracle_on_many_models(gpu, orc):
    """The error of the starting parameters, as the library computes it, against
    the oracle's for 1,000 models x 16 runs (every kind of plan)."""
    case = FitCase(orc, 1000, 16, sigma=0.05)
    got = case.fit_on_gpu(gpu, with_starts=False, refit_threshold=1e9)        # nothing is refitted: the objective only
    want = np.array([case.oracle_rmsle(j, case.theta0[j]) for j in range(case.n_models)])
    assert np.max(np.abs(got["before"] - want) / want) <= 1e-6
    assert np.array_equal(got["iters"], np.zeros(case.n_models, np.uint32))
    assert np.array_equal(got["theta"], case.theta0)                          # left alone, bit for bit
    assert np.array_equal(got["after"], got["before"])


def test_exact_data_are_recovered(gpu, orc):
    case = FitCase(orc, 200, 16, sigma=0.0)
    got = case.fit_on_gpu(gpu)
    F, wl = case.F, case.wl
    tb_wide = orc.enumerate_plans(wl.ints, workloads.Bounds(g_max=128))
    # the measurements are float32: the least error is that rounding, about 3e-8
    assert np.all(got["before"] > 1e-3)
    fit_err, pred_err = np.zeros(case.n_models), np.zeros(case.n_models)
    for j in range(case.n_models):
        e = case.oracle_rmsle(j, got["theta"][j])
        fit_err[j] = e
        assert abs(got["after"][j] - e) <= 1e-6 + 1e-5 * e
        tr = tb_wide.triples[tb_wide.triple_off[j]:tb_wide.triple_off[j + 1]]
        pick = np.linspace(0, len(tr) - 1, 24).astype(int)
        for o, c in ((0, 1), (6, 1), (13, 8), (11, 32)):                      # held-out runs of every kind
            a = F.predict(wl.coef[j], wl.ints[j], wl.env, got["theta"][j], tr[pick, 0], tr[pick, 1], tr[pick, 2], [o] * 24, [c] * 24)
            b = F.predict(wl.coef[j], wl.ints[j], wl.env, case.true[j], tr[pick, 0], tr[pick, 1], tr[pick, 2], [o] * 24, [c] * 24)
            pred_err[j] = max(pred_err[j], float(np.max(np.abs(a - b) / b)))
    exact = fit_err <= 1e-6
    print(f"exact data: {int(exact.sum())}/{case.n_models} models fitted to RMSLE <= 1e-6 (their worst held-out prediction "
          f"error {pred_err[exact].max():.2e}); the others: worst RMSLE {fit_err.max():.2e}, worst held-out error "
          f"{pred_err.max():.2e}; iterations per model {got['iters'].mean():.0f}")
    # an overlap exponent can stay on the plateau at its upper bound (a local minimum of the bounded problem)
    assert exact.mean() >= 0.93
    assert fit_err.max() <= 1e-3
    # held-out runs: the measurements are float32, and weakly determined parameters (an overlap exponent seen by two
    # or three runs) amplify that rounding; the oracle's own fit of these data shows the same spread
    pe = pred_err[exact]
    print(f"held-out prediction error of the exactly fitted models: median {np.median(pe):.2e}, 90th percentile "
          f"{np.percentile(pe, 90):.2e}, worst {pe.max():.2e}")
    assert np.median(pe) <= 1e-5 and np.percentile(pe, 90) <= 2e-4 and pe.max() <= 2e-2
    # float32 copies of the parameters
    assert np.allclose(got["params"].T, got["theta"], rtol=1e-6, atol=0)


def test_noisy_fit_reaches_the_oracles_minimum(gpu, orc):
    """5 % measurement noise.  The problem has several local minima; both sides
    use the same starting points.  Every result must be feasible, no worse than
    where it started, and its error as the oracle evaluates it must match what
    the library reports; the minimum itself must equal the oracle's in most
    models and be close in all."""
    case = FitCase(orc, 40, 16, sigma=0.05)
    got = case.fit_on_gpu(gpu)
    F, wl = case.F, case.wl
    rel = []
    for j in range(case.n_models):
        th = got["theta"][j]
        assert np.all(th >= 0) and np.all(th[F.IS_EXPONENT] >= 1) and np.all(th[F.IS_EXPONENT] <= F.K_MAX * (1 + 1e-12))
        e_gpu = case.oracle_rmsle(j, th)
        assert abs(got["after"][j] - e_gpu) <= 1e-6 * (1 + e_gpu)
        assert e_gpu <= case.oracle_rmsle(j, case.theta0[j])
        assert e_gpu <= case.oracle_rmsle(j, case.true[j]) * (1 + 1e-9)       # at least as good as the generating parameters
        _, e_orc, _ = F.fit_one(wl.coef[j], wl.ints[j], wl.env, case.theta0[j], *case.run_args(j),
                                case.y[j].astype(np.float64), start_offsets=case.dr.start_offsets)
        rel.append((e_gpu - e_orc) / e_orc)
    rel = np.array(rel)
    same = np.abs(rel) <= 1e-6
    print(f"noisy data: {int(same.sum())}/{len(rel)} minima equal to the oracle's; others: worst {rel.max():+.2e}, "
          f"best {rel.min():+.2e}; iterations per model {got['iters'].mean():.0f} (max {got['iters'].max()})")
    # observed on this seeded case: 37 of 40 equal, the others between -0.2 % and +0.009 % (a lower value means the
    # library found a better minimum than the oracle's routine)
    assert same.mean() >= 0.85
    assert rel.max() <= 1e-3


@pytest.mark.parametrize("n_samples,n_offload", [(7, 3), (24, 6), (40, 10), (64, 12)])
def test_group_widths_and_refit_threshold(gpu, orc, n_samples, n_offload):
    """Every group width of the kernel (8, 32, 64 lanes per model; 16 is covered
    above), and the refit rule: models below the threshold keep their parameters."""
    case = FitCase(orc, 60, n_samples, sigma=0.03, n_offload=n_offload)
    thr = float(np.median([case.oracle_rmsle(j, case.theta0[j]) for j in range(case.n_models)]))
    got = case.fit_on_gpu(gpu, refit_threshold=thr)
    kept = got["iters"] == 0
    assert 10 <= kept.sum() <= 50
    for j in range(case.n_models):
        before = case.oracle_rmsle(j, case.theta0[j])
        assert abs(got["before"][j] - before) <= 1e-6 * before
        if kept[j]:
            assert got["before"][j] <= np.float32(thr) and np.array_equal(got["theta"][j], case.theta0[j])
        else:
            e = case.oracle_rmsle(j, got["theta"][j])
            assert e <= before and abs(got["after"][j] - e) <= 1e-6 * (1 + e)


def test_fit_edge_cases(gpu, orc):
    import paper_2408_08586_amd as rk
    case = FitCase(orc, 12, 16, sigma=0.02)
    # ragged sample counts, a model without runs, invalid runs
    counts = np.array([16, 0, 7, 16, 9, 1, 16, 16, 3, 16, 16, 8])
    case.dr.option[3, 0] = 5                       # offload with ZeRO stage 1: not a valid plan
    case.d[6, 1] = 7                               # 7 * mu does not divide the batch
    got = case.fit_on_gpu(gpu, counts=counts)
    F, wl = case.F, case.wl
    for j in range(case.n_models):
        c = counts[j]
        args = tuple(a[:c] for a in case.run_args(j))
        y = case.y[j, :c].astype(np.float64)
        rm = lambda th: F.rmsle(F.predict(wl.coef[j], wl.ints[j], wl.env, th, *args), y)
        if c == 0:
            assert got["iters"][j] == 0 and got["before"][j] == 0 and np.array_equal(got["theta"][j], case.theta0[j])
            continue
        before = rm(case.theta0[j])
        assert abs(got["before"][j] - before) <= 1e-6 * before
        e = rm(got["theta"][j])
        assert e <= before and abs(got["after"][j] - e) <= 1e-6 * (1 + e)
    assert F.predict(wl.coef[6], wl.ints[6], wl.env, case.true[6], *case.run_args(6))[1] == 0      # the oracle calls that run invalid too
    # more runs than announced: flagged and left alone
    wl0 = workloads.Workload("fit", case.coef0, wl.ints, wl.bounds, wl.grid, wl.env, wl.cluster)
    run = gpu(wl0)
    S = case.n_samples
    flat = lambda a: np.ascontiguousarray(a).reshape(-1)
    smp = rk.Samples(np.arange(13) * S, flat(rk.pack_triples(case.d, case.t, case.p)), flat(case.dr.option),
                     flat(case.dr.cpus), flat(case.y))
    smp.c.max_samples = 8
    res = rk.FitResult(12)
    rk.rk_fit_models(run.ctx, run.jobs, run.env, smp, res)
    rk.rk_sync(run.ctx)
    assert np.all(res.iters.cpu().numpy().view(np.uint32) == 0xFFFFFFFF)
    assert np.array_equal(res.theta.cpu().numpy(), case.theta0)
    # argument errors
    smp.c.max_samples = rk.RK_FIT_MAX_SAMPLES + 1
    with pytest.raises(rk.RkError) as e:
        rk.rk_fit_models(run.ctx, run.jobs, run.env, smp, res)
    assert e.value.code == rk.RK_ERR_UNSUPPORTED
    smp.c.max_samples = 16
    with pytest.raises(rk.RkError) as e:
        rk.rk_fit_models(run.ctx, run.jobs, run.env, smp, res, start_offsets=np.zeros((rk.RK_FIT_MAX_STARTS + 1, 7)))
    assert e.value.code == rk.RK_ERR_UNSUPPORTED
    with pytest.raises(rk.RkError) as e:
        rk.rk_fit_models(run.ctx, run.jobs, run.env, smp, res, refit_threshold=-1.0)
    assert e.value.code == rk.RK_ERR_INVALID_ARG
    run.close()
