"""Pins for the oracle's model fitting (paper Sec. 4, "Continuous model
fitting": the seven parameters minimise the RMSLE between the model and the
measured throughputs of at least seven sample runs, three of them offloaded)."""
import numpy as np
import pytest

import workloads


@pytest.fixture(scope="module")
def F(orc):
    return orc.fitting


def samples(orc, wl, n_samples=16, g_max=64):
    tb = orc.enumerate_plans(wl.ints, workloads.Bounds(g_max=g_max))
    dr = workloads.fit_draws(wl.n_jobs, n_samples)
    d, t, p = workloads.fit_sample_triples(dr, tb.triple_off, tb.triples)
    return dr, d, t, p


def test_rmsle_is_the_definition(F):
    assert F.rmsle([3.0, 7.0], [3.0, 7.0]) == 0.0
    e = np.e
    # ln(1+pred) - ln(1+y) = 1 and -2  ->  sqrt((1 + 4) / 2)
    assert F.rmsle([e - 1, 0.0], [0.0, e * e - 1]) == pytest.approx(np.sqrt(2.5), rel=1e-15)
    # symmetric in over- and under-estimation by the same factor of (1 + x)
    assert F.rmsle([2 * 11 - 1], [10.0]) == pytest.approx(F.rmsle([10.0], [2 * 11 - 1]), rel=1e-15)


def test_predict_is_the_model_of_the_evaluation(orc, F):
    """Same numbers as the per-candidate evaluation when theta is the job's own
    (float32-exact) parameter tuple, and the closed form on one GPU."""
    wl = workloads.paper_scale()
    dr, d, t, p = samples(orc, wl)
    for j in (0, 7, 33):
        th = wl.coef[j, list(F.THETA_COLUMNS)].astype(np.float64)
        thr, ti = F.predict(wl.coef[j], wl.ints[j], wl.env, th, d[j], t[j], p[j], dr.option[j], dr.cpus[j], True)
        for i in range(d.shape[1]):
            o = int(dr.option[j, i])
            _, terms = orc.eval_one(wl.coef[j], wl.ints[j], wl.bounds, wl.env, d[j, i], t[j, i], p[j, i], o >> 2, (o >> 1) & 1,
                                    o & 1, dr.cpus[j, i], np.float32(np.inf))
            assert thr[i] == terms["thr"] and ti[i] == terms["T_iter"]
    # one GPU, no options: T = n*(1 + k_bwd)*t_fwd_sample*mu + k_opt*P + k_const  (sync with T_dp = 0 is T_bwd)
    cf, it = wl.coef[0].copy(), wl.ints[0]
    th = np.array([1.75, 3.0, 2e-12, 1e-9, 2.0, 2.0, 0.125])
    n = it[1] // it[2]
    want_T = n * (1 + th[0]) * float(cf[4]) * it[2] + th[2] * float(cf[0]) + th[6]
    thr, ti = F.predict(cf, it, wl.env, th, [1], [1], [1], [0], [4], True)
    assert ti[0] == pytest.approx(want_T, rel=1e-14) and thr[0] == pytest.approx(it[1] / want_T, rel=1e-14)
    # invalid samples predict 0
    assert F.predict(cf, it, wl.env, th, [7, 1, 1], [1, 1, 1], [1, 5, 1], [0, 0, 16], [1, 1, 1]).tolist() == [0, 0, 0]


def test_minimum_over_one_repeated_run_is_the_spread_of_the_data(orc, F):
    """All samples are the same run: the model predicts one number for all of
    them, and the least RMSLE is the population standard deviation of
    ln(1 + y), reached where ln(1 + pred) is their mean.  The constant term can
    produce any slower prediction, so measurements slower than the start are
    matched that way."""
    wl = workloads.paper_scale()
    cf, it = wl.coef[3], wl.ints[3]
    th0 = wl.coef[3, list(F.THETA_COLUMNS)].astype(np.float64)
    S = 9
    d, t, p, o, c = [2] * S, [1] * S, [1] * S, [0] * S, [4] * S
    pred0 = F.predict(cf, it, wl.env, th0, d, t, p, o, c)[0]
    z = np.array([0.3, -0.2, 0.1, 0.05, -0.4, 0.25, 0.0, -0.1, 0.15])
    y = pred0 * 0.6 * np.exp(0.1 * z)                   # slower than predicted
    th, val, before = F.fit_one(cf, it, wl.env, th0, d, t, p, o, c, y)
    assert val == pytest.approx(np.std(np.log1p(y)), rel=1e-7)
    got = F.predict(cf, it, wl.env, th, d, t, p, o, c)[0]
    assert np.log1p(got) == pytest.approx(np.mean(np.log1p(y)), rel=1e-7)
    assert before > val


def test_exact_data_are_recovered(orc, F):
    wl = workloads.large().subset(np.arange(6))
    dr, d, t, p = samples(orc, wl)
    tb = orc.enumerate_plans(wl.ints, workloads.Bounds(g_max=128))
    for j in range(wl.n_jobs):
        true = wl.coef[j, list(F.THETA_COLUMNS)].astype(np.float64)
        y = F.predict(wl.coef[j], wl.ints[j], wl.env, true, d[j], t[j], p[j], dr.option[j], dr.cpus[j])
        assert np.all(y > 0)
        th0 = F.project(true * dr.start_factor[j])
        th, val, before = F.fit_one(wl.coef[j], wl.ints[j], wl.env, th0, d[j], t[j], p[j], dr.option[j], dr.cpus[j], y,
                                    start_offsets=dr.start_offsets)
        assert before > 1e-3 and val < 1e-9
        # the fitted model predicts other plans of the same kinds as the truth does (held-out runs)
        tr = tb.triples[tb.triple_off[j]:tb.triple_off[j + 1]]
        pick = np.linspace(0, len(tr) - 1, 40).astype(int)
        for o, c in ((0, 1), (6, 1), (13, 8), (11, 32)):
            a = F.predict(wl.coef[j], wl.ints[j], wl.env, th, tr[pick, 0], tr[pick, 1], tr[pick, 2], [o] * 40, [c] * 40)
            b = F.predict(wl.coef[j], wl.ints[j], wl.env, true, tr[pick, 0], tr[pick, 1], tr[pick, 2], [o] * 40, [c] * 40)
            assert np.max(np.abs(a - b) / b) < 1e-5


def test_noisy_fit_is_a_constrained_stationary_point_and_beats_the_truth(orc, F):
    wl = workloads.large().subset(np.arange(5))
    dr, d, t, p = samples(orc, wl)
    for j in range(wl.n_jobs):
        cf, it = wl.coef[j], wl.ints[j]
        true = cf[list(F.THETA_COLUMNS)].astype(np.float64)
        args = (d[j], t[j], p[j], dr.option[j], dr.cpus[j])
        y = F.predict(cf, it, wl.env, true, *args) * np.exp(0.05 * dr.noise_z[j])
        th0 = F.project(true * dr.start_factor[j])
        th, val, before = F.fit_one(cf, it, wl.env, th0, *args, y, start_offsets=dr.start_offsets)
        assert val <= F.rmsle(F.predict(cf, it, wl.env, true, *args), y) + 1e-12      # no worse than the generating parameters
        assert val <= before
        assert np.all(th >= 0) and np.all(th[F.IS_EXPONENT] >= 1) and np.all(th[F.IS_EXPONENT] <= F.K_MAX)
        # first-order conditions by central differences on the mean squared error, in relative steps:
        # zero slope inside the set, slope pointing out of the set on a bound
        def mse(theta):
            return F.rmsle(F.predict(cf, it, wl.env, theta, *args), y) ** 2
        for i in range(F.N_THETA):
            h = 1e-6 * (th[i] if th[i] > 0 else th0[i])
            up, dn = th.copy(), th.copy()
            up[i] += h
            dn[i] -= h
            lo, hi = (1.0, F.K_MAX) if F.IS_EXPONENT[i] else (0.0, np.inf)
            at_lo, at_hi = th[i] - lo <= 1e-9 * max(lo, th0[i]), hi - th[i] <= 1e-9 * hi
            if at_lo:
                slope = (mse(up) - mse(th)) / h * (th0[i] if lo == 0 else 1.0)
                assert slope >= -1e-7
            elif at_hi:
                slope = (mse(th) - mse(dn)) / h
                assert slope <= 1e-7
            else:
                slope = (mse(up) - mse(dn)) / (2 * h) * th[i]
                assert abs(slope) <= 2e-7, (j, i, slope)


def test_refit_threshold_leaves_good_models_alone(orc, F):
    wl = workloads.paper_scale()
    dr, d, t, p = samples(orc, wl)
    j = 2
    true = wl.coef[j, list(F.THETA_COLUMNS)].astype(np.float64)
    args = (d[j], t[j], p[j], dr.option[j], dr.cpus[j])
    y = F.predict(wl.coef[j], wl.ints[j], wl.env, true, *args) * np.exp(0.02 * dr.noise_z[j])
    th, val, before = F.fit_one(wl.coef[j], wl.ints[j], wl.env, true, *args, y, refit_threshold=0.1)
    assert np.array_equal(th, true) and val == before and 0 < before < 0.1
    th, val, before = F.fit_one(wl.coef[j], wl.ints[j], wl.env, true, *args, y, refit_threshold=0.001)
    assert val < before
