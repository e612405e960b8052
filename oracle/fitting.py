"""Model fitting on the CPU oracle (paper Sec. 4, "Continuous model fitting").

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.

The seven fittable parameters of Table 1 (k_bwd, k_sync, k_opt, k_opt_off,
k_off, k_swap, k_const) are chosen to minimise the root mean squared
logarithmic error between the model's prediction and the measured throughputs
of sampled test runs.  The paper names the objective, not the minimiser; here
the objective is written out plainly and handed to a library least-squares
routine (scipy, float64, finite-difference Jacobian), started from the current
parameters and from a few perturbed copies that the caller supplies.

Readings (the paper is silent):
  * the error is taken on throughput, RMSLE = sqrt(mean((ln(1+pred) - ln(1+y))^2));
  * feasible set: k_bwd, k_opt, k_opt_off, k_const >= 0 and the three overlap
    exponents in [1, 32] (k = 1 is no overlap; at k = 32 the overlap function is
    within 2.2 % of the maximum of its arguments, and the definition
    (x^k + y^k)^(1/k) can still be evaluated literally in float64 for every
    time between 1e-9 s and 1e9 s);
  * a fit is only redone when its current error exceeds a threshold (the
    online update of the paper).
The search variables are q_i = theta_i / theta0_i for the four scales (so that
finite-difference steps make sense whatever the unit) and v = 1/k for the
exponents; this changes nothing about the feasible set.

Parity status: the objective is pinned (closed forms in the tests), exact data
are recovered, and the result satisfies the first-order conditions.  The
problem has several local minima on noisy data, so which one a minimiser ends
in is PARITY UNPINNED.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import _env, _p, lib

N_THETA = 7
IS_EXPONENT = np.array([0, 1, 0, 0, 1, 1, 0], bool)     # k_sync, k_off, k_swap
THETA_COLUMNS = (5, 6, 7, 8, 9, 10, 11)                 # their columns in the 17-coefficient job descriptor
K_MAX = 32.0


def project(theta):
    """Nearest point of the feasible set."""
    theta = np.asarray(theta, np.float64)
    return np.where(IS_EXPONENT, np.clip(theta, 1.0, K_MAX), np.maximum(theta, 0.0))


def predict(coef_row, ints_row, env, theta, d, t, p, option, cpus, want_t_iter=False, mu_shift=None):
    """Predicted throughput of the sample runs under the parameters theta (float64)."""
    cf = np.ascontiguousarray(coef_row, dtype=np.float32)
    it = np.ascontiguousarray(ints_row, dtype=np.uint32)
    th = np.ascontiguousarray(theta, dtype=np.float64)
    assert th.shape == (N_THETA,)
    u32 = lambda a: np.ascontiguousarray(a, dtype=np.uint32)
    d, t, p, option, cpus = u32(d), u32(t), u32(p), u32(option), u32(cpus)
    mu_shift = None if mu_shift is None else u32(mu_shift)
    n = len(d)
    thr = np.zeros(n, np.float64)
    ti = np.zeros(n, np.float64) if want_t_iter else None
    e = _env(env)
    rc = lib().ork_predict_f64(_p(cf), _p(it), C.byref(e), _p(th), C.c_uint32(n), _p(d), _p(t), _p(p), _p(mu_shift),
                               _p(option), _p(cpus), _p(thr), _p(ti))
    assert rc == 0
    return (thr, ti) if want_t_iter else thr


def rmsle(pred, y):
    pred, y = np.asarray(pred, np.float64), np.asarray(y, np.float64)
    if pred.size == 0:
        return 0.0
    return float(np.sqrt(np.mean((np.log1p(pred) - np.log1p(y)) ** 2)))


def fit_one(coef_row, ints_row, env, theta0, d, t, p, option, cpus, y, refit_threshold=0.0, start_offsets=None):
    """Minimise the RMSLE over the feasible set, starting from theta0 and from
    theta0 with scales multiplied by exp(offset) and 1/k multiplied by
    exp(offset) for each row of start_offsets ([R][7], drawn by the caller); the
    best result wins, the earlier start on ties.
    Returns (theta, rmsle, rmsle at the projected theta0)."""
    from scipy.optimize import least_squares
    y = np.asarray(y, np.float64)
    logy = np.log1p(y)
    theta0 = project(theta0)
    scale = np.where(IS_EXPONENT, 1.0, np.where(theta0 > 0, theta0, 1.0))
    lower = np.where(IS_EXPONENT, 1.0 / K_MAX, 0.0)
    upper = np.where(IS_EXPONENT, 1.0, np.inf)

    def theta_of(q):
        return np.where(IS_EXPONENT, 1.0 / q, q * scale)

    def q_of(theta):
        return np.where(IS_EXPONENT, 1.0 / theta, theta / scale)

    def residuals(q):
        return np.log1p(predict(coef_row, ints_row, env, theta_of(q), d, t, p, option, cpus)) - logy

    before = rmsle(predict(coef_row, ints_row, env, theta0, d, t, p, option, cpus), y)
    if len(y) == 0 or before <= refit_threshold:
        return theta0, before, before
    q0 = q_of(theta0)
    starts = [q0] + ([] if start_offsets is None else [np.clip(q0 * np.exp(np.asarray(o, np.float64)), lower, upper)
                                                       for o in start_offsets])
    best_q, best = q0, before
    for start in starts:
        inside = np.clip(start, lower + 1e-12, np.where(np.isfinite(upper), upper - 1e-12, np.inf))   # strictly interior
        sol = least_squares(residuals, inside, jac="3-point", method="trf", bounds=(lower, upper),
                            xtol=1e-15, ftol=1e-15, gtol=1e-15, max_nfev=2000)
        val = float(np.sqrt(np.mean(sol.fun ** 2)))
        if val < best:
            best_q, best = sol.x, val
    return theta_of(best_q), best, before
