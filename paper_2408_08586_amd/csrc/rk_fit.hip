// Model fitting (paper Sec. 4, "Continuous model fitting"): the seven
// fittable parameters of every model type are chosen to minimise the root mean
// squared logarithmic error between Eq. 1 and measured runs.
//
// A group of W lanes (W = 8..64, the smallest power of two that holds a
// model's runs) fits one model; lane i holds run i.  Everything of a run that
// does not depend on the parameters is computed once.  One iteration of the
// projected Levenberg-Marquardt method evaluates the run's residual and its
// seven derivatives (analytic) at the trial point, sums the normal equations
// over the group with lane shuffles, and every lane solves the same 7x7 system
// by Cholesky factorisation.  All control flow is uniform over the wavefront
// (groups that have finished idle under a predicate) so that the shuffles are
// always executed by every lane.  float64 throughout.
#include <type_traits>

#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int FIT_THREADS = 256;
constexpr int NP = RK_FIT_PARAMS;
enum { TH_BWD, TH_SYNC, TH_OPT, TH_OPT_OFF, TH_OFF, TH_SWAP, TH_CONST };

__device__ __forceinline__ bool is_exponent(int i) { return i == TH_SYNC || i == TH_OFF || i == TH_SWAP; }

struct FitArgs {
    JobDev jobs;
    rk_env env;
    uint32_t n_fits;
    const uint32_t *sample_off, *triple, *option, *cpus;
    const float *thr;
    uint32_t max_iter, n_starts;
    double refit_threshold;
    double offsets[RK_FIT_MAX_STARTS][NP];
    rk_fit_result out;
};

// Overlap of two stages (Sec. 4.3), (x^k + y^k)^(1/k) as M*(1 + r^k)^(1/k) with
// r = min/max, with its derivatives by the first argument and by k.
__device__ __forceinline__ void overlap(double k, double x, double y, double &f, double &fx, double &fk) {
    const double M = fmax(x, y), m = fmin(x, y);
    if (!(m > 0.0)) { f = M; fx = x >= y ? 1.0 : 0.0; fk = 0.0; return; }
    const double r = m / M, lr = log(r);
    const double rk = exp(k * lr);
    const double L = log1p(rk);
    f = M * exp(L / k);
    const double g = exp(L * (1.0 / k - 1.0));            // derivative by the larger argument
    fx = x >= y ? g : g * rk / r;
    fk = f * (rk * lr / ((1.0 + rk) * k) - L / (k * k));
}

// What a run contributes that does not depend on the parameters.
struct Run {
    double Tfwd, gc, aTfwd, am1, Tdp, Tconst, opt_scale, Toff, logy, b;
    bool off, valid;
};

__device__ Run load_run(const FitArgs &A, uint32_t j, uint32_t i) {
    Run R = {};
    const uint32_t packed = A.triple[i], o = A.option[i], c = A.cpus[i];
    const double d = RK_TRIPLE_D(packed), t = RK_TRIPLE_T(packed), p = RK_TRIPLE_P(packed);
    const uint32_t di = RK_TRIPLE_D(packed), ti = RK_TRIPLE_T(packed), pi = RK_TRIPLE_P(packed);
    const uint32_t z = o >> 2, gc = (o >> 1) & 1u, off = o & 1u;
    const uint32_t layers = A.jobs.layers[j], gb = A.jobs.gbatch[j], mu = A.jobs.mbatch[j] << RK_TRIPLE_V(packed);
    R.logy = log1p((double)A.thr[i]);
    R.valid = di > 0 && pi > 0 && o < 16u && mu > 0 && gb % (di * mu) == 0 && layers % pi == 0 && !(off && z < 2) &&
              !(off && c == 0);
    if (!R.valid) return R;
    const double P = A.jobs.P_bytes[j], s = A.jobs.seq[j], h = A.jobs.hidden[j], eb = A.jobs.elem_bytes[j];
    const double tfs = A.jobs.t_fwd_sample[j], b = gb, l = layers;
    const double n = (double)(gb / (di * mu));
    const bool pp = pi > 1;
    const double m = pp ? n : 1.0, a = pp ? 1.0 : n;
    R.b = b;
    R.Tfwd = tfs * mu / (t * p) * (m + p - 1.0);
    R.gc = gc;
    R.aTfwd = a * R.Tfwd;
    R.am1 = pp ? 0.0 : a - 1.0;
    const uint32_t N = A.env.gpus_per_node;
    const double bi = A.env.B_intra, bx = A.env.B_inter;
    double Bdp = bi, Btp = bi, Bpp = bi;
    if ((unsigned long long)di * ti * pi > N) {
        Btp = (N % ti == 0) ? bi : bx;
        Bdp = (N % ((unsigned long long)ti * di) == 0) ? bi : bx;
        Bpp = bx;
    }
    const double Vdp = di > 1 ? P * 2.0 * (d - 1.0) / (d * t * p) : 0.0;
    const double Vtp = ti > 1 ? eb * 4.0 * 2.0 * (t - 1.0) * b * s * h * l / (d * t) : 0.0;
    const double Vpp = pp ? eb * 2.0 * p * b * s * h / (d * t) : 0.0;
    R.Tdp = Vdp / Bdp;
    R.Tconst = Vtp / Btp + (pp ? Vpp / Bpp : 0.0);
    const double Psi = P / (t * p);
    R.off = off != 0;
    R.opt_scale = off ? Psi / (d * (double)c) : Psi / (z >= 1 ? d : 1.0);
    R.Toff = Psi / (d * (double)A.env.B_pcie);
    return R;
}

// Residual ln(1+pred) - ln(1+y) of a run at the search point x (scales, 1/k)
// and its derivatives by x.
__device__ __forceinline__ void residual(const Run &R, const double (&x)[NP], double &res, double (&J)[NP]) {
#pragma unroll
    for (int i = 0; i < NP; ++i) J[i] = 0.0;
    if (!R.valid) { res = -R.logy; return; }
    const double ks = 1.0 / x[TH_SYNC], kf = 1.0 / x[TH_OFF], kw = 1.0 / x[TH_SWAP];
    const double Tb = x[TH_BWD] * R.Tfwd + R.gc * R.Tfwd;
    double sync, sx, sk;
    overlap(ks, Tb, R.Tdp, sync, sx, sk);
    double T = R.aTfwd + R.am1 * Tb + sync + R.Tconst + x[TH_CONST];
    double G[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) G[i] = 0.0;
    G[TH_BWD] = R.Tfwd * (R.am1 + sx);
    G[TH_SYNC] = sk;
    G[TH_CONST] = 1.0;
    if (R.off) {
        const double Topt = x[TH_OPT_OFF] * R.opt_scale;
        double f1, f1x, f1k, f2, f2x, f2k;
        overlap(kf, R.Tdp, R.Toff, f1, f1x, f1k);
        overlap(kw, Topt, R.Toff, f2, f2x, f2k);
        T += f1 + f2;
        G[TH_OPT_OFF] = f2x * R.opt_scale;
        G[TH_OFF] = f1k;
        G[TH_SWAP] = f2k;
    } else {
        T += x[TH_OPT] * R.opt_scale;
        G[TH_OPT] = R.opt_scale;
    }
    const double thr = R.b / T;
    res = log1p(thr) - R.logy;
    const double w = -(thr / (T * (1.0 + thr)));
    // chain rule to the search variables: k = 1/v, dk/dv = -k^2
    J[TH_BWD] = w * G[TH_BWD];
    J[TH_SYNC] = w * G[TH_SYNC] * (-ks * ks);
    J[TH_OPT] = w * G[TH_OPT];
    J[TH_OPT_OFF] = w * G[TH_OPT_OFF];
    J[TH_OFF] = w * G[TH_OFF] * (-kf * kf);
    J[TH_SWAP] = w * G[TH_SWAP] * (-kw * kw);
    J[TH_CONST] = w * G[TH_CONST];
}

// Sum over the group of W lanes, the same bits in every lane (both partners of every step add the same two values).
// Inside a row of 16 lanes the partners are reached by data-parallel-primitive moves (neighbour, neighbour pair,
// mirrored halves of 8, mirrored halves of 16), beyond it by shuffles; all 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = (uint32_t)b, hi = (uint32_t)(b >> 32);
    const uint32_t l2 = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, 0xF, 0xF, false);
    const uint32_t h2 = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, 0xF, 0xF, false);
    return __longlong_as_double((long long)(((unsigned long long)h2 << 32) | l2));
}
template <int W>
__device__ __forceinline__ double group_sum(double v) {
    if (W >= 2) v += dpp_f64<0xB1>(v);                      // quad_perm [1,0,3,2]
    if (W >= 4) v += dpp_f64<0x4E>(v);                      // quad_perm [2,3,0,1]
    if (W >= 8) v += dpp_f64<0x141>(v);                     // row_half_mirror
    if (W >= 16) v += dpp_f64<0x140>(v);                    // row_mirror
#pragma unroll
    for (int off = 16; off < W; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Normal equations of the group: A = J^T J (upper triangle, row-major packed), g = J^T r, F = r^T r.
struct Normal { double A[NP * (NP + 1) / 2], g[NP], F; };

__device__ __forceinline__ int tri(int i, int j) { return i * NP - i * (i - 1) / 2 + (j - i); }   // i <= j

template <int W>
__device__ __forceinline__ void normal_equations(double res, const double (&J)[NP], Normal &Nq) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
#pragma unroll
        for (int j = i; j < NP; ++j) Nq.A[tri(i, j)] = group_sum<W>(J[i] * J[j]);
        Nq.g[i] = group_sum<W>(J[i] * res);
    }
    Nq.F = group_sum<W>(res * res);
}

// Solves (A + lam*diag(D)) delta = -g on the free variables (fixed ones get 0).
// Returns false when the matrix is not positive definite.
__device__ __forceinline__ bool solve_step(const Normal &Nq, const double (&D)[NP], double lam, const bool (&fixed)[NP],
                                           double (&delta)[NP]) {
    double M[NP][NP], rhs[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const double a = i <= j ? Nq.A[tri(i, j)] : Nq.A[tri(j, i)];
            M[i][j] = (fixed[i] || fixed[j]) ? (i == j ? 1.0 : 0.0) : (i == j ? a + lam * D[i] : a);
        }
        rhs[i] = fixed[i] ? 0.0 : -Nq.g[i];
    }
    bool ok = true;
#pragma unroll
    for (int j = 0; j < NP; ++j) {                        // Cholesky, lower triangle in place
        double s = M[j][j];
#pragma unroll
        for (int k = 0; k < j; ++k) s -= M[j][k] * M[j][k];
        ok = ok && s > 0.0 && isfinite(s);
        const double piv = sqrt(s > 0.0 ? s : 1.0);
        M[j][j] = piv;
#pragma unroll
        for (int i = j + 1; i < NP; ++i) {
            double v = M[i][j];
#pragma unroll
            for (int k = 0; k < j; ++k) v -= M[i][k] * M[j][k];
            M[i][j] = v / piv;
        }
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) {                        // forward
        double v = rhs[i];
#pragma unroll
        for (int k = 0; k < i; ++k) v -= M[i][k] * rhs[k];
        rhs[i] = v / M[i][i];
    }
#pragma unroll
    for (int i = NP - 1; i >= 0; --i) {                   // backward
        double v = rhs[i];
#pragma unroll
        for (int k = i + 1; k < NP; ++k) v -= M[k][i] * delta[k];
        delta[i] = v / M[i][i];
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) ok = ok && isfinite(delta[i]);
    return ok;
}

__device__ __forceinline__ double lower_of(int i) { return is_exponent(i) ? 1.0 / RK_FIT_K_MAX : 0.0; }
__device__ __forceinline__ double upper_of(int i) { return is_exponent(i) ? 1.0 : __builtin_huge_val(); }
__device__ __forceinline__ double clip(int i, double v) { return fmin(fmax(v, lower_of(i)), upper_of(i)); }

template <int W>
__global__ __launch_bounds__(FIT_THREADS) void k_fit(FitArgs A) {
    constexpr double GTOL = 1e-14, XTOL = 1e-13, KICK_TO = 0.3;
    const uint32_t lane = threadIdx.x % W;
    const uint32_t fit = blockIdx.x * (FIT_THREADS / W) + threadIdx.x / W;
    const bool have_fit = fit < A.n_fits;
    uint32_t s0 = 0, S = 0;
    if (have_fit) { s0 = A.sample_off[fit]; S = A.sample_off[fit + 1] - s0; }
    Run R = {};
    if (lane < S) R = load_run(A, fit, s0 + lane);
    // a lane without a run contributes nothing at all
    const bool has_run = lane < S;

    double x0[NP];
    if (have_fit) {
        x0[TH_BWD] = A.jobs.k_bwd[fit]; x0[TH_SYNC] = A.jobs.k_sync[fit]; x0[TH_OPT] = A.jobs.k_opt[fit];
        x0[TH_OPT_OFF] = A.jobs.k_opt_off[fit]; x0[TH_OFF] = A.jobs.k_off[fit]; x0[TH_SWAP] = A.jobs.k_swap[fit];
        x0[TH_CONST] = A.jobs.k_const[fit];
    } else {
#pragma unroll
        for (int i = 0; i < NP; ++i) x0[i] = 1.0;
    }
    double th0[NP];                                       // the current parameters on the feasible set
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        th0[i] = is_exponent(i) ? fmin(fmax(x0[i], 1.0), RK_FIT_K_MAX) : fmax(x0[i], 0.0);
        if (!(th0[i] == th0[i])) th0[i] = is_exponent(i) ? 1.0 : 0.0;   // NaN in the descriptor
        x0[i] = is_exponent(i) ? 1.0 / th0[i] : th0[i];   // exponents are searched as 1/k
    }

    auto evaluate = [&](const double (&x)[NP], Normal &Nq) {
        double res = 0.0, J[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) J[i] = 0.0;
        if (has_run) residual(R, x, res, J);
        normal_equations<W>(res, J, Nq);
    };

    Normal cur;
    evaluate(x0, cur);
    const double inv_S = S ? 1.0 / (double)S : 0.0;
    const double before = sqrt(cur.F * inv_S);
    const bool too_many = S > (uint32_t)W;                // more runs than the caller announced: left alone, flagged
    const bool refit = have_fit && S > 0 && !too_many && before > A.refit_threshold;

    double best_x[NP], best_F = cur.F;
#pragma unroll
    for (int i = 0; i < NP; ++i) best_x[i] = x0[i];
    uint32_t iters = 0;
    bool improved = false;

    // One descent from x; `enabled` is the group's predicate (the loops run for
    // the whole wavefront).  A better end point replaces the best one.
    auto descend = [&](double (&x)[NP], bool enabled) {
        evaluate(x, cur);
        double D[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) D[i] = cur.A[tri(i, i)];
        double lam = 1e-3, nu = 2.0;
        bool active = enabled;
        for (uint32_t it = 0; it < A.max_iter; ++it) {
            if (!__any(active)) break;
            if (active) ++iters;
            bool fixed[NP];
            double worst = 0.0;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                D[i] = fmax(D[i], cur.A[tri(i, i)]);
                fixed[i] = (x[i] <= lower_of(i) && cur.g[i] > 0.0) || (x[i] >= upper_of(i) && cur.g[i] < 0.0) || !(D[i] > 0.0);
                if (!fixed[i]) worst = fmax(worst, fabs(cur.g[i]) / sqrt(D[i]));
            }
            const double scale = fmax(sqrt(cur.F), 1e-300);
            const bool converged = worst <= GTOL * scale;
            double delta[NP];
            const bool ok = solve_step(cur, D, lam, fixed, delta);
            double xn[NP], de[NP], moved = 0.0;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                xn[i] = ok ? clip(i, x[i] + delta[i]) : x[i];
                de[i] = xn[i] - x[i];
                moved = fmax(moved, fabs(de[i]) * sqrt(fmax(D[i], 0.0)));
            }
            const bool small = ok && moved <= XTOL * scale;
            // the trial point: residual and derivatives of the lane's run, and the group's error there (every lane of the
            // wavefront, finished groups too); its normal equations replace the current ones below, where it is accepted
            double res_t = 0.0, J_t[NP];
#pragma unroll
            for (int i = 0; i < NP; ++i) J_t[i] = 0.0;
            if (has_run) residual(R, xn, res_t, J_t);
            const double F_t = group_sum<W>(res_t * res_t);
            double pred = 0.0;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                double Ad = 0.0;
#pragma unroll
                for (int j = 0; j < NP; ++j) Ad += (i <= j ? cur.A[tri(i, j)] : cur.A[tri(j, i)]) * de[j];
                pred -= de[i] * (2.0 * cur.g[i] + Ad);
            }
            const bool go = active && !converged && !small;
            const bool accept = go && ok && F_t < cur.F && pred > 0.0;
            if (accept) {
                const double rho = (cur.F - F_t) / pred, q = 2.0 * rho - 1.0;
                lam = fmax(lam * fmax(1.0 / 3.0, 1.0 - q * q * q), 1e-15);
                nu = 2.0;
#pragma unroll
                for (int i = 0; i < NP; ++i) x[i] = xn[i];
            } else if (go) {
                lam *= nu;
                nu *= 2.0;
                if (lam > 1e20) active = false;
            }
            if (converged || small) active = false;
            // (the sums run in every lane; a group keeps its own where it did not accept)
#pragma unroll
            for (int i = 0; i < NP; ++i) {
#pragma unroll
                for (int j = i; j < NP; ++j) {
                    const double a = group_sum<W>(J_t[i] * J_t[j]);
                    cur.A[tri(i, j)] = accept ? a : cur.A[tri(i, j)];
                }
                const double g = group_sum<W>(J_t[i] * res_t);
                cur.g[i] = accept ? g : cur.g[i];
            }
            cur.F = accept ? F_t : cur.F;
        }
        if (enabled && cur.F < best_F) {
            best_F = cur.F;
            improved = true;
#pragma unroll
            for (int i = 0; i < NP; ++i) best_x[i] = x[i];
        }
    };

    for (uint32_t start = 0; start <= A.n_starts; ++start) {
        double x[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) x[i] = start == 0 ? x0[i] : clip(i, x0[i] * exp(A.offsets[start - 1][i]));
        descend(x, refit);
    }
    // An overlap exponent that ended on a bound sits on a plateau (at k = 32 the
    // overlap function no longer feels k): try again from the best point with
    // that exponent moved back inside, twice over the three exponents.
    auto kick = [&](auto which) {
        constexpr int i = decltype(which)::value;
        double x[NP];
#pragma unroll
        for (int k = 0; k < NP; ++k) x[k] = best_x[k];
        const bool on_bound = x[i] <= lower_of(i) * (1.0 + 1e-9) || x[i] >= 1.0 - 1e-9;
        x[i] = KICK_TO;
        descend(x, refit && on_bound);
    };
    for (int round = 0; round < 2; ++round) {
        kick(std::integral_constant<int, TH_SYNC>{});
        kick(std::integral_constant<int, TH_OFF>{});
        kick(std::integral_constant<int, TH_SWAP>{});
    }

    if (have_fit && lane == 0) {
        double th[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) th[i] = !improved ? th0[i] : (is_exponent(i) ? 1.0 / best_x[i] : best_x[i]);
        const rk_fit_result &o = A.out;
        if (o.k_bwd) o.k_bwd[fit] = (float)th[TH_BWD];
        if (o.k_sync) o.k_sync[fit] = (float)th[TH_SYNC];
        if (o.k_opt) o.k_opt[fit] = (float)th[TH_OPT];
        if (o.k_opt_off) o.k_opt_off[fit] = (float)th[TH_OPT_OFF];
        if (o.k_off) o.k_off[fit] = (float)th[TH_OFF];
        if (o.k_swap) o.k_swap[fit] = (float)th[TH_SWAP];
        if (o.k_const) o.k_const[fit] = (float)th[TH_CONST];
        if (o.theta) {
#pragma unroll
            for (int i = 0; i < NP; ++i) o.theta[(size_t)fit * NP + i] = th[i];
        }
        if (o.rmsle_before) o.rmsle_before[fit] = (float)before;
        if (o.rmsle_after) o.rmsle_after[fit] = (float)sqrt(best_F * inv_S);
        if (o.iters) o.iters[fit] = too_many ? 0xFFFFFFFFu : iters;
    }
}

template <int W>
void launch_fit(const FitArgs &A, hipStream_t s) {
    const uint32_t per_block = FIT_THREADS / W;
    k_fit<W><<<(A.n_fits + per_block - 1) / per_block, FIT_THREADS, 0, s>>>(A);
}

}  // namespace

extern "C" int32_t rk_fit_models(rk_ctx *ctx, const rk_jobs *jobs, const rk_env *env, const rk_samples *samples,
                                 const rk_fit_options *options, const rk_fit_result *result) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!jobs || !samples || !options || !result) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if ((rc = rk_check_env(ctx, env))) return rc;
    if (jobs->n_jobs == 0) return RK_OK;
    if (!samples->sample_off || !samples->triple || !samples->option || !samples->cpus || !samples->thr)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "samples: null array");
    if (!jobs->P_bytes || !jobs->seq || !jobs->hidden || !jobs->elem_bytes || !jobs->t_fwd_sample || !jobs->k_bwd ||
        !jobs->k_sync || !jobs->k_opt || !jobs->k_opt_off || !jobs->k_off || !jobs->k_swap || !jobs->k_const ||
        !jobs->layers || !jobs->gbatch || !jobs->mbatch)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs: null array");
    if (samples->max_samples > RK_FIT_MAX_SAMPLES)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u runs per model, at most %u", samples->max_samples, RK_FIT_MAX_SAMPLES);
    if (options->n_starts > RK_FIT_MAX_STARTS)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u extra starting points, at most %u", options->n_starts, RK_FIT_MAX_STARTS);
    if (options->n_starts > 0 && !options->start_offsets) return rk_fail(ctx, RK_ERR_INVALID_ARG, "start_offsets is null");
    if (!(options->refit_threshold >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "refit_threshold negative or NaN");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    FitArgs A;
    A.jobs = job_dev(jobs);
    A.env = *env;
    A.n_fits = jobs->n_jobs;
    A.sample_off = samples->sample_off; A.triple = samples->triple; A.option = samples->option;
    A.cpus = samples->cpus; A.thr = samples->thr;
    A.max_iter = options->max_iter; A.n_starts = options->n_starts;
    A.refit_threshold = (double)options->refit_threshold;
    for (uint32_t s = 0; s < RK_FIT_MAX_STARTS; ++s)
        for (int i = 0; i < NP; ++i) {
            const double v = s < options->n_starts ? options->start_offsets[(size_t)s * NP + i] : 0.0;
            if (!(v == v) || v > 700.0 || v < -700.0) return rk_fail(ctx, RK_ERR_INVALID_ARG, "start offset out of range");
            A.offsets[s][i] = v;
        }
    A.out = *result;
    const uint32_t ms = samples->max_samples;
    if (ms <= 8) launch_fit<8>(A, ctx->stream);
    else if (ms <= 16) launch_fit<16>(A, ctx->stream);
    else if (ms <= 32) launch_fit<32>(A, ctx->stream);
    else launch_fit<64>(A, ctx->stream);
    RK_CHECK_LAUNCH(ctx, "k_fit");
    return RK_OK;
}
