// Service-level support (paper Sec. 5.2, "Scheduling algorithm design"):
// the minimum demand of guaranteed jobs, and the evaluation of chosen points
// of the plan space (a guaranteed job's baseline is its original plan at its
// requested resources).
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int MINRES_THREADS = 256;
constexpr int POINT_THREADS = 256;

struct SlaReq {
    const uint32_t *guaranteed, *req_g, *req_c, *req_m;
    const float *base_thr;
};

// One wavefront per job.  Lanes take consecutive GPU counts (segments) of the
// job, so every (CPU level, memory tier) row is read coalesced; a lane keeps
// the first (level, tier) in ascending order that qualifies at its segment,
// and the lowest qualifying segment of the wavefront wins.
__global__ __launch_bounds__(MINRES_THREADS) void k_min_res(TableDev tb, GridDev grid, uint32_t jb, uint32_t je,
                                                            const float *__restrict__ best_thr, SlaReq R,
                                                            int32_t *__restrict__ min_seg,
                                                            uint32_t *__restrict__ min_c,
                                                            uint32_t *__restrict__ min_m) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t j = jb + blockIdx.x * (MINRES_THREADS / 64) + (threadIdx.x >> 6);
    if (j >= je) return;                                   // whole wavefront
    const uint32_t o = j - jb;
    int32_t out_s = -1;
    uint32_t out_c = 0, out_m = 0;
    if (R.guaranteed[j]) {
        const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
        const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
        const uint64_t jbase = (uint64_t)n_rows * (s0 - tb.seg_off[jb]);
        const uint32_t rg = R.req_g[j];
        const uint32_t c_req = R.req_c[j] < grid.n_cpu ? R.req_c[j] : grid.n_cpu - 1;
        const uint32_t m_req = R.req_m[j] < n_mem ? R.req_m[j] : n_mem - 1;
        const float base_thr = R.base_thr[j];
        // number of segments within the request (GPU counts ascend)
        uint32_t lo = 0, hi = ns;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (tb.seg_g[s0 + mid] <= rg) lo = mid + 1; else hi = mid;
        }
        const uint32_t n_ok = lo;
        if (n_ok > 0) {
            out_s = (int32_t)(n_ok - 1); out_c = c_req; out_m = m_req;   // the request itself unless less will do
            for (uint32_t base = 0; base < n_ok; base += 64) {
                const uint32_t s = base + lane;
                uint32_t mine = 0xFFFFFFFFu;               // (level << 8 | tier) of this lane's first hit
                if (s < n_ok) {
                    for (uint32_t c = 0; c <= c_req && mine == 0xFFFFFFFFu; ++c)
                        for (uint32_t m = 0; m <= m_req; ++m) {
                            const float v = best_thr[jbase + (uint64_t)(c * n_mem + m) * ns + s];
                            if (v > 0.f && v >= base_thr) { mine = (c << 8) | m; break; }
                        }
                }
                const unsigned long long hits = __ballot(mine != 0xFFFFFFFFu);
                if (hits) {
                    const uint32_t first = (uint32_t)__ffsll((long long)hits) - 1u;
                    const uint32_t cm = (uint32_t)__builtin_amdgcn_readlane((int)mine, (int)first);
                    out_s = (int32_t)(base + first); out_c = cm >> 8; out_m = cm & 255u;
                    break;
                }
            }
        }
    }
    if (lane == 0) { min_seg[o] = out_s; min_c[o] = out_c; min_m[o] = out_m; }
}

// One thread per point: the candidate's value exactly as the candidate
// evaluation computes it (same functions, same order).
template <bool WITH_FEAS>
__global__ __launch_bounds__(POINT_THREADS) void k_eval_points(JobDev jobs, TableDev tb, GridDev grid, rk_env env,
                                                               uint32_t n_jobs, uint32_t option_mask, uint64_t n_points,
                                                               const uint32_t *__restrict__ pt_job,
                                                               const uint32_t *__restrict__ pt_plan,
                                                               const uint32_t *__restrict__ pt_c,
                                                               const uint32_t *__restrict__ pt_m,
                                                               float *__restrict__ thr, uint8_t *__restrict__ feas) {
    const uint64_t i = (uint64_t)blockIdx.x * POINT_THREADS + threadIdx.x;
    if (i >= n_points) return;
    const uint32_t j = pt_job[i], plan = pt_plan[i], ci = pt_c[i], mi = pt_m[i];
    float out = 0.f;
    uint32_t why = RK_INFEASIBLE_STRUCT;
    bool valid = j < n_jobs && ci < grid.n_cpu && mi < grid.n_mem;
    uint32_t t0 = 0;
    if (valid) {
        t0 = tb.triple_off[j];
        valid = (plan >> 4) < tb.triple_off[j + 1] - t0;
    }
    if (valid) {
        const uint32_t o = plan & 15u, z = o >> 2, gc = (o >> 1) & 1u, off = o & 1u;
        const bool allowed = ((option_mask >> o) & 1u) && (!off || z >= 2);
        if (allowed) {
            const Job J = load_job(jobs, j);
            const Triple T = triple_terms(J, env, tb.triples[t0 + (plan >> 4)]);
            why = gpu_mem_fits(J, env, T, z, gc, off) ? 0u : RK_INFEASIBLE_GPU_MEM;
            if (!off) {
                if (!why) out = thr_plain(J, T, z, gc);
            } else {
                if (!(host_bytes_needed(J, T) <= tier_bytes(grid, mi, T.g))) why |= RK_INFEASIBLE_HOST_MEM;
                if (!why) {
                    const Offload O = offload_terms(J, env, T);
                    out = thr_offload(T, O, gc, swap_term(J, O, cpus_of(grid, ci, T.g)));
                }
            }
        }
    }
    thr[i] = out;
    if (WITH_FEAS) feas[i] = (uint8_t)why;
}


// ------------------------------------------------------------------ who is privileged when the loop runs
// Floors and states for Algorithm 1's Schedule loops from the service levels (paper Sec. 5.2: the guaranteed jobs whose
// demands are within their tenant's remaining quota are scheduled first; a job's quota usage is its minimum demand).
// One workgroup.  Running guaranteed jobs are charged first, all at once (a quota that cannot go below zero ends at
// max(0, quota - sum) whatever the order); the queued ones are gathered in job order, their tenants in LDS.  A
// wavefront per tenant then walks the list 64 entries at a time: a ballot finds the tenant's jobs among them, their
// demands are already in the lanes' registers, and only the quota arithmetic of those jobs runs one after another.
constexpr int PRIV_THREADS = 1024;

struct PrivArgs {
    TableDev tb;
    GridDev grid;
    uint32_t n_jobs, n_tenants;
    const uint32_t *guaranteed, *tenant, *quota_g, *quota_c;
    const int32_t *min_seg;
    const uint32_t *min_c;
    const uint8_t *state_in;     // may be null
    const int32_t *cur_seg;
    const uint32_t *cur_c;
    int32_t *floor_seg;
    uint32_t *floor_c;
    uint8_t *state_out;
    uint32_t *list;              // queued guaranteed jobs in job order: job, tenant (n_tenants: none), GPUs, CPUs
};

__global__ __launch_bounds__(PRIV_THREADS) void k_privileged(PrivArgs A) {
    __shared__ unsigned long long qg[RK_MAX_TENANTS], qc[RK_MAX_TENANTS];
    __shared__ uint32_t sh_scan[PRIV_THREADS / 64], sh_n;
    __shared__ uint16_t sh_tenant[RK_MAX_JOBS_PER_ROUND];   // tenant of every list entry (n_tenants: none)
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, J = A.n_jobs, T = A.n_tenants;
    if (tid < T) { qg[tid] = 0ull; qc[tid] = 0ull; }
    if (tid == 0) sh_n = 0u;
    __syncthreads();
    auto ns_of = [&](uint32_t j) { return A.tb.seg_off[j + 1] - A.tb.seg_off[j]; };
    auto has_min = [&](uint32_t j) { return A.min_seg[j] >= 0 && (uint32_t)A.min_seg[j] < ns_of(j) && A.tenant[j] < T; };
    auto level_of = [&](uint32_t j) { return A.min_c[j] < A.grid.n_cpu ? A.min_c[j] : A.grid.n_cpu - 1u; };
    auto holds = [&](uint32_t j) {
        const bool in = !A.state_in || A.state_in[j] == 0 || A.state_in[j] == 2;
        return in && A.cur_seg[j] >= 0 && (uint32_t)A.cur_seg[j] < ns_of(j) && A.cur_c[j] < A.grid.n_cpu;
    };
    // the running guaranteed jobs: their floors, and what they use of their tenants' quotas
    for (uint32_t base = 0; base < J; base += PRIV_THREADS) {
        const uint32_t j = base + tid;
        bool queued = false;
        uint32_t tn = T, g = 0, c = 0;
        if (j < J) {
            int32_t fs = -1;
            uint32_t fc = 0;
            const uint8_t st = A.state_in ? A.state_in[j] : (uint8_t)0;
            if (A.guaranteed[j]) {
                const bool with_min = has_min(j);
                if (with_min) {
                    g = A.tb.seg_g[A.tb.seg_off[j] + (uint32_t)A.min_seg[j]];
                    c = cpus_of(A.grid, level_of(j), g);
                    tn = A.tenant[j];
                }
                if (holds(j)) {
                    if (with_min) {
                        fs = A.min_seg[j]; fc = level_of(j);
                        atomicAdd(&qg[tn], (unsigned long long)g);
                        atomicAdd(&qc[tn], (unsigned long long)c);
                    }
                } else if (st == 0) {
                    queued = true;
                }
            }
            A.floor_seg[j] = fs; A.floor_c[j] = fc; A.state_out[j] = st;
        }
        // the queued ones of this batch go to the list, in job order
        uint32_t inc = queued ? 1u : 0u;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(inc, off, 64);
            if ((int)lane >= off) inc += o;
        }
        if (lane == 63) sh_scan[wave] = inc;
        __syncthreads();
        uint32_t before = sh_n, all = 0;
        for (uint32_t w = 0; w < PRIV_THREADS / 64; ++w) { if (w < wave) before += sh_scan[w]; all += sh_scan[w]; }
        if (queued) {
            uint32_t *e = A.list + 4 * (size_t)(before + inc - 1u);
            e[0] = j; e[1] = tn; e[2] = g; e[3] = c;
            sh_tenant[before + inc - 1u] = (uint16_t)tn;
        }
        __syncthreads();
        if (tid == 0) sh_n += all;
        __syncthreads();
    }
    const uint32_t n_queued = sh_n;
    for (uint32_t t = wave; t < T; t += PRIV_THREADS / 64) {
        const unsigned long long ug = qg[t], uc = qc[t], hg = A.quota_g[t], hc = A.quota_c[t];
        unsigned long long left_g = hg > ug ? hg - ug : 0ull, left_c = hc > uc ? hc - uc : 0ull;   // the same in all lanes
        for (uint32_t base = 0; base < n_queued; base += 64u) {
            const uint32_t i = base + lane;
            const bool mine = i < n_queued && sh_tenant[i] == t;
            unsigned long long todo = __ballot(mine);
            if (!todo) continue;
            uint32_t j = 0, g = 0, c = 0;
            if (mine) { j = A.list[4 * (size_t)i]; g = A.list[4 * (size_t)i + 2]; c = A.list[4 * (size_t)i + 3]; }
            bool granted = false;
            while (todo) {                                   // this tenant's jobs among the 64, in job order
                const int b = __ffsll((long long)todo) - 1;
                todo &= todo - 1ull;
                const uint32_t gb = __shfl(g, b, 64), cb = __shfl(c, b, 64);
                const bool fits = gb <= left_g && cb <= left_c;
                if (fits) { left_g -= gb; left_c -= cb; }
                if ((int)lane == b) granted = fits;
            }
            if (mine) {
                if (granted) { A.floor_seg[j] = A.min_seg[j]; A.floor_c[j] = level_of(j); }
                else A.state_out[j] = 1;
            }
        }
    }
    // queued guaranteed jobs without a minimum demand or with an unknown tenant wait
    for (uint32_t i = tid; i < n_queued; i += PRIV_THREADS)
        if (A.list[4 * (size_t)i + 1] >= T) A.state_out[A.list[4 * (size_t)i]] = 1;
}

}  // namespace

int32_t rk_launch_min_res(rk_ctx *ctx, const TableDev &tb, const rk_alloc_grid *grid, uint32_t jb, uint32_t je,
                          const float *best_thr, const rk_sla *sla, int32_t *min_seg, uint32_t *min_c,
                          uint32_t *min_m) {
    if (je <= jb) return RK_OK;
    const uint32_t per_block = MINRES_THREADS / 64;
    const uint32_t blocks = (je - jb + per_block - 1) / per_block;
    const SlaReq R = {sla->guaranteed, sla->req_g, sla->req_c, sla->req_m, sla->base_thr};
    k_min_res<<<blocks, MINRES_THREADS, 0, ctx->stream>>>(tb, grid_dev(grid), jb, je, best_thr, R, min_seg, min_c, min_m);
    RK_CHECK_LAUNCH(ctx, "k_min_res");
    return RK_OK;
}

extern "C" {

int32_t rk_min_res(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid, uint32_t jb, uint32_t je,
                   const float *best_thr, const rk_sla *sla, int32_t *min_seg, uint32_t *min_c, uint32_t *min_m) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (je == jb) return RK_OK;
    if (!best_thr || !min_seg || !min_c || !min_m) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (!sla || !sla->guaranteed || !sla->req_g || !sla->req_c || !sla->req_m || !sla->base_thr)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "sla: guaranteed, request or baseline array is null");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    return rk_launch_min_res(ctx, table_dev(table), grid, jb, je, best_thr, sla, min_seg, min_c, min_m);
}

int32_t rk_eval_points(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                       const rk_env *env, uint64_t n_points, const uint32_t *pt_job, const uint32_t *pt_plan,
                       const uint32_t *pt_c, const uint32_t *pt_m, float *thr, uint8_t *feas) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs is null");
    if ((rc = rk_check_table(ctx, table, 0, jobs->n_jobs))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if ((rc = rk_check_env(ctx, env))) return rc;
    if (n_points == 0) return RK_OK;
    if (!pt_job || !pt_plan || !pt_c || !pt_m || !thr) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (n_points > 0x7FFFFFFFull * POINT_THREADS) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "too many points for one call");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    const unsigned blocks = (unsigned)((n_points + POINT_THREADS - 1) / POINT_THREADS);
    if (feas)
        k_eval_points<true><<<blocks, POINT_THREADS, 0, ctx->stream>>>(job_dev(jobs), table_dev(table), grid_dev(grid), *env,
                                                                      jobs->n_jobs, table->option_mask, n_points, pt_job,
                                                                      pt_plan, pt_c, pt_m, thr, feas);
    else
        k_eval_points<false><<<blocks, POINT_THREADS, 0, ctx->stream>>>(job_dev(jobs), table_dev(table), grid_dev(grid), *env,
                                                                       jobs->n_jobs, table->option_mask, n_points, pt_job,
                                                                       pt_plan, pt_c, pt_m, thr, nullptr);
    RK_CHECK_LAUNCH(ctx, "k_eval_points");
    return RK_OK;
}

int32_t rk_privileged(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid, const rk_sla *sla,
                      const int32_t *min_seg, const uint32_t *min_c, const rk_job_state *held, int32_t *floor_seg,
                      uint32_t *floor_c, uint8_t *state_out) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, 0, table ? table->n_jobs : 0))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    const uint32_t J = table->n_jobs;
    if (J == 0) return RK_OK;
    if (!sla || !sla->guaranteed || !sla->tenant || (sla->n_tenants > 0 && (!sla->quota_g || !sla->quota_c)))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "sla: guaranteed, tenant or quota array is null");
    if (sla->n_tenants > RK_MAX_TENANTS) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than %u tenants", RK_MAX_TENANTS);
    if (!min_seg || !min_c || !held || !held->cur_seg || !held->cur_c || !floor_seg || !floor_c || !state_out)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    PrivArgs A;
    A.tb = table_dev(table); A.grid = grid_dev(grid); A.n_jobs = J; A.n_tenants = sla->n_tenants;
    A.guaranteed = sla->guaranteed; A.tenant = sla->tenant; A.quota_g = sla->quota_g; A.quota_c = sla->quota_c;
    A.min_seg = min_seg; A.min_c = min_c;
    A.state_in = held->state; A.cur_seg = held->cur_seg; A.cur_c = held->cur_c;
    A.floor_seg = floor_seg; A.floor_c = floor_c; A.state_out = state_out;
    if ((rc = rk_scratch(ctx, SL_PRIV_LIST, (size_t)J * 16, (void **)&A.list))) return rc;
    k_privileged<<<1, PRIV_THREADS, 0, ctx->stream>>>(A);
    RK_CHECK_LAUNCH(ctx, "k_privileged");
    return RK_OK;
}

}  // extern "C"
