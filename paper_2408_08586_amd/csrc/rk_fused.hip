// Fused path: evaluation (paper Sec. 4), best plan per segment (GetBestPlan,
// Sec. 5.2) and curves (Sec. 5.2, Fig. 6) in one kernel, one workgroup per
// job, without writing the candidates to memory.
//
// It exploits the structure of the model: plans without offload do not depend
// on the CPUs or the memory tier, so their per-segment maximum is taken once;
// offload plans depend on the CPUs only through the swap term and on the tier
// only through feasibility.  All values come from the functions of rk_model.h,
// so the results are bit-identical to the materialising path.
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int FUSED_THREADS = 256;

struct FusedLds {          // element counts of the dynamic LDS regions
    uint32_t max_nt, max_ns, rows_per_pass;
};

__host__ __device__ inline size_t fused_lds_bytes(const FusedLds &L) {
    return (size_t)L.max_ns * 8 + (size_t)L.rows_per_pass * L.max_ns * 8 + (size_t)L.max_nt * 4 * 8 + (size_t)L.max_ns * 4;
}

__global__ __launch_bounds__(FUSED_THREADS) void k_fused(JobDev jobs, TableDev tb, GridDev grid, rk_env env,
                                                         uint32_t jb, uint32_t option_mask, FusedLds L,
                                                         uint32_t c_per_pass, uint32_t m_per_pass,
                                                         float *__restrict__ best_thr, uint32_t *__restrict__ best_plan,
                                                         float *__restrict__ curve_thr, uint32_t *__restrict__ curve_plan,
                                                         uint32_t *__restrict__ curve_g) {
    extern __shared__ unsigned long long lds64[];
    unsigned long long *seg_plain = lds64;                                   // [max_ns]
    unsigned long long *seg_best = seg_plain + L.max_ns;                     // [rows_per_pass][max_ns]
    float *t_base0 = reinterpret_cast<float *>(seg_best + (size_t)L.rows_per_pass * L.max_ns);
    float *t_base1 = t_base0 + L.max_nt;
    float *t_topt = t_base1 + L.max_nt;
    float *t_toff = t_topt + L.max_nt;
    float *t_host = t_toff + L.max_nt;
    float *t_invk = t_host + L.max_nt;
    uint32_t *t_info = reinterpret_cast<uint32_t *>(t_invk + L.max_nt);      // ok bits | segment << 4
    uint32_t *t_g = t_info + L.max_nt;
    uint32_t *l_segg = t_g + L.max_nt;                                       // [max_ns] GPUs of the job's segments

    const uint32_t tid = threadIdx.x;
    const uint32_t j = jb + blockIdx.x;
    const uint32_t t0 = tb.triple_off[j], nt = tb.triple_off[j + 1] - t0;
    const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    const uint64_t sbase = (uint64_t)n_rows * (s0 - tb.seg_off[jb]);
    const Job J = load_job(jobs, j);

    // per segment: nothing found yet, its GPU count, and its number in the info word of each of its triples
    for (uint32_t s = tid; s < ns; s += FUSED_THREADS) {
        seg_plain[s] = 0ull;
        l_segg[s] = tb.seg_g[s0 + s];
        const uint32_t first = tb.seg_first[s0 + s];
        const uint32_t last = s + 1 < ns ? tb.seg_first[s0 + s + 1] : nt;
        for (uint32_t t = first; t < last; ++t) t_info[t] = s << 4;
    }
    __syncthreads();

    // phase 1: one thread per triple
    for (uint32_t tl = tid; tl < nt; tl += FUSED_THREADS) {
        const Triple T = triple_terms(J, env, tb.triples[t0 + tl]);
        const uint32_t lo = t_info[tl] >> 4;               // segment of the triple
        unsigned long long k = 0;
#pragma unroll
        for (uint32_t z = 0; z < 4; ++z)
#pragma unroll
            for (uint32_t gc = 0; gc < 2; ++gc) {
                const uint32_t o = z * 4 + gc * 2;
                if (((option_mask >> o) & 1u) && gpu_mem_fits(J, env, T, z, gc, 0)) {
                    const unsigned long long c = make_key(thr_plain(J, T, z, gc), tl * 16 + o);
                    k = c > k ? c : k;
                }
            }
        if (k >> 32) atomicMax(&seg_plain[lo], k);
        uint32_t ok = 0;
#pragma unroll
        for (uint32_t z = 2; z < 4; ++z)
#pragma unroll
            for (uint32_t gc = 0; gc < 2; ++gc) {
                const uint32_t o = z * 4 + gc * 2 + 1;
                if (((option_mask >> o) & 1u) && gpu_mem_fits(J, env, T, z, gc, 1)) ok |= 1u << ((z - 2) * 2 + gc);
            }
        t_info[tl] = ok | (lo << 4);
        t_g[tl] = T.g;
        if (ok) {
            const Offload O = offload_terms(J, env, T);
            t_base0[tl] = O.base[0]; t_base1[tl] = O.base[1];
            t_topt[tl] = O.topt_num; t_toff[tl] = O.Toff; t_invk[tl] = O.inv_kswap;
            t_host[tl] = host_bytes_needed(J, T);
            // T.b is the same for every triple of the job
        }
    }

    // A pass keeps the keys of some rows in LDS: several CPU levels with all their tiers, or, when the rows of one
    // level do not fit, some tiers of one level (m_per_pass < n_mem only together with c_per_pass == 1).  Either
    // way the rows of a pass are neighbours in the output, starting at row c_lo * n_mem + m_lo.
    const float fb = (float)J.gbatch;
    for (uint32_t c_lo = 0; c_lo < grid.n_cpu; c_lo += c_per_pass)
    for (uint32_t m_lo = 0; m_lo < n_mem; m_lo += m_per_pass) {
        const uint32_t c_hi = c_lo + c_per_pass < grid.n_cpu ? c_lo + c_per_pass : grid.n_cpu;
        const uint32_t m_hi = m_lo + m_per_pass < n_mem ? m_lo + m_per_pass : n_mem;
        const uint32_t m_cnt = m_hi - m_lo;
        const uint32_t pass_rows = (c_hi - c_lo) * m_cnt;
        const uint32_t row0 = c_lo * n_mem + m_lo;
        for (uint32_t i = tid; i < pass_rows * ns; i += FUSED_THREADS) seg_best[(size_t)(i / ns) * L.max_ns + i % ns] = 0ull;
        __syncthreads();

        // phase 2: one item per (CPU level, triple with a usable offload plan)
        const uint32_t items = (c_hi - c_lo) * nt;
        for (uint32_t i = tid; i < items; i += FUSED_THREADS) {
            const uint32_t tl = i % nt, ci = c_lo + i / nt;
            const uint32_t info = t_info[tl], ok = info & 15u;
            if (!ok) continue;
            const uint32_t seg = info >> 4, g = t_g[tl];
            Offload O;
            O.base[0] = t_base0[tl]; O.base[1] = t_base1[tl];
            O.topt_num = t_topt[tl]; O.Toff = t_toff[tl]; O.inv_kswap = t_invk[tl];
            Triple Tb; Tb.b = fb;
            const float sw = swap_term(J, O, cpus_of(grid, ci, g));
            const float v0 = thr_offload(Tb, O, 0, sw), v1 = thr_offload(Tb, O, 1, sw);
            unsigned long long k = 0;
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {          // plan-index order: (z2,gc0) (z2,gc1) (z3,gc0) (z3,gc1)
                if ((ok >> q) & 1u) {
                    const uint32_t o = (2 + (q >> 1)) * 4 + (q & 1u) * 2 + 1;
                    const unsigned long long c = make_key((q & 1u) ? v1 : v0, tl * 16 + o);
                    k = c > k ? c : k;
                }
            }
            const float need = t_host[tl];
            for (uint32_t mi = m_lo; mi < m_hi; ++mi)
                if (need <= tier_bytes(grid, mi, g))
                    atomicMax(&seg_best[(size_t)((ci - c_lo) * m_cnt + (mi - m_lo)) * L.max_ns + seg], k);
        }
        __syncthreads();

        // phase 3: merge with the plans without offload, write, then the running maximum along each row.  The
        // wavefronts split the pass's rows; a wavefront walks its rows 64 entries at a time: the running maximum is
        // a segmented scan over packed keys (throughput bits, inverted segment index, GPUs of the segment: the lower
        // segment wins among equal throughputs), a row that continues from the previous 64 entries takes their last
        // key along, and the plan comes from the winning segment's merged key.
        {
            constexpr uint32_t WAVES = FUSED_THREADS / 64;
            const uint32_t lane = tid & 63u, wave = tid >> 6;
            const uint32_t per = (pass_rows + WAVES - 1) / WAVES;
            const uint32_t r_lo = wave * per < pass_rows ? wave * per : pass_rows;
            const uint32_t r_hi = r_lo + per < pass_rows ? r_lo + per : pass_rows;
            const uint32_t n = (r_hi - r_lo) * ns;
            unsigned long long carry = 0;
            for (uint32_t base = 0; base < n; base += 64) {
                const uint32_t i = base + lane;
                const bool in = i < n;
                const uint32_t rl = r_lo + i / ns, s = i % ns;
                const uint64_t out = sbase + (uint64_t)(row0 + rl) * ns + s;
                unsigned long long ck = 0;
                if (in) {
                    unsigned long long k = seg_best[(size_t)rl * L.max_ns + s];
                    const unsigned long long kp = seg_plain[s];
                    k = kp > k ? kp : k;
                    seg_best[(size_t)rl * L.max_ns + s] = k;
                    if (best_thr) {
                        best_thr[out] = key_thr(k);
                        best_plan[out] = key_plan(k);
                    }
                    if (k >> 32) ck = (k & 0xFFFFFFFF00000000ull) | ((0xFFFFu - s) << 16) | l_segg[s];
                }
#pragma unroll
                for (uint32_t d = 1; d < 64; d <<= 1) {
                    const unsigned long long o = __shfl_up(ck, d, 64);
                    if (lane >= d && s >= d) ck = o > ck ? o : ck;      // the lane d below is in the same row
                }
                if (s > lane) ck = carry > ck ? carry : ck;             // the row began before these 64 entries
                carry = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(ck >> 32), 63) << 32) |
                        (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)ck, 63);
                if (in) {
                    uint32_t plan = RK_NO_PLAN;
                    if (ck) plan = key_plan(seg_best[(size_t)rl * L.max_ns + (0xFFFFu - ((uint32_t)(ck >> 16) & 0xFFFFu))]);
                    curve_thr[out] = __uint_as_float((uint32_t)(ck >> 32));
                    curve_plan[out] = plan;
                    curve_g[out] = (uint32_t)ck & 0xFFFFu;
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

int32_t rk_launch_fused(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                        const rk_env *env, uint32_t jb, uint32_t je, float *best_thr, uint32_t *best_plan,
                        float *curve_thr, uint32_t *curve_plan, uint32_t *curve_g) {
    if (je == jb) return RK_OK;
    FusedLds L;
    L.max_nt = table->max_triples_per_job ? table->max_triples_per_job : 1;
    L.max_ns = table->max_segs_per_job ? table->max_segs_per_job : 1;
    // rows per pass so that their segment keys stay within 48 KiB: whole CPU levels (all tiers of each) when a level
    // fits, otherwise one level at a time and as many of its tiers as fit (a row of 2,048 segments takes 16 KiB)
    const size_t one_row = (size_t)L.max_ns * 8, level_bytes = (size_t)grid->n_mem * one_row;
    uint32_t c_per_pass = 1, m_per_pass = grid->n_mem;
    if (level_bytes <= 48 * 1024) {
        c_per_pass = (uint32_t)((48 * 1024) / level_bytes);
        if (c_per_pass > grid->n_cpu) c_per_pass = grid->n_cpu;
    } else {
        m_per_pass = (uint32_t)((48 * 1024) / one_row);
        if (m_per_pass < 1) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 6144 segments per job");
    }
    L.rows_per_pass = c_per_pass * m_per_pass;
    const size_t lds = fused_lds_bytes(L);
    if (lds > 160 * 1024) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "job too large for the fused kernel");
    if (lds > 64 * 1024 && !ctx->fused_lds_raised) {
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_fused),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        ctx->fused_lds_raised = true;
    }
    k_fused<<<je - jb, FUSED_THREADS, lds, ctx->stream>>>(job_dev(jobs), table_dev(table), grid_dev(grid), *env, jb,
                                                         table->option_mask, L, c_per_pass, m_per_pass, best_thr,
                                                         best_plan, curve_thr, curve_plan, curve_g);
    RK_CHECK_LAUNCH(ctx, "k_fused");
    return RK_OK;
}

extern "C" int32_t rk_job_curves(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                                 const rk_alloc_grid *grid, const rk_env *env, uint32_t jb, uint32_t je,
                                 float *best_thr, uint32_t *best_plan, float *curve_thr, uint32_t *curve_plan,
                                 uint32_t *curve_g, uint64_t cap_segs) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs is null");
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if (jobs->n_jobs != table->n_jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs and table disagree on n_jobs");
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if ((rc = rk_check_env(ctx, env))) return rc;
    RK_HIP(ctx, hipSetDevice(ctx->device));
    uint64_t nt, ns;
    if ((rc = rk_range_offsets(ctx, table, jb, je, &nt, &ns))) return rc;
    const uint64_t need = (uint64_t)grid->n_cpu * grid->n_mem * ns;
    if (need == 0) return RK_OK;
    if (!curve_thr || !curve_plan || !curve_g) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null curve buffer");
    if ((best_thr == nullptr) != (best_plan == nullptr)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "best_thr and best_plan must both be given or both be null");
    if (cap_segs < need) return rk_fail(ctx, RK_ERR_CAPACITY, "outputs hold %llu entries, %llu needed",
                                        (unsigned long long)cap_segs, (unsigned long long)need);
    return rk_launch_fused(ctx, jobs, table, grid, env, jb, je, best_thr, best_plan, curve_thr, curve_plan, curve_g);
}
