// Greedy marginal-gain allocation over the resource sensitivity curves
// (paper Sec. 5.2: prefer the jobs that gain the most per unit of resource,
// GPU slopes before CPU slopes; memory is granted last from the chosen plan's
// estimate).  One workgroup per scheduling round; the per-job state lives in
// LDS, every step is a workgroup-wide argmax over cached per-job best steps.
//
// Slopes are float32, ((v1 - v0) / ref_thr) / delta, compared exactly; ties go
// to the smaller target and then to the lower job index.
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int ALLOC_THREADS = 1024;
constexpr int ALLOC_WAVES = ALLOC_THREADS / 64;

struct AllocLds {
    float *slope;        // cached best step of each job (0 = none)
    uint16_t *tgt;       // its target: segment index (GPU pass) or CPU level (CPU pass)
    uint16_t *aux;       // GPU pass: GPUs the step needs; CPU pass: GPUs the job holds
    int16_t *gi;         // granted segment index, -1 = no GPUs
    uint16_t *ci;        // granted CPU level
};

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// workgroup-wide maximum of a key; every thread gets the result
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long *red) {
    v = wave_max_u64(v);
    if ((threadIdx.x & 63u) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long m = red[0];
#pragma unroll
    for (int w = 1; w < ALLOC_WAVES; ++w) m = red[w] > m ? red[w] : m;
    __syncthreads();
    return m;
}

__device__ __forceinline__ unsigned long long cpu_cost(const GridDev &G, uint32_t ci, uint32_t g) {
    return G.cpu_mode ? (unsigned long long)G.cpu_levels[ci] * g : (unsigned long long)G.cpu_levels[ci];
}

__global__ __launch_bounds__(ALLOC_THREADS) void k_allocate(
    const float *__restrict__ ref_thr, TableDev tb, GridDev grid, const uint32_t *__restrict__ round_off,
    const rk_cluster *__restrict__ clusters, uint32_t jb, uint32_t max_jobs,
    const float *__restrict__ best_thr, const uint32_t *__restrict__ best_plan,
    const float *__restrict__ curve_thr, rk_assign *__restrict__ assign, float *__restrict__ totals) {
    extern __shared__ unsigned long long lds_raw[];
    unsigned long long *red = lds_raw;                                        // [ALLOC_WAVES]
    AllocLds S;
    S.slope = reinterpret_cast<float *>(red + ALLOC_WAVES);
    S.tgt = reinterpret_cast<uint16_t *>(S.slope + max_jobs);
    S.aux = S.tgt + max_jobs;
    S.gi = reinterpret_cast<int16_t *>(S.aux + max_jobs);
    S.ci = reinterpret_cast<uint16_t *>(S.gi + max_jobs);

    const uint32_t tid = threadIdx.x, rnd = blockIdx.x;
    const uint32_t J0 = round_off[rnd], nj = round_off[rnd + 1] - J0;
    const rk_cluster cl = clusters[rnd];
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem, m_top = n_mem - 1;
    const uint32_t seg_base = tb.seg_off[jb];
    unsigned long long freeG = cl.G, freeC = cl.C;

    // position of (job, row, segment) in the segment-layout arrays
    auto at = [&](uint32_t j, uint32_t ci, uint32_t mi, uint32_t s) -> uint64_t {
        const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
        return (uint64_t)n_rows * (s0 - seg_base) + (uint64_t)(ci * n_mem + mi) * ns + s;
    };

    // best GPU step of local job jl under the current free capacity
    auto gpu_step = [&](uint32_t jl) {
        const uint32_t j = J0 + jl;
        const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
        const int32_t cur_i = S.gi[jl];
        const uint32_t g_cur = cur_i < 0 ? 0u : tb.seg_g[s0 + cur_i];
        const uint64_t row = (uint64_t)n_rows * (s0 - seg_base) + (uint64_t)m_top * ns;   // ci = 0
        const float cur = cur_i < 0 ? 0.f : curve_thr[row + cur_i];
        const float ref = ref_thr[j];
        const unsigned long long c_cur = cur_i < 0 ? 0ull : cpu_cost(grid, 0, g_cur);
        float top = 0.f;
        uint32_t top_s = 0, top_dg = 0;
        for (uint32_t s = (uint32_t)(cur_i + 1); s < ns; ++s) {
            const uint32_t dg = tb.seg_g[s0 + s] - g_cur;
            if (dg > freeG) break;
            const float v = curve_thr[row + s];
            if (!(v > cur)) continue;
            if (cpu_cost(grid, 0, g_cur + dg) - c_cur > freeC) continue;
            float sl = (v - cur) / ref;
            sl = sl / (float)dg;
            if (sl > top) { top = sl; top_s = s; top_dg = dg; }
        }
        S.slope[jl] = top;
        S.tgt[jl] = (uint16_t)top_s;
        S.aux[jl] = (uint16_t)top_dg;
    };

    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) { S.gi[jl] = -1; S.ci[jl] = 0; }
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) gpu_step(jl);
    __syncthreads();

    // ---- GPU pass
    for (;;) {
        unsigned long long k = 0;
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            const unsigned long long c = ((unsigned long long)__float_as_uint(S.slope[jl]) << 32) | (0xFFFFFFFFu - jl);
            k = c > k ? c : k;
        }
        k = block_max_u64(k, red);
        if (!(k >> 32)) break;                                  // no positive slope left
        const uint32_t jw = 0xFFFFFFFFu - (uint32_t)k;
        const uint32_t dg = S.aux[jw];
        const bool first = S.gi[jw] < 0;
        const unsigned long long dc = grid.cpu_mode ? (unsigned long long)grid.cpu_levels[0] * dg
                                                    : (first ? (unsigned long long)grid.cpu_levels[0] : 0ull);
        freeG -= dg;
        freeC -= dc;
        __syncthreads();                                        // everyone has read the winner's state
        if (tid == (jw % ALLOC_THREADS)) S.gi[jw] = (int16_t)S.tgt[jw];
        // cached steps that no longer fit, and the winner's next step, are recomputed
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            bool redo = jl == jw;
            if (!redo && S.slope[jl] > 0.f) {
                const uint32_t need_g = S.aux[jl];
                const unsigned long long need_c = grid.cpu_mode ? (unsigned long long)grid.cpu_levels[0] * need_g
                                                                : (S.gi[jl] < 0 ? (unsigned long long)grid.cpu_levels[0] : 0ull);
                redo = need_g > freeG || need_c > freeC;
            }
            if (redo) gpu_step(jl);
        }
        __syncthreads();
    }

    // ---- CPU pass
    auto cpu_step = [&](uint32_t jl) {
        const int32_t cur_i = S.gi[jl];
        float top = 0.f;
        uint32_t top_c = 0;
        if (cur_i >= 0) {
            const uint32_t j = J0 + jl, g = S.aux[jl], c0 = S.ci[jl];
            const float cur = best_thr[at(j, c0, m_top, (uint32_t)cur_i)];
            const float ref = ref_thr[j];
            const unsigned long long have = cpu_cost(grid, c0, g);
            for (uint32_t c = c0 + 1; c < grid.n_cpu; ++c) {
                const unsigned long long dc = cpu_cost(grid, c, g) - have;
                if (dc > freeC) break;
                const float v = best_thr[at(j, c, m_top, (uint32_t)cur_i)];
                if (!(v > cur)) continue;
                float sl = (v - cur) / ref;
                sl = sl / (float)dc;
                if (sl > top) { top = sl; top_c = c; }
            }
        }
        S.slope[jl] = top;
        S.tgt[jl] = (uint16_t)top_c;
    };
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
        const int32_t cur_i = S.gi[jl];
        S.aux[jl] = cur_i < 0 ? (uint16_t)0 : (uint16_t)tb.seg_g[tb.seg_off[J0 + jl] + cur_i];
    }
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) cpu_step(jl);
    __syncthreads();
    for (;;) {
        unsigned long long k = 0;
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            const unsigned long long c = ((unsigned long long)__float_as_uint(S.slope[jl]) << 32) | (0xFFFFFFFFu - jl);
            k = c > k ? c : k;
        }
        k = block_max_u64(k, red);
        if (!(k >> 32)) break;
        const uint32_t jw = 0xFFFFFFFFu - (uint32_t)k;
        freeC -= cpu_cost(grid, S.tgt[jw], S.aux[jw]) - cpu_cost(grid, S.ci[jw], S.aux[jw]);
        __syncthreads();
        if (tid == (jw % ALLOC_THREADS)) S.ci[jw] = S.tgt[jw];
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            bool redo = jl == jw;
            if (!redo && S.slope[jl] > 0.f)
                redo = cpu_cost(grid, S.tgt[jl], S.aux[jl]) - cpu_cost(grid, S.ci[jl], S.aux[jl]) > freeC;
            if (redo) cpu_step(jl);
        }
        __syncthreads();
    }

    // ---- memory, in job order, by the first wavefront: lanes load a batch of
    // 64 jobs, then take their decisions one after the other
    if (tid < 64) {
        float freeM = cl.host_mem_gb;
        double sum = 0.0;
        for (uint32_t base = 0; base < nj; base += 64) {
            const uint32_t jl = base + tid;
            const bool have = jl < nj && S.gi[jl] >= 0;
            uint32_t g = 0, c_lvl = 0, s_i = 0, j = 0;
            unsigned long long choice = 0;      // 4 bits per prefix length: best tier among tiers 0..k
            uint32_t valid = 0;                 // bit k: that best throughput is positive
            float thr_m[RK_MAX_MEM_LEVELS];
            if (have) {
                j = J0 + jl; g = S.aux[jl]; c_lvl = S.ci[jl]; s_i = (uint32_t)S.gi[jl];
                float bv = 0.f;
                uint32_t bm = 0;
#pragma unroll
                for (uint32_t m = 0; m < RK_MAX_MEM_LEVELS; ++m) {
                    thr_m[m] = 0.f;
                    if (m < n_mem) {
                        const float v = best_thr[at(j, c_lvl, m, s_i)];
                        thr_m[m] = v;
                        if (v > bv) { bv = v; bm = m; }
                        choice |= (unsigned long long)bm << (4 * m);
                        if (bv > 0.f) valid |= 1u << m;
                    }
                }
            }
            rk_assign out = {0u, 0u, 0.f, RK_NO_PLAN, 0.f};
            for (uint32_t turn = 0; turn < 64 && base + turn < nj; ++turn) {
                float spent = 0.f;
                if (tid == turn && have) {
                    int32_t k = -1;                         // last tier that still fits (tiers ascend)
                    for (uint32_t m = 0; m < n_mem; ++m) {
                        float cost = grid.mem_levels_gb[m];
                        if (grid.mem_mode) cost = cost * (float)g;
                        if (cost <= freeM) k = (int32_t)m;
                    }
                    if (k >= 0 && ((valid >> k) & 1u)) {
                        const uint32_t bm = (uint32_t)(choice >> (4 * k)) & 15u;
                        float cost = grid.mem_levels_gb[bm];
                        if (grid.mem_mode) cost = cost * (float)g;
                        spent = cost;
                        float v = 0.f;
#pragma unroll
                        for (uint32_t m = 0; m < RK_MAX_MEM_LEVELS; ++m) if (m == bm) v = thr_m[m];
                        out.g = g;
                        out.c = (uint32_t)cpu_cost(grid, c_lvl, g);
                        out.mem_gb = cost;
                        out.plan = best_plan[at(j, c_lvl, bm, s_i)];
                        out.thr = v;
                        sum += (double)v / (double)ref_thr[j];
                    }
                }
                spent = __shfl(spent, (int)turn, 64);
                freeM = freeM - spent;
            }
            if (jl < nj) assign[(J0 - jb) + jl] = out;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (tid == 0) totals[rnd] = (float)sum;
    }
}

}  // namespace

int32_t rk_launch_allocate(rk_ctx *ctx, const float *ref_thr, const TableDev &tb, const rk_alloc_grid *grid,
                               uint32_t n_rounds, const uint32_t *d_round_off, const rk_cluster *d_clusters,
                               uint32_t jb, uint32_t max_jobs, const float *best_thr, const uint32_t *best_plan,
                               const float *curve_thr, rk_assign *assign, float *totals) {
    if (n_rounds == 0) return RK_OK;
    if (max_jobs > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "a round has %u jobs, the allocation kernel takes up to %u", max_jobs,
                       RK_MAX_JOBS_PER_ROUND);
    const uint32_t mj = max_jobs ? ((max_jobs + 1u) & ~1u) : 2u;
    const size_t lds = ALLOC_WAVES * 8 + (size_t)mj * (4 + 2 + 2 + 2 + 2);
    static bool raised[64] = {};
    if (lds > 64 * 1024 && !raised[ctx->device & 63]) {
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_allocate),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        raised[ctx->device & 63] = true;
    }
    k_allocate<<<n_rounds, ALLOC_THREADS, lds, ctx->stream>>>(ref_thr, tb, grid_dev(grid), d_round_off, d_clusters, jb,
                                                             mj, best_thr, best_plan, curve_thr, assign, totals);
    RK_CHECK_LAUNCH(ctx, "k_allocate");
    return RK_OK;
}

extern "C" int32_t rk_allocate(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                               const rk_alloc_grid *grid, const rk_cluster *cluster, uint32_t jb, uint32_t je,
                               const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                               rk_assign *assign, float *total) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (!cluster || !ref_thr || !best_thr || !best_plan || !curve_thr || !assign || !total)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (!(cluster->host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    // round meta: [jb, je] and the cluster, staged through the scratch
    struct Meta { uint32_t off[2]; uint32_t pad[2]; rk_cluster cl; } meta = {{jb, je}, {0, 0}, *cluster};
    void *d_meta;
    if ((rc = rk_scratch(ctx, SL_ROUND_META, sizeof(Meta), &d_meta))) return rc;
    RK_HIP(ctx, hipMemcpyAsync(d_meta, &meta, sizeof(Meta), hipMemcpyHostToDevice, ctx->stream));
    // the copy reads a stack object: wait for it before returning
    RK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const uint32_t *d_off = reinterpret_cast<const uint32_t *>(d_meta);
    const rk_cluster *d_cl = reinterpret_cast<const rk_cluster *>(reinterpret_cast<const char *>(d_meta) + 16);
    return rk_launch_allocate(ctx, ref_thr, table_dev(table), grid, 1, d_off, d_cl, jb, je - jb, best_thr, best_plan,
                           curve_thr, assign, total);
}
