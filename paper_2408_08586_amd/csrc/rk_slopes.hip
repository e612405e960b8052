// The slope table of the resource sensitivity curves (paper Sec. 5.2: a job's slope, per resource type, is the
// throughput change per unit of the resource; Fig. 6): for every row (CPU level, memory tier) and GPU count of a job
// the step the allocation rules take from there - the larger count with the highest float32 slope
// ((v1 - v0) / ref_thr) / delta, the smaller count among equal slopes - and likewise the next CPU level; per row
// also the first step from nothing.  The same arithmetic, in the same order, as the greedy and the Schedule loops use
// for their steps; the table itself does not depend on the cluster.
//
// A workgroup per job, a thread per (row, count) entry; an entry looks at the counts above it (the levels above it),
// which a job has a few dozen of at most.
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int SLOPE_THREADS = 256;

struct SlopeArgs {
    const float *ref_thr;
    TableDev tb;
    GridDev grid;
    uint32_t jb;
    const float *best_thr, *curve_thr;
    float *gpu_slope, *from0_slope, *cpu_slope;
    int32_t *gpu_next, *from0_next;
    uint32_t *cpu_next;
};

__global__ __launch_bounds__(SLOPE_THREADS) void k_curve_slopes(SlopeArgs A) {
    const uint32_t j = A.jb + blockIdx.x;
    const uint32_t s0 = A.tb.seg_off[j], ns = A.tb.seg_off[j + 1] - s0;
    const uint32_t n_mem = A.grid.n_mem, n_cpu = A.grid.n_cpu, rows = n_cpu * n_mem;
    const uint64_t base = (uint64_t)rows * (s0 - A.tb.seg_off[A.jb]);
    const float ref = A.ref_thr[j];
    // the next GPU step from count s of a row (s = -1: from nothing)
    auto gpu_step = [&](uint64_t row, int32_t s, float &top, int32_t &nxt) {
        const float cur = s < 0 ? 0.f : A.curve_thr[row + (uint32_t)s];
        const uint32_t g = s < 0 ? 0u : A.tb.seg_g[s0 + (uint32_t)s];
        top = 0.f; nxt = -1;
        for (uint32_t t = (uint32_t)(s + 1); t < ns; ++t) {
            const float v = A.curve_thr[row + t];
            if (!(v > cur)) continue;
            float sl = (v - cur) / ref;
            sl = sl / (float)(A.tb.seg_g[s0 + t] - g);
            if (sl > top) { top = sl; nxt = (int32_t)t; }
        }
    };
    for (uint32_t e = threadIdx.x; e < rows * ns; e += SLOPE_THREADS) {
        const uint32_t r = e / ns, s = e - r * ns, ci = r / n_mem, mi = r - ci * n_mem;
        const uint64_t row = base + (uint64_t)r * ns;
        float top;
        int32_t nxt;
        gpu_step(row, (int32_t)s, top, nxt);
        A.gpu_slope[row + s] = top; A.gpu_next[row + s] = nxt;
        const float cur = A.best_thr[row + s];
        const uint32_t g = A.tb.seg_g[s0 + s];
        float ctop = 0.f;
        uint32_t cnxt = n_cpu;
        for (uint32_t c = ci + 1; c < n_cpu; ++c) {
            const float v = A.best_thr[base + ((uint64_t)c * n_mem + mi) * ns + s];
            if (!(v > cur)) continue;
            float sl = (v - cur) / ref;
            sl = sl / (float)(cpus_of(A.grid, c, g) - cpus_of(A.grid, ci, g));
            if (sl > ctop) { ctop = sl; cnxt = c; }
        }
        A.cpu_slope[row + s] = ctop; A.cpu_next[row + s] = cnxt;
    }
    for (uint32_t r = threadIdx.x; r < rows; r += SLOPE_THREADS) {
        float top;
        int32_t nxt;
        gpu_step(base + (uint64_t)r * ns, -1, top, nxt);
        A.from0_slope[(uint64_t)rows * blockIdx.x + r] = top; A.from0_next[(uint64_t)rows * blockIdx.x + r] = nxt;
    }
}

}  // namespace

extern "C" int32_t rk_curve_slopes(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                   const rk_alloc_grid *grid, uint32_t job_begin, uint32_t job_end,
                                   const float *best_thr, const float *curve_thr, float *gpu_slope, int32_t *gpu_next,
                                   float *from0_slope, int32_t *from0_next, float *cpu_slope, uint32_t *cpu_next,
                                   uint64_t cap_segs) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, job_begin, job_end))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (job_end == job_begin) return RK_OK;
    uint64_t n_triples, n_segs;
    if ((rc = rk_range_offsets(ctx, table, job_begin, job_end, &n_triples, &n_segs))) return rc;
    const uint64_t need = (uint64_t)grid->n_cpu * grid->n_mem * n_segs;
    if (cap_segs < need)
        return rk_fail(ctx, RK_ERR_CAPACITY, "slope arrays hold %llu entries, %llu needed", (unsigned long long)cap_segs, (unsigned long long)need);
    if (!ref_thr || !from0_slope || !from0_next ||
        (need > 0 && (!best_thr || !curve_thr || !gpu_slope || !gpu_next || !cpu_slope || !cpu_next)))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    SlopeArgs A;
    A.ref_thr = ref_thr; A.tb = table_dev(table); A.grid = grid_dev(grid); A.jb = job_begin;
    A.best_thr = best_thr; A.curve_thr = curve_thr;
    A.gpu_slope = gpu_slope; A.gpu_next = gpu_next; A.from0_slope = from0_slope; A.from0_next = from0_next;
    A.cpu_slope = cpu_slope; A.cpu_next = cpu_next;
    k_curve_slopes<<<job_end - job_begin, SLOPE_THREADS, 0, ctx->stream>>>(A);
    RK_CHECK_LAUNCH(ctx, "k_curve_slopes");
    return RK_OK;
}
