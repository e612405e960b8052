// Context, error reporting, scratch memory and argument validation.
#include <cmath>
#include <cstdlib>
#include <cstring>

#include "rk_internal.h"

int32_t rk_fail(rk_ctx *ctx, int32_t code, const char *fmt, ...) {
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

int32_t rk_scratch(rk_ctx *ctx, int slot, size_t bytes, void **out) {
    if (bytes == 0) bytes = 256;
    if (ctx->scratch_bytes[slot] < bytes) {
        if (ctx->scratch[slot]) {
            // buffers may still be read by enqueued kernels
            RK_HIP(ctx, hipStreamSynchronize(ctx->stream));
            RK_HIP(ctx, hipFree(ctx->scratch[slot]));
            ctx->scratch[slot] = nullptr;
            ctx->scratch_bytes[slot] = 0;
        }
        size_t want = bytes + bytes / 4;
        want = (want + 255) & ~(size_t)255;
        RK_HIP(ctx, hipMalloc(&ctx->scratch[slot], want));
        ctx->scratch_bytes[slot] = want;
    }
    *out = ctx->scratch[slot];
    return RK_OK;
}

int32_t rk_check_grid(rk_ctx *ctx, const rk_alloc_grid *g) {
    if (!g) return rk_fail(ctx, RK_ERR_INVALID_ARG, "grid is null");
    if (g->n_cpu < 1 || g->n_cpu > RK_MAX_CPU_LEVELS) return rk_fail(ctx, RK_ERR_INVALID_ARG, "n_cpu out of range");
    if (g->n_mem < 1 || g->n_mem > RK_MAX_MEM_LEVELS) return rk_fail(ctx, RK_ERR_INVALID_ARG, "n_mem out of range");
    if (g->cpu_mode > 1 || g->mem_mode > 1) return rk_fail(ctx, RK_ERR_INVALID_ARG, "bad cpu_mode / mem_mode");
    for (uint32_t i = 0; i < g->n_cpu; ++i) {
        if (g->cpu_levels[i] < 1) return rk_fail(ctx, RK_ERR_INVALID_ARG, "cpu level below 1");
        if (g->cpu_levels[i] > (1u << 20)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "cpu level above 2^20");
        if (i && g->cpu_levels[i] <= g->cpu_levels[i - 1]) return rk_fail(ctx, RK_ERR_INVALID_ARG, "cpu levels not ascending");
    }
    for (uint32_t i = 0; i < g->n_mem; ++i) {
        if (!(g->mem_levels_gb[i] >= 0.f) || !std::isfinite(g->mem_levels_gb[i]))
            return rk_fail(ctx, RK_ERR_INVALID_ARG, "memory tier negative or not finite");
        if (i && !(g->mem_levels_gb[i] > g->mem_levels_gb[i - 1])) return rk_fail(ctx, RK_ERR_INVALID_ARG, "memory tiers not ascending");
    }
    return RK_OK;
}

int32_t rk_check_env(rk_ctx *ctx, const rk_env *e) {
    if (!e) return rk_fail(ctx, RK_ERR_INVALID_ARG, "env is null");
    if (!(e->B_intra > 0.f) || !(e->B_inter > 0.f) || !(e->B_pcie > 0.f) || !(e->gpu_mem_cap >= 0.f))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "env bandwidths must be positive");
    if (e->gpus_per_node < 1) return rk_fail(ctx, RK_ERR_INVALID_ARG, "gpus_per_node below 1");
    return RK_OK;
}

int32_t rk_check_table(rk_ctx *ctx, const rk_plan_table *t, uint32_t jb, uint32_t je) {
    if (!t) return rk_fail(ctx, RK_ERR_INVALID_ARG, "table is null");
    if (!t->triple_off || !t->triples || !t->seg_off || !t->seg_g || !t->seg_first)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "table buffer is null");
    if (jb > je || je > t->n_jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "job range [%u,%u) outside the table's %u jobs", jb, je, t->n_jobs);
    return RK_OK;
}

int32_t rk_range_offsets(rk_ctx *ctx, const rk_plan_table *t, uint32_t jb, uint32_t je,
                         uint64_t *n_triples, uint64_t *n_segs) {
    if (jb == 0 && je == t->n_jobs) {
        *n_triples = t->n_triples; *n_segs = t->n_segs;
        return RK_OK;
    }
    if (t->h_triple_off && t->h_seg_off) {
        *n_triples = t->h_triple_off[je] - t->h_triple_off[jb];
        *n_segs = t->h_seg_off[je] - t->h_seg_off[jb];
        return RK_OK;
    }
    uint32_t *h = ctx->h_pinned;
    RK_HIP(ctx, hipMemcpyAsync(h + 0, t->triple_off + jb, 4, hipMemcpyDeviceToHost, ctx->stream));
    RK_HIP(ctx, hipMemcpyAsync(h + 1, t->triple_off + je, 4, hipMemcpyDeviceToHost, ctx->stream));
    RK_HIP(ctx, hipMemcpyAsync(h + 2, t->seg_off + jb, 4, hipMemcpyDeviceToHost, ctx->stream));
    RK_HIP(ctx, hipMemcpyAsync(h + 3, t->seg_off + je, 4, hipMemcpyDeviceToHost, ctx->stream));
    RK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    *n_triples = h[1] - h[0];
    *n_segs = h[3] - h[2];
    return RK_OK;
}

extern "C" {

int32_t rk_create(rk_ctx **out, int32_t device_id, void *hip_stream) {
    if (!out) return RK_ERR_INVALID_ARG;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device_id < 0 || device_id >= n) return RK_ERR_DEVICE;
    rk_ctx *ctx = (rk_ctx *)calloc(1, sizeof(rk_ctx));
    if (!ctx) return RK_ERR_DEVICE;
    ctx->device = device_id;
    ctx->stream = (hipStream_t)hip_stream;
    if (hipSetDevice(device_id) != hipSuccess ||
        hipHostMalloc((void **)&ctx->h_pinned, 64 * sizeof(uint32_t), hipHostMallocDefault) != hipSuccess) {
        free(ctx);
        return RK_ERR_DEVICE;
    }
    if (rk_allocate_setup(ctx) != RK_OK) {
        (void)hipHostFree(ctx->h_pinned);
        free(ctx);
        return RK_ERR_DEVICE;
    }
    *out = ctx;
    return RK_OK;
}

int32_t rk_destroy(rk_ctx *ctx) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (int i = 0; i < RK_SCRATCH_SLOTS; ++i)
        if (ctx->scratch[i]) (void)hipFree(ctx->scratch[i]);
    if (ctx->h_pinned) (void)hipHostFree(ctx->h_pinned);
    if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
    if (ctx->counts_ev) (void)hipEventDestroy(ctx->counts_ev);
    if (ctx->sim_stream) {
        (void)hipStreamSynchronize(ctx->sim_stream);
        (void)hipStreamDestroy(ctx->sim_stream);
        (void)hipEventDestroy(ctx->sim_ev[0]);
        (void)hipEventDestroy(ctx->sim_ev[1]);
    }
    free(ctx);
    return RK_OK;
}

int32_t rk_sync(rk_ctx *ctx) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    RK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return RK_OK;
}

const char *rk_last_error(const rk_ctx *ctx) { return ctx ? ctx->err : "null context"; }

}  // extern "C"
