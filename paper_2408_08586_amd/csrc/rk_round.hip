// Whole scheduling rounds on the device: enumerate -> fused evaluation /
// best plan / curves -> [minimum demands, privileged phase] -> greedy
// allocation (paper Sec. 5.2, Algorithm 1 over cluster totals).
#include <cstring>

#include "rk_internal.h"

namespace {

// what a round leaves in the context's buffers for a step that follows it
struct RoundKeep {
    rk_plan_table tb;
    float *best_thr, *curve_thr;
    uint32_t *best_plan;
    int32_t *min_seg;        // null without service levels
    bool curves_only;        // set by the caller: stop after the curves, no allocation
};

// sla == NULL: every job is best-effort.  round_jobs != NULL: the rounds are made of slots, slot i
// schedules job round_jobs[i]; every job is enumerated and evaluated once however many slots use it.
int32_t schedule_rounds(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                        const rk_alloc_grid *grid, const rk_env *env, uint32_t n_rounds,
                        const uint32_t *round_off, const uint32_t *round_jobs, const rk_cluster *clusters,
                        const rk_sla *sla, rk_assign *assign, float *totals, RoundKeep *keep = nullptr) {
    int32_t rc;
    if (!jobs || !bounds || !round_off || !clusters || !totals || (!assign && jobs->n_jobs > 0))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (!jobs->ref_thr && jobs->n_jobs > 0) return rk_fail(ctx, RK_ERR_INVALID_ARG, "ref_thr is null");
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if ((rc = rk_check_env(ctx, env))) return rc;
    if (n_rounds == 0) return RK_OK;
    const uint32_t J = jobs->n_jobs;
    uint32_t max_jobs = 0;
    const uint32_t n_slots = round_off[n_rounds];
    if (round_off[0] != 0 || (!round_jobs && n_slots != J))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "round_off must run from 0 to n_jobs");
    if (round_jobs) {
        if (sla) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "rounds that share jobs take no service levels");
        for (uint32_t i = 0; i < n_slots; ++i)
            if (round_jobs[i] >= J) return rk_fail(ctx, RK_ERR_INVALID_ARG, "round_jobs[%u] = %u is not a job", i, round_jobs[i]);
    }
    for (uint32_t r = 0; r < n_rounds; ++r) {
        if (round_off[r + 1] < round_off[r]) return rk_fail(ctx, RK_ERR_INVALID_ARG, "round_off not ascending");
        const uint32_t n = round_off[r + 1] - round_off[r];
        max_jobs = n > max_jobs ? n : max_jobs;
        if (!(clusters[r].host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    }
    if (max_jobs > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "a round has %u jobs, the allocation kernel takes up to %u", max_jobs,
                       RK_MAX_JOBS_PER_ROUND);
    RK_HIP(ctx, hipSetDevice(ctx->device));

    // round ranges and clusters go up first; the wait inside the enumeration covers the copy.
    // A single round travels in the kernel arguments instead.
    const size_t off_bytes = (((size_t)n_rounds + 1) * 4 + 15) & ~(size_t)15;
    char *d_meta = nullptr;
    uint32_t *d_jmap = nullptr;
    if (round_jobs && n_slots > 0) {
        if ((rc = rk_scratch(ctx, SL_JMAP, (size_t)n_slots * 4, (void **)&d_jmap))) return rc;
        RK_HIP(ctx, hipMemcpyAsync(d_jmap, round_jobs, (size_t)n_slots * 4, hipMemcpyHostToDevice, ctx->stream));
    }
    if (n_rounds > 1) {
        if ((rc = rk_scratch(ctx, SL_ROUND_META, off_bytes + (size_t)n_rounds * sizeof(rk_cluster), (void **)&d_meta))) return rc;
        RK_HIP(ctx, hipMemcpyAsync(d_meta, round_off, ((size_t)n_rounds + 1) * 4, hipMemcpyHostToDevice, ctx->stream));
        RK_HIP(ctx, hipMemcpyAsync(d_meta + off_bytes, clusters, (size_t)n_rounds * sizeof(rk_cluster), hipMemcpyHostToDevice, ctx->stream));
    }

    // internal plan table in scratch memory; grown on demand
    rk_plan_table tb;
    memset(&tb, 0, sizeof(tb));
    uint64_t cap_t = ctx->scratch_bytes[SL_TB_TRIPLES] / 4, cap_s = ctx->scratch_bytes[SL_TB_SEGG] / 4;
    if (cap_t < (uint64_t)J * 256) cap_t = (uint64_t)J * 256;
    if (cap_s < (uint64_t)J * 32) cap_s = (uint64_t)J * 32;
    for (int attempt = 0; attempt < 2; ++attempt) {
        if ((rc = rk_scratch(ctx, SL_TB_TOFF, ((size_t)J + 1) * 4, (void **)&tb.triple_off))) return rc;
        if ((rc = rk_scratch(ctx, SL_TB_SOFF, ((size_t)J + 1) * 4, (void **)&tb.seg_off))) return rc;
        if ((rc = rk_scratch(ctx, SL_TB_TRIPLES, cap_t * 4, (void **)&tb.triples))) return rc;
        if ((rc = rk_scratch(ctx, SL_TB_SEGG, cap_s * 4, (void **)&tb.seg_g))) return rc;
        if ((rc = rk_scratch(ctx, SL_TB_SEGF, cap_s * 4, (void **)&tb.seg_first))) return rc;
        tb.cap_triples = cap_t;
        tb.cap_segs = cap_s;
        rc = rk_enumerate_plans(ctx, jobs, bounds, &tb);
        if (rc != RK_ERR_CAPACITY) break;
        cap_t = tb.n_triples;
        cap_s = tb.n_segs;
    }
    if (rc) return rc;
    if (tb.max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");

    const uint64_t n_rows = (uint64_t)grid->n_cpu * grid->n_mem;
    const size_t n_out = (size_t)(n_rows * tb.n_segs);
    float *best_thr, *curve_thr;
    uint32_t *best_plan, *curve_plan, *curve_g;
    if ((rc = rk_scratch(ctx, SL_BEST_THR, n_out * 4, (void **)&best_thr))) return rc;
    if ((rc = rk_scratch(ctx, SL_BEST_PLAN, n_out * 4, (void **)&best_plan))) return rc;
    if ((rc = rk_scratch(ctx, SL_CURVE_THR, n_out * 4, (void **)&curve_thr))) return rc;
    if ((rc = rk_scratch(ctx, SL_CURVE_PLAN, n_out * 4, (void **)&curve_plan))) return rc;
    if ((rc = rk_scratch(ctx, SL_CURVE_G, n_out * 4, (void **)&curve_g))) return rc;

    if ((rc = rk_launch_fused(ctx, jobs, &tb, grid, env, 0, J, best_thr, best_plan, curve_thr, curve_plan, curve_g))) return rc;
    if (keep) {
        keep->tb = tb; keep->best_thr = best_thr; keep->best_plan = best_plan; keep->curve_thr = curve_thr; keep->min_seg = nullptr;
        if (keep->curves_only) return RK_OK;
    }
    SlaDev S = {};
    if (sla && J > 0) {
        int32_t *min_seg;
        uint32_t *min_c, *min_m;
        if ((rc = rk_scratch(ctx, SL_MIN_SEG, (size_t)J * 4, (void **)&min_seg))) return rc;
        if ((rc = rk_scratch(ctx, SL_MIN_C, (size_t)J * 4, (void **)&min_c))) return rc;
        if ((rc = rk_scratch(ctx, SL_MIN_M, (size_t)J * 4, (void **)&min_m))) return rc;
        if ((rc = rk_launch_min_res(ctx, table_dev(&tb), grid, 0, J, best_thr, sla, min_seg, min_c, min_m))) return rc;
        S = SlaDev{sla->guaranteed, sla->tenant, min_seg, min_c, sla->n_tenants, sla->quota_g, sla->quota_c};
        if (keep) keep->min_seg = min_seg;
    }
    return rk_launch_allocate(ctx, jobs->ref_thr, table_dev(&tb), grid, n_rounds,
                              reinterpret_cast<const uint32_t *>(d_meta),
                              d_meta ? reinterpret_cast<const rk_cluster *>(d_meta + off_bytes) : nullptr,
                              n_rounds == 1 ? &clusters[0] : nullptr, 0, round_jobs ? n_slots : J, max_jobs,
                              tb.max_segs_per_job, best_thr, best_plan, curve_thr, (sla && J > 0) ? &S : nullptr, nullptr,
                              d_jmap, assign, totals);
}

}  // namespace

extern "C" {

int32_t rk_schedule_rounds(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                           const rk_alloc_grid *grid, const rk_env *env, uint32_t n_rounds,
                           const uint32_t *round_off, const rk_cluster *clusters, rk_assign *assign,
                           float *totals) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    return schedule_rounds(ctx, jobs, bounds, grid, env, n_rounds, round_off, nullptr, clusters, nullptr, assign, totals);
}

int32_t rk_schedule_rounds_shared(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                                  const rk_alloc_grid *grid, const rk_env *env, uint32_t n_rounds,
                                  const uint32_t *round_off, const uint32_t *round_jobs, const rk_cluster *clusters,
                                  rk_assign *assign, float *totals) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!round_jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "round_jobs is null");
    return schedule_rounds(ctx, jobs, bounds, grid, env, n_rounds, round_off, round_jobs, clusters, nullptr, assign, totals);
}

int32_t rk_schedule_round(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                          const rk_alloc_grid *grid, const rk_env *env, const rk_cluster *cluster,
                          rk_assign *assign, float *total) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!jobs || !cluster) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    const uint32_t off[2] = {0u, jobs->n_jobs};
    return schedule_rounds(ctx, jobs, bounds, grid, env, 1, off, nullptr, cluster, nullptr, assign, total);
}

int32_t rk_schedule_round_sla(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                              const rk_alloc_grid *grid, const rk_env *env, const rk_cluster *cluster,
                              const rk_sla *sla, rk_assign *assign, float *total) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!jobs || !cluster) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    int32_t rc;
    if (jobs->n_jobs > 0 && (rc = rk_check_sla(ctx, sla, true))) return rc;
    const uint32_t off[2] = {0u, jobs->n_jobs};
    return schedule_rounds(ctx, jobs, bounds, grid, env, 1, off, nullptr, cluster, jobs->n_jobs > 0 ? sla : nullptr, assign,
                           total);
}

int32_t rk_schedule_round_placed(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                                 const rk_alloc_grid *grid, const rk_env *env, const rk_nodes *nodes, const rk_sla *sla,
                                 rk_assign *assign, rk_assign *placed, uint32_t *place_off, rk_place_entry *entries,
                                 uint64_t cap_entries, uint32_t *status, float *total, rk_place_result *result) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!jobs || !nodes || !total) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (jobs->n_jobs > 0 && !placed) return rk_fail(ctx, RK_ERR_INVALID_ARG, "placed is null");
    int32_t rc;
    if (sla && jobs->n_jobs > 0 && (rc = rk_check_sla(ctx, sla, true))) return rc;
    // the amounts are decided against what the nodes hold together, then the nodes are walked
    const uint64_t G = (uint64_t)nodes->n_nodes * nodes->gpus_per_node, Cc = (uint64_t)nodes->n_nodes * nodes->cpus_per_node;
    if (G > 0xFFFFFFFFull || Cc > 0xFFFFFFFFull) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "cluster too large");
    const rk_cluster cluster = {(uint32_t)G, (uint32_t)Cc, (float)nodes->n_nodes * nodes->mem_per_node_gb};
    const uint32_t off[2] = {0u, jobs->n_jobs};
    RoundKeep keep;
    keep.curves_only = false;
    if ((rc = schedule_rounds(ctx, jobs, bounds, grid, env, 1, off, nullptr, &cluster, jobs->n_jobs > 0 ? sla : nullptr, assign,
                              total, &keep))) return rc;
    return rk_launch_place_plans(ctx, jobs, &keep.tb, grid, env, nodes, keep.best_thr, assign, keep.min_seg, nullptr, nullptr,
                                 placed, place_off, entries, cap_entries, status, total, result);
}

int32_t rk_schedule_round_nodes(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                                const rk_alloc_grid *grid, const rk_env *env, const rk_nodes *nodes,
                                const rk_job_state *jobs_state, const uint32_t *prev_off,
                                const rk_place_entry *prev_entries, uint64_t n_prev_entries, rk_assign *assign,
                                rk_assign *placed, uint32_t *place_off, rk_place_entry *entries, uint64_t cap_entries,
                                float *total, uint32_t *stats) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!jobs || !nodes || !total || !jobs_state || !place_off) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    const uint32_t J = jobs->n_jobs;
    if (J > 0 && (!assign || !placed || !entries || !jobs_state->cur_seg || !jobs_state->cur_c))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (placed == assign && J > 0) return rk_fail(ctx, RK_ERR_INVALID_ARG, "placed must not be assign");
    if ((prev_off == nullptr) != (prev_entries == nullptr))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "the earlier placement needs both its offsets and its entries");
    if (nodes->n_nodes == 0 || nodes->n_nodes > RK_MAX_NODES || nodes->gpus_per_node == 0 ||
        nodes->gpus_per_node > 65535u || nodes->cpus_per_node > 65535u || !(nodes->mem_per_node_gb >= 0.f))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "nodes: 1..%u nodes of 1..65535 GPUs, at most 65535 CPUs, memory >= 0", RK_MAX_NODES);
    int32_t rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (grid->cpu_mode != 1u)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "the search over nodes needs CPU levels per GPU (cpu_mode 1)");
    const uint64_t gpus = (uint64_t)nodes->n_nodes * nodes->gpus_per_node;
    if (gpus > (1u << 20)) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 2^20 GPUs on the nodes");
    if (J > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u jobs, the allocation kernels take up to %u", J, RK_MAX_JOBS_PER_ROUND);
    if (cap_entries < gpus && J > 0)
        return rk_fail(ctx, RK_ERR_CAPACITY, "entries: %llu records, %llu may be needed", (unsigned long long)cap_entries, (unsigned long long)gpus);
    // plan table and curves of all jobs in the context's buffers, then the loop over the nodes, then the plans for the splits
    const rk_cluster whole = {(uint32_t)gpus, 0u, 0.f};
    const uint32_t off[2] = {0u, J};
    RoundKeep keep;
    keep.curves_only = true;
    if ((rc = schedule_rounds(ctx, jobs, bounds, grid, env, 1, off, nullptr, &whole, nullptr, assign, total, &keep))) return rc;
    if ((rc = rk_launch_reschedule_nodes(ctx, jobs->ref_thr, &keep.tb, grid, nodes, keep.best_thr, keep.best_plan, keep.curve_thr,
                                         jobs_state, prev_off, prev_entries, n_prev_entries, assign, place_off, entries, total,
                                         stats))) return rc;
    return rk_launch_best_plan_placed(ctx, jobs, &keep.tb, grid, env, assign, place_off, entries, placed, total);
}

}  // extern "C"
