// Internal declarations shared by the translation units of the library:
// the context, error helpers and host-side launch wrappers.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "rubick.h"

enum { RK_SCRATCH_SLOTS = 56 };

struct rk_ctx {
    int device;
    hipStream_t stream;
    char err[512];
    void *scratch[RK_SCRATCH_SLOTS];        // grow-only device buffers owned by the context
    size_t scratch_bytes[RK_SCRATCH_SLOTS];
    uint32_t *h_pinned;                     // 64 pinned host words for counts coming back
    uint32_t *h_stage;                      // pinned staging for the plan-table offsets, grown on demand
    size_t h_stage_words;
    uint32_t park_stride;                   // enumeration: words per job between its two passes
    hipEvent_t counts_ev;                   // enumeration: the counts have reached the host (made on demand)
    hipStream_t sim_stream;                 // simulation: its own stream (a tick is captured as a graph), made on demand
    hipEvent_t sim_ev[2];                   // ... ordered after and before the context's stream with these
    bool fused_lds_raised;                  // fused kernel: its dynamic LDS limit has been raised for this context
    bool loop_lds_raised;                   // the Schedule loop over totals: likewise
    bool nodes_lds_raised;                  // the Schedule loop over nodes: likewise
    unsigned char *static_scratch;          // this device's copy of the static scratch array (rk_allocate_static)
    bool place_lds_raised;                  // placement kernel: its dynamic LDS limit has been raised for this context
};

// scratch slots
enum {
    SL_CNT_T = 0, SL_CNT_S, SL_TOTALS,            // enumeration: per-job counts, totals
    SL_TB_TOFF, SL_TB_TRIPLES, SL_TB_SOFF, SL_TB_SEGG, SL_TB_SEGF,   // internal plan table of a round
    SL_BEST_THR, SL_BEST_PLAN, SL_CURVE_THR, SL_CURVE_PLAN, SL_CURVE_G,  // round intermediates
    SL_ROUND_META,                                // per-round job ranges and clusters
    SL_HULL_KEY, SL_HULL_RAW, SL_HULL_DG, SL_HULL_DC, SL_HULL_TGT,   // walk steps of the greedy allocation
    SL_ST_GI, SL_ST_G, SL_ST_CI, SL_ST_FREEC, SL_ST_PARTIAL,         // its per-job and per-round state
    SL_ST_STEP_SLOPE, SL_ST_STEP_TGT, SL_ST_STEP_DG, SL_ST_FREEG,
    SL_HIST_G, SL_HIST_C,                                             // cost histograms over the step keys
    SL_PARK,                                             // enumeration: sorted keys between its two passes
    SL_FL_GI, SL_FL_CI, SL_FL_WAITS, SL_FL_CAP0,         // service-level floors of the allocation
    SL_MIN_SEG, SL_MIN_C, SL_MIN_M,                      // minimum demands of a round
    SL_SIM_STATE, SL_SIM_ASSIGN,                         // simulation: per-job state, the tick's assignment
    SL_JMAP,                                             // rounds that share jobs: slot -> job
    SL_ENUM_BACK,                                        // enumeration: totals and offsets in one piece for the host
    SL_PLACE_RESULT,                                     // placement: its four summary words
    SL_ENUM_LEADER,                                      // enumeration: the job whose search a job shares
    SL_RS_F32, SL_RS_U32, SL_RS_U64,                     // the Schedule loop: cached slopes; order, marks and saved states; CPU needs
    SL_EVAL_PARTIAL,                                     // evaluation with best plan: keys of the segments that span tiles
    SL_PLACE_KEEP,                                       // placement: which jobs keep their earlier parts
    SL_PRIV_LIST,                                        // privileged jobs of the loop: the queued guaranteed jobs
    SL_SIM_PLACES,                                       // simulation over nodes: where the jobs are, where they go
    SL_ND_NODES, SL_ND_U32, SL_ND_F32, SL_ND_U64,        // the Schedule loop over nodes: node tables and their copy; per-job words
    SL_COUNT
};
static_assert(SL_COUNT <= RK_SCRATCH_SLOTS, "more scratch slots than the context holds");

int32_t rk_fail(rk_ctx *ctx, int32_t code, const char *fmt, ...);
int32_t rk_scratch(rk_ctx *ctx, int slot, size_t bytes, void **out);

#define RK_HIP(ctx, call)                                                              \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess)                                                          \
            return rk_fail((ctx), RK_ERR_DEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define RK_CHECK_LAUNCH(ctx, name)                                                     \
    do {                                                                               \
        hipError_t e_ = hipGetLastError();                                             \
        if (e_ != hipSuccess)                                                          \
            return rk_fail((ctx), RK_ERR_DEVICE, "launch of %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// argument validation shared by the entry points
int32_t rk_check_grid(rk_ctx *ctx, const rk_alloc_grid *grid);
int32_t rk_check_env(rk_ctx *ctx, const rk_env *env);
int32_t rk_check_table(rk_ctx *ctx, const rk_plan_table *table, uint32_t job_begin, uint32_t job_end);
// need_request: the request and baseline arrays must be present as well
int32_t rk_check_sla(rk_ctx *ctx, const rk_sla *sla, bool need_request);
// triple_off / seg_off at job_begin and job_end (host mirrors, or two copies back)
int32_t rk_range_offsets(rk_ctx *ctx, const rk_plan_table *table, uint32_t job_begin, uint32_t job_end,
                         uint64_t *n_triples, uint64_t *n_segs);

// device-side view of the plan table
struct TableDev {
    const uint32_t *__restrict__ triple_off;
    const uint32_t *__restrict__ triples;
    const uint32_t *__restrict__ seg_off;
    const uint32_t *__restrict__ seg_g;
    const uint32_t *__restrict__ seg_first;
};

static inline TableDev table_dev(const rk_plan_table *t) {
    return TableDev{t->triple_off, t->triples, t->seg_off, t->seg_g, t->seg_first};
}

// service-level inputs of the allocation; min_seg / min_c are indexed from the call's first job
struct SlaDev {
    const uint32_t *guaranteed, *tenant;
    const int32_t *min_seg;
    const uint32_t *min_c;
    uint32_t n_tenants;
    const uint32_t *quota_g, *quota_c;
};

// what a job does in a round that starts from floors
enum : uint8_t { RK_JOB_NORMAL = 0, RK_JOB_OUT = 1, RK_JOB_FROZEN = 2 };

// floors computed by the caller of the allocation (device arrays, indexed from the call's first job;
// cap0 = per round [free GPUs | free CPUs] left after the floors)
struct FloorsDev {
    int32_t *gi;
    uint32_t *ci;
    uint8_t *state;
    unsigned long long *cap0;
};

// launch wrappers (each enqueues on ctx->stream)
int32_t rk_launch_fused(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                        const rk_alloc_grid *grid, const rk_env *env, uint32_t jb, uint32_t je,
                        float *best_thr, uint32_t *best_plan, float *curve_thr, uint32_t *curve_plan,
                        uint32_t *curve_g);
// one_cluster != NULL: a single round over [jb, jb + n_jobs) with that cluster, carried in the
// kernel arguments; otherwise n_rounds rounds described by the device arrays.
// sla != NULL: service-level floors first (the quotas apply to every round alike);
// given != NULL: the floors are there already.
// d_jmap != NULL: slot j of the call (rounds, state, results are in slots) uses the plan table, curves and
// reference throughput of job d_jmap[j]; the curve arrays then cover the whole table from job 0.
int32_t rk_launch_allocate(rk_ctx *ctx, const float *ref_thr, const TableDev &tb, const rk_alloc_grid *grid,
                           uint32_t n_rounds, const uint32_t *d_round_off, const rk_cluster *d_clusters,
                           const rk_cluster *one_cluster, uint32_t jb, uint32_t n_jobs, uint32_t max_jobs,
                           uint32_t max_segs_per_job, const float *best_thr, const uint32_t *best_plan,
                           const float *curve_thr, const SlaDev *sla, const FloorsDev *given, const uint32_t *d_jmap,
                           rk_assign *assign, float *totals, bool static_scratch = false);
// static_scratch: the working buffers are pieces of the library's static device array (nothing is allocated; a
// round that needs more than the array holds is refused) instead of the context's grow-only buffers.
// Once per context, device current: finds this device's copy of that array and raises the LDS limits of the
// allocation kernels.
int32_t rk_allocate_setup(rk_ctx *ctx);
// minimum demands of the guaranteed jobs of [jb, je)
int32_t rk_launch_min_res(rk_ctx *ctx, const TableDev &tb, const rk_alloc_grid *grid, uint32_t jb, uint32_t je,
                          const float *best_thr, const rk_sla *sla, int32_t *min_seg, uint32_t *min_c,
                          uint32_t *min_m);

// placement that feeds the plan, over all jobs of the table (arguments as rk_place_plans, already validated)
int32_t rk_launch_place_plans(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                              const rk_env *env, const rk_nodes *nodes, const float *best_thr, const rk_assign *assign,
                              const int32_t *min_seg, const uint32_t *prev_off, const rk_place_entry *prev_entries,
                              rk_assign *placed, uint32_t *place_off, rk_place_entry *entries,
                              uint64_t cap_entries, uint32_t *status, float *total, rk_place_result *result);

// Algorithm 1's Schedule loop over the cluster's totals (arguments as rk_reschedule, already validated, device current)
int32_t rk_launch_reschedule(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table, const rk_alloc_grid *grid,
                             const rk_cluster *cluster, const float *best_thr, const uint32_t *best_plan,
                             const float *curve_thr, const rk_job_state *jobs_state, rk_assign *assign, float *total,
                             uint32_t *stats);
// ... and over its nodes (arguments as rk_reschedule_nodes, already validated, device current; entries holds at least
// n_nodes * gpus_per_node records)
int32_t rk_launch_reschedule_nodes(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                   const rk_alloc_grid *grid, const rk_nodes *nodes, const float *best_thr,
                                   const uint32_t *best_plan, const float *curve_thr, const rk_job_state *jobs_state,
                                   const uint32_t *prev_off, const rk_place_entry *prev_entries, uint64_t n_prev_entries,
                                   rk_assign *assign, uint32_t *place_off, rk_place_entry *entries, float *total,
                                   uint32_t *stats);
// GetBestPlan(j, placement) for a given placement (arguments as rk_best_plan_placed, already validated, device current)
int32_t rk_launch_best_plan_placed(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                                   const rk_env *env, const rk_assign *assign, const uint32_t *place_off,
                                   const rk_place_entry *entries, rk_assign *placed, float *total);
