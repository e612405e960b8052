/*
 * rubick.h - C ABI of the GPU plan-evaluation library (gfx950 / MI355X).
 *
 * The library evaluates the performance model of the Rubick scheduler
 * (arxiv 2408.08586, Sec. 4) for every (job x execution plan x resource
 * allocation) candidate, masks plans that do not fit in memory, takes the
 * best plan per (job, allocation) (GetBestPlan, Sec. 5.2 / Algorithm 1),
 * builds the per-job resource sensitivity curves (Sec. 5.2, Fig. 6) and runs a
 * slope-ordered greedy allocation over them (Sec. 5.2).
 *
 * Conventions
 *  - Every function returns RK_OK (0) or a negative error code; the text of
 *    the last error of a context is available from rk_last_error().  Nothing
 *    throws, aborts or allocates memory the caller must free.
 *  - Pointers marked [device] are device pointers on the context's GPU and
 *    must be 16-byte aligned; pointers marked [host] are ordinary host
 *    pointers.  Structs are host structs passed by pointer and are read
 *    before the call returns.  The caller owns every input and output buffer;
 *    the context owns only its scratch memory.  Inputs are never modified.
 *  - Work is enqueued on the context's HIP stream and calls return without
 *    waiting, except where a count has to come back to the host (stated per
 *    function).  rk_sync() waits for everything enqueued so far.
 *  - A context is not thread-safe; use one per host thread.
 *
 * Vocabulary (symbols as in Table 1 of the paper)
 *  triple    (d, t, p): data / tensor / pipeline parallel sizes, g = d*t*p GPUs
 *  option    o = z*4 + gc*2 + off: ZeRO stage z in 0..3, gradient
 *            checkpointing gc, offload off (ZeRO-Offload needs z >= 2)
 *  plan      (triple, option); plan index inside a job = triple_index*16 + o
 *  row       (cpu level ci, memory tier mi) of the allocation grid,
 *            r = ci*n_mem + mi
 *  candidate (job, row, plan)
 *  segment   all plans of one job with the same GPU count g
 *
 * Array layouts (jb = first job of the range a call works on)
 *  candidates: 16*n_rows*(triple_off[j]-triple_off[jb]) + (r*nt_j + tl)*16 + o
 *  segments  : n_rows*(seg_off[j]-seg_off[jb]) + r*ns_j + s
 *  with nt_j / ns_j the number of triples / segments of job j.
 */
#ifndef RUBICK_H
#define RUBICK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RK_OK                 0
#define RK_ERR_INVALID_ARG   (-1)   /* null pointer, bad size, bad level order ... */
#define RK_ERR_CAPACITY      (-2)   /* an output buffer is too small; needed size reported */
#define RK_ERR_DEVICE        (-3)   /* a HIP call failed; see rk_last_error() */
#define RK_ERR_UNSUPPORTED   (-4)   /* input outside the documented limits */

#define RK_NO_PLAN            0xFFFFFFFFu
#define RK_MAX_CPU_LEVELS     64
#define RK_MAX_MEM_LEVELS     16
#define RK_MAX_G              65535u   /* largest g_max */
#define RK_MAX_PP             4095u    /* largest pp_max */
#define RK_MAX_TRIPLES_PER_JOB 2048u
#define RK_MAX_JOBS_PER_ROUND 12288u   /* limit of the greedy allocation kernel */

/* reason bits of the optional feasibility output (0 = feasible) */
#define RK_INFEASIBLE_STRUCT  1u   /* option not allowed, or offload with z < 2 */
#define RK_INFEASIBLE_GPU_MEM 2u   /* estimated GPU memory above env.gpu_mem_cap */
#define RK_INFEASIBLE_HOST_MEM 4u  /* offloaded state above the memory tier */

/* packed triple: d in bits 0..15, log2(t) in bits 16..17, p in bits 18..29,
 * micro-batch shift v in bits 30..31 (the plan runs micro-batches of mu * 2^v samples) */
#define RK_TRIPLE_D(x)  ((x) & 0xFFFFu)
#define RK_TRIPLE_T(x)  (1u << (((x) >> 16) & 3u))
#define RK_TRIPLE_P(x)  (((x) >> 18) & 0xFFFu)
#define RK_TRIPLE_V(x)  ((x) >> 30)

typedef struct rk_ctx rk_ctx;

/* Job descriptors, struct of arrays of length n_jobs, all [device].
 * Model constants and fitted coefficients of Table 1 plus the coefficients of
 * the memory estimate (the paper delegates that estimate to the training
 * frameworks, Sec. 6; the form used here is documented with
 * rk_eval_candidates). */
typedef struct {
    uint32_t n_jobs;
    const float *P_bytes;       /* parameter size in bytes */
    const float *seq;           /* s */
    const float *hidden;        /* h */
    const float *elem_bytes;    /* bytes per activation element */
    const float *t_fwd_sample;  /* forward seconds of one sample, whole model, one GPU */
    const float *k_bwd, *k_sync, *k_opt, *k_opt_off, *k_off, *k_swap, *k_const;
    const float *mem_state;     /* scale of the model-state bytes */
    const float *mem_act;       /* activation bytes per token*hidden*layer */
    const float *mem_act_gc;    /* same, kept with gradient checkpointing */
    const float *mem_const;     /* constant bytes per GPU */
    const float *ref_thr;       /* reference throughput that normalises gains */
    const uint32_t *layers;     /* l */
    const uint32_t *gbatch;     /* b, global batch (kept fixed, Sec. 3) */
    const uint32_t *mbatch;     /* micro-batch size mu; b/(d*mu*2^v) micro-batches per replica */
} rk_jobs;

/* Plan space bounds: d*t*p <= g_max, t in {1,2,4,8} and <= tp_max, p <= pp_max
 * and p | layers, (d*mu*2^v) | b.  Option masks: bit v set = value v allowed.
 * mu_mask: micro-batch sizes a plan may use, bit v = mu * 2^v samples (Sec. 4.1
 * "Gradient Accumulation", Table 1: the numbers of micro-batches m and of
 * accumulation steps a belong to the plan); 1 = only the job's own mu. */
typedef struct {
    uint32_t g_max, tp_max, pp_max;
    uint32_t zero_mask;         /* 4 bits */
    uint32_t gc_mask;           /* 2 bits */
    uint32_t off_mask;          /* 2 bits */
    uint32_t mu_mask;           /* 4 bits, not 0 */
} rk_plan_bounds;

/* Plan table (CSR over jobs). Buffers are caller-owned [device]; the scalar
 * fields and the optional host mirrors are written by rk_enumerate_plans. */
typedef struct {
    uint32_t *triple_off;       /* [device] [n_jobs+1] */
    uint32_t *triples;          /* [device] [cap_triples] packed, order g, t, p, v ascending */
    uint32_t *seg_off;          /* [device] [n_jobs+1] */
    uint32_t *seg_g;            /* [device] [cap_segs] GPU count of each segment */
    uint32_t *seg_first;        /* [device] [cap_segs] first triple of the segment (job-local) */
    uint64_t cap_triples, cap_segs;
    uint32_t *h_triple_off;     /* [host] optional mirror [n_jobs+1], may be NULL */
    uint32_t *h_seg_off;        /* [host] optional mirror [n_jobs+1], may be NULL */
    /* outputs */
    uint64_t n_triples, n_segs;
    uint32_t n_jobs;
    uint32_t max_triples_per_job, max_segs_per_job;
    uint32_t option_mask;       /* bit o set: option code o allowed by the bounds */
} rk_plan_table;

/* Allocation grid: CPU levels and host-memory tiers, both ascending. */
typedef struct {
    uint32_t n_cpu;
    uint32_t cpu_levels[RK_MAX_CPU_LEVELS];   /* >= 1 */
    uint32_t cpu_mode;          /* 0: CPUs of the whole job; 1: CPUs per GPU (c = level*g) */
    uint32_t n_mem;
    float mem_levels_gb[RK_MAX_MEM_LEVELS];   /* GiB */
    uint32_t mem_mode;          /* 0: GiB of the whole job; 1: GiB per GPU */
} rk_alloc_grid;

/* Environment constants of Table 1 plus the node shape. */
typedef struct {
    float B_intra, B_inter, B_pcie;   /* bytes/s */
    float gpu_mem_cap;                /* bytes */
    uint32_t gpus_per_node;
} rk_env;

typedef struct {
    uint32_t G, C;              /* free GPUs and CPUs of the cluster */
    float host_mem_gb;          /* free host memory, GiB */
} rk_cluster;

/* Result of the allocation for one job; g == 0: not scheduled this round. */
typedef struct {
    uint32_t g, c;
    float mem_gb;
    uint32_t plan;              /* plan index inside the job, or RK_NO_PLAN */
    float thr;                  /* predicted samples/s */
} rk_assign;

/* Context: binds a device and a stream.  hip_stream is a hipStream_t (NULL =
 * the default stream).  rk_destroy frees the scratch memory. */
int32_t rk_create(rk_ctx **ctx, int32_t device_id, void *hip_stream);
int32_t rk_destroy(rk_ctx *ctx);
int32_t rk_sync(rk_ctx *ctx);
const char *rk_last_error(const rk_ctx *ctx);

/* Plan enumeration (Sec. 3 "execution plans", Table 1: d*t*p = g; Fig. 6:
 * only some GPU counts are valid because of the partitioning constraints).
 * Factorises every g <= g_max on the device and writes the table.
 * With table->triples == NULL only the counts (n_triples, n_segs, maxima) are
 * produced.  Too small capacities give RK_ERR_CAPACITY with the counts set and
 * the table's triples and segments untouched (the offsets are written).
 * Waits until the counts have come back to the host; the kernel that fills the
 * table may still be running on the stream when the call returns. */
int32_t rk_enumerate_plans(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                           rk_plan_table *table);

/* Candidate evaluation (Sec. 4, Eq. 1: T_iter = T_cc + T_oo + k_const,
 * throughput = b / T_iter) with memory-feasibility masking (Sec. 5.2: a plan
 * must train without running out of GPU memory; host memory is allocated from
 * the plan's estimate).  Jobs [job_begin, job_end).
 *   thr  [device] float32 per candidate, 0 where infeasible
 *   feas [device] optional reason bits per candidate (NULL to skip)
 *   cap  capacity of thr (and feas) in elements; *n_needed (optional, [host])
 *        receives the candidate count of the range.
 * Memory estimate, float32, one rounding per operation in this order:
 *   Psi = P_bytes/(t*p); kappa = 8 | 2+6/d | 1+7/d | 8/d (ZeRO 0..3),
 *   with offload 1 (z=2) | 1/d (z=3); S = (mem_state*kappa)*Psi;
 *   mu = the plan's micro-batch size (the job's mbatch * 2^v);
 *   tok = (mu*seq)*hidden; base = ((tok*(l/p))/t)*min(p, b/(d*mu));
 *   A = mem_act*base, or mem_act_gc*base + (mem_act*tok)/t with checkpointing;
 *   M_gpu = (S+A)+mem_const <= gpu_mem_cap;
 *   H_host = ((mem_state*(7/d))*Psi)*g <= tier bytes (GiB*2^30, *g per GPU).
 * Needs the host offsets: uses the table's host mirrors when present, else
 * copies two offsets back (waits for the stream). */
int32_t rk_eval_candidates(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                           const rk_alloc_grid *grid, const rk_env *env,
                           uint32_t job_begin, uint32_t job_end,
                           float *thr, uint8_t *feas_or_null, uint64_t cap, uint64_t *n_needed);

/* Best plan per segment and row (GetBestPlan, Sec. 5.2): maximum throughput,
 * lowest plan index among equal maxima; a segment without a feasible plan
 * gives (0, RK_NO_PLAN).  thr must hold non-negative, non-NaN values in the
 * candidate layout of the same job range.  cap_segs = capacity of the outputs;
 * *n_needed (optional, [host]) receives n_rows * segments of the range. */
int32_t rk_best_plan(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid,
                     uint32_t job_begin, uint32_t job_end, const float *thr,
                     float *best_thr, uint32_t *best_plan, uint64_t cap_segs, uint64_t *n_needed);

/* rk_eval_candidates and rk_best_plan in one pass over jobs [job_begin,
 * job_end) (Sec. 4, Eq. 1 and GetBestPlan, Sec. 5.2): thr (and feas, if given)
 * receive exactly what rk_eval_candidates writes, best_thr / best_plan exactly
 * what rk_best_plan then gives on that thr, but the candidates are reduced
 * while they are still in registers, so the tensor is written once and not
 * read back.  cap = capacity of thr (and feas) in candidates, cap_segs = of the
 * two segment outputs in entries; RK_ERR_CAPACITY when either is too small.
 * A segment whose plans lie in more than one 64-triple tile is finished by a
 * second, small kernel from keys kept in a buffer the context owns (it grows
 * on first use: 16 bytes per tile and row).  At most 65535 jobs per call. */
int32_t rk_eval_best_plan(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                          const rk_alloc_grid *grid, const rk_env *env,
                          uint32_t job_begin, uint32_t job_end,
                          float *thr, uint8_t *feas_or_null, uint64_t cap,
                          float *best_thr, uint32_t *best_plan, uint64_t cap_segs);

/* Resource sensitivity curves from the per-segment maxima (Sec. 5.2, Fig. 6):
 * per job and row, over the job's GPU counts in ascending order, the best
 * throughput achievable within that many GPUs, its plan and the smallest GPU
 * count reaching it (0 while nothing is feasible). Same layout as the inputs. */
int32_t rk_curves(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid,
                  uint32_t job_begin, uint32_t job_end,
                  const float *best_thr, const uint32_t *best_plan,
                  float *curve_thr, uint32_t *curve_plan, uint32_t *curve_g, uint64_t cap_segs);

/* The slope table of the curves (Sec. 5.2: a job's slope, per resource type, is
 * the throughput change per unit of the resource; Fig. 6): the steps the
 * allocation rules take, independent of the cluster.  For jobs [job_begin,
 * job_end), arrays in segment layout ([job][CPU level][tier][GPU count]):
 *   gpu_slope, gpu_next   from that GPU count to the larger count with the
 *                         highest float32 slope ((v1 - v0) / ref_thr) / (g1 - g0)
 *                         on the curve of the row, the smaller count among equal
 *                         slopes; index of that count in the job's list, -1 and
 *                         slope 0 when no larger count is better
 *   cpu_slope, cpu_next   at that GPU count from the row's CPU level to the level
 *                         with the highest ((best' - best) / ref_thr) / (CPUs' -
 *                         CPUs), the lower level among equals; n_cpu and slope 0
 *                         when no higher level is better
 *   from0_slope, from0_next   per job and row ([job][CPU level][tier]): the first
 *                         GPU step of a job that holds nothing
 * best_thr, curve_thr as rk_best_plan / rk_curves (or rk_job_curves) write them
 * for the same range.  cap_segs = capacity of the four segment-layout outputs. */
int32_t rk_curve_slopes(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                        const rk_alloc_grid *grid, uint32_t job_begin, uint32_t job_end,
                        const float *best_thr, const float *curve_thr, float *gpu_slope, int32_t *gpu_next,
                        float *from0_slope, int32_t *from0_next, float *cpu_slope, uint32_t *cpu_next,
                        uint64_t cap_segs);

/* Evaluation + best plan + curves in one pass without materialising the
 * candidates; results are identical to rk_eval_candidates -> rk_best_plan ->
 * rk_curves.  best_thr / best_plan may be NULL. */
int32_t rk_job_curves(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                      const rk_alloc_grid *grid, const rk_env *env,
                      uint32_t job_begin, uint32_t job_end,
                      float *best_thr_or_null, uint32_t *best_plan_or_null,
                      float *curve_thr, uint32_t *curve_plan, uint32_t *curve_g, uint64_t cap_segs);

/* Greedy allocation over the curves of jobs [job_begin, job_end) (Sec. 5.2:
 * jobs that gain the most per unit of resource first, GPU slopes before CPU
 * slopes, memory from the chosen plan last).  The arrays are in segment
 * layout of the same job range (they may be NULL when the table has no
 * segment at all: then no job gets anything).  float32 slopes
 * ((v1-v0)/ref_thr)/delta.
 *   assign [device] one record per job of the range
 *   total  [device] one float: sum of thr/ref_thr over scheduled jobs */
int32_t rk_allocate(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                    const rk_alloc_grid *grid, const rk_cluster *cluster,
                    uint32_t job_begin, uint32_t job_end,
                    const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                    rk_assign *assign, float *total);

/* rk_allocate for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results; the working buffers
 * (walk steps, per-job state, histograms) are pieces of one 12 MiB array that
 * lives in the library's image on every device instead of buffers the context
 * allocates on demand.  The call allocates and frees nothing and copies
 * nothing.  Limits: (je - jb) * max(longest GPU-count list of a job,
 * grid->n_cpu) <= RK_STATIC_MAX_STEPS and je - jb <= RK_MAX_JOBS_PER_ROUND,
 * otherwise RK_ERR_UNSUPPORTED and nothing is launched.  All calls on one
 * device share that array, whatever their context or stream, and it keeps the
 * last call's contents (the kernels clear what they need cleared): two calls
 * that overlap in time on one device race; calls on one stream, or ordered by
 * events, are fine. */
#define RK_STATIC_MAX_STEPS 524288u
int32_t rk_allocate_static(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                           const rk_alloc_grid *grid, const rk_cluster *cluster,
                           uint32_t job_begin, uint32_t job_end,
                           const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                           rk_assign *assign, float *total);

/* What the jobs of the table hold and are guaranteed, all [device], one entry
 * per job.  state: 0 the job takes part; 2 it keeps exactly what it holds (it
 * takes no step and gives nothing: a job that must not be reconfigured now);
 * any other value: it takes no part and holds nothing (NULL: all take part).  cur_seg: index of the GPU count it holds in its
 * list, -1 nothing; cur_c: the CPU level it holds.  floor_seg / floor_c: its
 * minimum demand as rk_min_res gives it (-1, or NULL: none). */
typedef struct {
    const uint8_t *state;
    const int32_t *cur_seg;
    const uint32_t *cur_c;
    const int32_t *floor_seg;
    const uint32_t *floor_c;
} rk_job_state;

/* Algorithm 1's Schedule as the loop it is written as, from the state the jobs
 * are in (Sec. 5.2 "Scheduling algorithm design" and the paragraph on shrinking:
 * running jobs keep what they hold unless a job with a higher slope, or one
 * below its minimum demand, takes it).  Over all jobs of the table, arrays in
 * segment layout as for rk_allocate.
 *  - Privileged jobs first, in job order: those with a floor that hold fewer
 *    GPUs than it.  Then all others that take part, sorted once by their GPU
 *    slope, then CPU slope (descending), then index.
 *  - ScheduleJob(j), for GPUs and then CPUs: while j has a next step (below its
 *    floor: to the floor with the floor's CPU level; otherwise the larger
 *    amount with the highest float32 slope ((v1-v0)/ref_thr)/delta, the smaller
 *    amount among equal slopes), what the step needs is gathered from what is
 *    free, then from the other jobs, always the one with the lowest slope among
 *    those above their own floor (GetLowestSlopeOverMinJob; lower index on
 *    ties).  A job that gives steps down to the largest amount with a lower
 *    throughput (the smallest with the same throughput if it holds more than
 *    it uses), not below its floor; its slope is the normalised throughput it
 *    loses per unit given.  It may be shrunk when j's slope is higher than its
 *    own or j is below its floor.  The step is committed when all was found
 *    (a GPU step needs its CPUs at j's level free or freed by the same shrinks)
 *    and, unless j is below its floor, j gains more than the others lose;
 *    otherwise every job is put back and j's search in that resource ends.
 *  - Memory last, as in rk_allocate.  A job shrunk to nothing is preempted.
 *   assign  [device] n_jobs records; total [device] one float
 *   stats   [device] four words or NULL: steps committed, jobs that needed more
 *           than a look (a step that was free to take, or a job it might shrink),
 *           shrinks applied, steps taken back
 * Limits: at most RK_MAX_JOBS_PER_ROUND jobs.  One workgroup runs the loop: the
 * rule is sequential. */
int32_t rk_reschedule(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                      const rk_alloc_grid *grid, const rk_cluster *cluster,
                      const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                      const rk_job_state *jobs_state, rk_assign *assign, float *total, uint32_t *stats);

/* Many independent rounds of that loop over the same jobs and curves at once, a
 * workgroup per round (what-if questions: other capacities, other states of the
 * jobs; Sec. 5.2: the curves do not depend on the cluster's state).
 *   clusters     [host] n_rounds entries: capacity of round r
 *   jobs_state   arrays [device]; state_stride 0: every round starts from the same
 *                state (n_jobs entries per array); state_stride n_jobs: round r
 *                reads entries [r * n_jobs, (r + 1) * n_jobs) of every array given
 *   assign       [device] n_rounds * n_jobs records, round r at r * n_jobs
 *   totals       [device] n_rounds floats
 *   stats        [device] 4 * n_rounds words or NULL
 * Every round's result is what rk_reschedule gives for its cluster and state.
 * Limits: n_rounds <= 65535, n_rounds * n_jobs <= 2^26. */
int32_t rk_reschedule_rounds(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                             const rk_alloc_grid *grid, uint32_t n_rounds, const rk_cluster *clusters,
                             const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                             const rk_job_state *jobs_state, uint32_t state_stride, rk_assign *assign,
                             float *totals, uint32_t *stats_or_null);

/* One scheduling round end to end: enumerate -> evaluate -> best plan ->
 * curves -> greedy allocation, all on the device.  Waits once for the plan
 * counts. assign [device] n_jobs records, total [device] one float. */
int32_t rk_schedule_round(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                          const rk_alloc_grid *grid, const rk_env *env, const rk_cluster *cluster,
                          rk_assign *assign, float *total);

/* n_rounds independent rounds over one concatenated job array: round r owns
 * jobs [round_off[r], round_off[r+1]) and cluster clusters[r] (both [host]).
 * assign [device] n_jobs records, totals [device] n_rounds floats. */
int32_t rk_schedule_rounds(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                           const rk_alloc_grid *grid, const rk_env *env,
                           uint32_t n_rounds, const uint32_t *round_off, const rk_cluster *clusters,
                           rk_assign *assign, float *totals);

/* Rounds that share jobs (Sec. 5.2: the curves "can be computed in parallel or
 * even prior to the scheduling, and then cached for reuse"): round r schedules
 * the slots [round_off[r], round_off[r+1]) and slot i stands for job
 * round_jobs[i] of the job array (both [host]; a job may appear in any number
 * of rounds, at most once per round).  Every job is enumerated and evaluated
 * once.  assign [device] one record per slot, totals [device] n_rounds floats.
 * Results per round are those of rk_schedule_round on the round's jobs in slot
 * order. */
int32_t rk_schedule_rounds_shared(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                                  const rk_alloc_grid *grid, const rk_env *env,
                                  uint32_t n_rounds, const uint32_t *round_off, const uint32_t *round_jobs,
                                  const rk_cluster *clusters, rk_assign *assign, float *totals);

/* ---- service-level floors (Sec. 5.2 "Scheduling algorithm design") -------- */

#define RK_MAX_TENANTS 256u

/* Service-level inputs.  Per-job arrays are [device], length n_jobs of the
 * job array, indexed by job.  quota_* are [device] [n_tenants]. */
typedef struct {
    const uint32_t *guaranteed; /* != 0: guaranteed job; 0: best-effort */
    const uint32_t *tenant;     /* tenant index (>= n_tenants: the job waits) */
    const uint32_t *req_g;      /* requested GPUs */
    const uint32_t *req_c;      /* requested CPU level (index into the grid, clamped) */
    const uint32_t *req_m;      /* requested memory tier (index into the grid, clamped) */
    const float *base_thr;      /* throughput of the request with the job's original plan */
    uint32_t n_tenants;         /* <= RK_MAX_TENANTS */
    const uint32_t *quota_g;    /* GPUs the tenant's guaranteed jobs may hold */
    const uint32_t *quota_c;    /* CPUs likewise */
} rk_sla;

/* Throughput of chosen points (Sec. 4, Eq. 1, same arithmetic and masking as
 * rk_eval_candidates): point i is job pt_job[i], plan index pt_plan[i] inside
 * the job (triple*16 + option), CPU level pt_c[i], memory tier pt_m[i], all
 * [device] [n_points].  thr [device] receives 0 for infeasible points and for
 * points whose indices are out of range; feas_or_null [device] the reason
 * bits (RK_INFEASIBLE_STRUCT for out-of-range points).  Serves e.g. the
 * baseline of a guaranteed job: its original plan at its requested resources. */
int32_t rk_eval_points(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                       const rk_alloc_grid *grid, const rk_env *env, uint64_t n_points,
                       const uint32_t *pt_job, const uint32_t *pt_plan, const uint32_t *pt_c,
                       const uint32_t *pt_m, float *thr, uint8_t *feas_or_null);

/* Minimum demand of the guaranteed jobs in [job_begin, job_end) (Sec. 5.2: the
 * fewest resources, not above the request in any dimension, with which the
 * best plan reaches the baseline performance).  "Fewest" = fewest GPUs, then
 * fewest CPUs, then the smallest memory tier; a point qualifies when
 * best_thr > 0 and best_thr >= base_thr.  If none qualifies the request itself
 * (GPU count rounded down to a valid one) is the minimum.  best_thr is in
 * segment layout of the range.  Outputs [device], one per job of the range:
 * min_seg = segment index inside the job, or -1 for best-effort jobs and for
 * requests below the job's smallest valid GPU count; min_c, min_m = levels. */
int32_t rk_min_res(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid,
                   uint32_t job_begin, uint32_t job_end, const float *best_thr, const rk_sla *sla,
                   int32_t *min_seg, uint32_t *min_c, uint32_t *min_m);

/* rk_allocate with service-level floors (Sec. 5.2: guaranteed jobs within
 * their tenant's quota are served first with at least their minimum demand,
 * the rest goes to the highest slopes).  Privileged phase, in job order: a
 * guaranteed job whose minimum (min_seg, min_c of the range, [device]) fits
 * its tenant's remaining quota and the free GPUs and CPUs is granted it;
 * otherwise it waits (g = 0 in the result) and takes no part in the round.
 * Then the greedy runs from these floors on what is left; a job's GPU steps
 * are valued at its floor's CPU level.  sla->req_* and base_thr are not read. */
int32_t rk_allocate_sla(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                        const rk_alloc_grid *grid, const rk_cluster *cluster,
                        uint32_t job_begin, uint32_t job_end,
                        const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                        const rk_sla *sla, const int32_t *min_seg, const uint32_t *min_c,
                        rk_assign *assign, float *total);

/* rk_schedule_round with service levels: enumerate -> evaluate / best plan /
 * curves -> minimum demands -> privileged phase -> greedy from the floors. */
int32_t rk_schedule_round_sla(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                              const rk_alloc_grid *grid, const rk_env *env, const rk_cluster *cluster,
                              const rk_sla *sla, rk_assign *assign, float *total);

/* ---- model fitting (Sec. 4 "Continuous model fitting") -------------------- */

#define RK_FIT_PARAMS 7          /* k_bwd, k_sync, k_opt, k_opt_off, k_off, k_swap, k_const */
#define RK_FIT_MAX_STARTS 8u
#define RK_FIT_MAX_SAMPLES 64u   /* per model */
#define RK_FIT_K_MAX 32.0        /* largest overlap exponent the fit may choose */

/* Measured test runs, CSR over the models (= jobs of the job array): run i of
 * model j used the plan (triple[i], option[i]) on cpus[i] CPUs and reached
 * thr[i] samples/s.  Arrays are [device]. */
typedef struct {
    const uint32_t *sample_off; /* [n_jobs+1] */
    const uint32_t *triple;     /* packed (d,t,p) as in the plan table */
    const uint32_t *option;     /* option code z*4 + gc*2 + off */
    const uint32_t *cpus;       /* CPUs of the job in that run */
    const float *thr;           /* measured throughput */
    uint32_t max_samples;       /* largest number of runs of one model, <= RK_FIT_MAX_SAMPLES */
} rk_samples;

typedef struct {
    uint32_t max_iter;          /* iterations per starting point */
    float refit_threshold;      /* a model whose current RMSLE is <= this keeps its parameters */
    uint32_t n_starts;          /* extra starting points, <= RK_FIT_MAX_STARTS */
    const double *start_offsets;/* [host] [n_starts][7]: the four scales are multiplied by exp(offset),
                                   1/k of the three exponents likewise */
} rk_fit_options;

/* Results, all [device], one entry per model; any pointer may be NULL. */
typedef struct {
    float *k_bwd, *k_sync, *k_opt, *k_opt_off, *k_off, *k_swap, *k_const;   /* fitted parameters, float32 */
    double *theta;              /* [n_jobs][7] the same in float64 */
    float *rmsle_before;        /* error of the current parameters (projected onto the feasible set) */
    float *rmsle_after;         /* error of the returned parameters */
    uint32_t *iters;            /* iterations spent, all starting points together; 0 = left unchanged;
                                   UINT32_MAX = the model has more runs than max_samples and was left unchanged */
} rk_fit_result;

/* Fits the seven fittable parameters of every model (Table 1; Sec. 4: they
 * minimise the root mean squared logarithmic error between Eq. 1 and the
 * measured runs, at least seven runs per model, three of them offloaded; the
 * model is updated again when its error exceeds a threshold).
 *   error   = sqrt(mean((ln(1+pred) - ln(1+thr))^2)) over the model's runs, float64;
 *             a structurally invalid run predicts 0
 *   set     = k_bwd, k_opt, k_opt_off, k_const >= 0; k_sync, k_off, k_swap in [1, RK_FIT_K_MAX]
 *   method  = projected Levenberg-Marquardt in (scales, 1/k) from the job's current
 *             parameters and from each extra starting point; then, twice over the three
 *             exponents, one that sits on a bound is moved to k = 1/0.3 and the descent
 *             repeated from the best point; the lowest error wins, the earlier on ties
 * The remaining coefficients of the jobs (P_bytes ... t_fwd_sample, layers, batch
 * sizes) are the known constants of the model.  Memory feasibility plays no part. */
int32_t rk_fit_models(rk_ctx *ctx, const rk_jobs *jobs, const rk_env *env, const rk_samples *samples,
                      const rk_fit_options *options, const rk_fit_result *result);

/* ---- reconfiguration penalty and discrete-time simulation (Sec. 5.2, 7.4) -- */

/* Arrival trace, [device] arrays of one entry per job of the plan table. */
typedef struct {
    const double *arrival;      /* seconds */
    const double *work;         /* samples to train */
    const double *delta;        /* checkpoint-resume cost of one reconfiguration, seconds */
} rk_trace;

/* Nodes of the cluster, all alike. */
#define RK_MAX_NODES 4096u
typedef struct {
    uint32_t n_nodes;           /* 1..RK_MAX_NODES */
    uint32_t gpus_per_node;     /* 1..65535 */
    uint32_t cpus_per_node;     /* 0..65535 */
    float mem_per_node_gb;      /* GiB of host memory */
} rk_nodes;

typedef struct {
    double dt;                  /* tick length, seconds, > 0 */
    uint32_t n_ticks;
    uint32_t policy;            /* the round of every tick: 0 the greedy from scratch (as rk_allocate) with the
                                   frozen jobs charged first; 1 Algorithm 1's Schedule loop from what the jobs
                                   hold (as rk_reschedule: running jobs keep it unless a job with a higher
                                   slope takes it; frozen jobs in state 2); 2 the same loop over nodes */
    double gate;                /* threshold of the reconfiguration rule (the paper uses 0.97) */
    const rk_nodes *nodes;      /* [host] policy 2 only (otherwise not read): the loop searches node by node (as
                                   rk_reschedule_nodes) from the placement the last tick left; the grid's CPU
                                   levels must be per GPU */
} rk_sim_options;

/* Results, all [device]; per job: finish (seconds, -1 if unfinished), n_reconf,
 * progress (samples), held (seconds with resources); per tick: GPUs in use,
 * total normalised throughput, number of frozen jobs.  Any pointer may be NULL. */
typedef struct {
    double *finish;
    uint32_t *n_reconf;
    double *progress;
    double *held;
    uint32_t *gpus_in_use;      /* [n_ticks] */
    float *totals;              /* [n_ticks] */
    uint32_t *frozen;           /* [n_ticks] */
} rk_sim_result;

/* Discrete-time simulation of the whole job set on cached curves (Sec. 5.2: the
 * curves do not depend on the cluster's state and can be computed once; the
 * reconfiguration rule compares (T - N*delta)/T with a threshold; Sec. 7.4: a
 * discrete-time simulator).  The arrays best_thr, best_plan, curve_thr are in
 * segment layout of all jobs (as rk_job_curves writes them for [0, n_jobs)).
 * Every tick k, at t = k*dt:
 *   - a job is active when arrival <= t and it has not finished;
 *   - an active job holding GPUs is frozen unless T - (N+1)*delta > gate*T, with
 *     T the seconds it has held resources and N its reconfigurations so far;
 *   - one round: inactive jobs take no part, frozen jobs keep their GPUs and
 *     CPUs.  Policy 0: the greedy from scratch (as rk_allocate), the frozen jobs
 *     charged first.  Policy 1 (Sec. 5.2: the policy is triggered whenever jobs
 *     are submitted or completed; here every tick): the Schedule loop from what
 *     the jobs hold (as rk_reschedule, no floors);
 *   - a job that keeps running with different (GPUs, CPUs, plan) is reconfigured:
 *     N += 1 and delta seconds are owed; starting from or stopping at zero is free;
 *   - a job holding GPUs pays owed seconds out of the tick, then trains at the
 *     round's throughput; it finishes inside the tick at t + paid + remaining/thr.
 * Times and progress are float64.  Runs on a stream of its own, ordered after the
 * work already enqueued on the context's stream (the first tick eagerly, the
 * others as replays of one captured HIP graph); with more than one tick the call
 * returns when the simulation has finished. */
int32_t rk_simulate(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                    const rk_alloc_grid *grid, const rk_cluster *cluster,
                    const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                    const rk_trace *trace, const rk_sim_options *options, const rk_sim_result *result);

/* One part of a job's placement: g GPUs, c CPUs and mem_gb GiB on a node. */
typedef struct { uint32_t node, g, c; float mem_gb; } rk_place_entry;

typedef struct {
    uint32_t n_entries;         /* parts written */
    uint32_t n_placed;          /* jobs with status 1 */
    uint32_t n_failed;          /* jobs with status 2 */
    uint32_t in_order;          /* 1: the job-by-job search ran (some node's CPUs or memory could bind) */
} rk_place_result;

/* Node-level placement of an allocation (Sec. 5.2, Algorithm 1, ScheduleJob:
 * the job walks the nodes in order, takes what each has free and records
 * {node, resources}; it is placed only when its whole amount has been found).
 * Jobs are taken in index order, every node starts empty.  On a node a job
 * of (g, c, mem) takes the most GPUs k, up to what it still lacks, such that
 * ceil(c*k/g) CPUs and mem*k/g GiB are free there; the part is booked with
 * floor(c*(done+k)/g) - floor(c*done/g) CPUs (done = its GPUs on earlier nodes,
 * so the parts add up to c) and mem*k/g GiB (float32).  A job whose g GPUs
 * are not found takes nothing.
 *   assign     [device] n_jobs records (as rk_allocate writes them); g == 0: no parts;
 *              mem_gb must not be negative (a NaN or negative amount gives an unspecified placement)
 *   place_off  [device] n_jobs + 1 offsets into entries (CSR over jobs)
 *   entries    [device] cap_entries records; cap_entries >= n_nodes * gpus_per_node
 *   status     [device] n_jobs words: 0 nothing to place, 1 placed, 2 not placed
 *   result     [host] or NULL; when given the call waits for the stream */
int32_t rk_place(rk_ctx *ctx, const rk_nodes *nodes, uint32_t n_jobs, const rk_assign *assign,
                 uint32_t *place_off, rk_place_entry *entries, uint64_t cap_entries, uint32_t *status,
                 rk_place_result *result);

/* Placement that feeds the plan (Sec. 5.2, Algorithm 1, ScheduleJob: after the
 * walk over the nodes the plan is selected given the found placement and memory
 * is allocated from its estimate; last paragraph of Sec. 5.2: a job placed on
 * several nodes is predicted with the inter-node bandwidth; Sec. 4.1: the
 * bottleneck bandwidth of a communication group decides).  Over all jobs of the
 * table, in index order, every node starts empty:
 *  - a job tries first fit (as rk_place) with the amounts of assign[j], which
 *    must be a valid GPU count of the job, a CPU level and a memory tier of the
 *    grid at that count, with a feasible plan there (what rk_allocate and its
 *    relatives write; any other record gets status 3, books nothing and counts
 *    among result->n_failed);
 *  - if the nodes do not hold them it falls back to its next smaller GPU count
 *    that has a feasible plan at the same CPU level and memory tier (CPUs and
 *    GiB follow the grid's modes), and so on, but not below its floor
 *    (min_seg[j] = segment index, NULL or -1 = none): what the search found is
 *    accepted as long as the minimum demand is met;
 *  - the plan of a placed job is searched again among the plans of its GPU
 *    count, each evaluated (Sec. 4, Eq. 1, arithmetic of rk_eval_candidates)
 *    with bandwidths from the actual node split: ranks fill the job's GPU slots
 *    in placement order, tensor-parallel ranks adjacent, then data-parallel,
 *    then pipeline stages, and a kind of group uses B_intra only if every group
 *    of that kind has all its ranks on one node.
 *  - with an earlier placement of the same jobs (prev_off, prev_entries, in
 *    the layout this call writes; both NULL: every node starts empty) running
 *    jobs stay where they are (ScheduleJob adds to what a job holds): a job
 *    whose amounts are what its earlier parts add up to - the same GPUs and
 *    CPUs, every part what first fit books for these amounts on that split -
 *    keeps those parts (status 1); all kept jobs are booked, in index order,
 *    before any other job looks for room.  If the kept parts do not fit the
 *    nodes the earlier placement is ignored as a whole.  Must not alias the
 *    output buffers.
 *   best_thr  [device] segment layout of all jobs (tells which counts have a feasible plan)
 *   placed    [device] n_jobs records: the amounts placed, the plan and its throughput
 *             (zeros and RK_NO_PLAN for a job that got nothing)
 *   place_off, entries, cap_entries, result: as rk_place
 *   status    [device] 0 nothing to place, 1 placed as asked, 2 placed with fewer GPUs, 3 not placed
 *   total     [device] one float: sum of thr/ref_thr over the placed jobs */
int32_t rk_place_plans(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                       const rk_env *env, const rk_nodes *nodes, const float *best_thr, const rk_assign *assign,
                       const int32_t *min_seg_or_null, const uint32_t *prev_off_or_null,
                       const rk_place_entry *prev_entries_or_null, rk_assign *placed, uint32_t *place_off,
                       rk_place_entry *entries, uint64_t cap_entries, uint32_t *status, float *total,
                       rk_place_result *result);

/* GetBestPlan(j, placement) for a placement that is there already (Sec. 5.2,
 * Algorithm 1, ScheduleJob after the search; Sec. 4.1: the bottleneck
 * bandwidth of a communication group decides): for every job with parts in
 * (place_off, entries) the best plan of the GPU count its parts add up to, at
 * the CPU level and memory tier of assign[j], evaluated with the bandwidths of
 * the actual node split - the selection rk_place_plans makes after placing,
 * without placing anything and without waiting for the stream.  The parts must
 * be in the order the job's ranks fill them (ascending nodes for the library's
 * own placements).
 *   assign     [device] n_jobs records: g, c, mem_gb locate the CPU level and tier
 *              (amounts that are not on the grid give an empty record)
 *   place_off  [device] n_jobs + 1 offsets into entries [device]
 *   placed     [device] n_jobs records: the amounts placed, plan and throughput
 *   total      [device] one float: sum of thr / ref_thr */
int32_t rk_best_plan_placed(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                            const rk_alloc_grid *grid, const rk_env *env, const rk_assign *assign,
                            const uint32_t *place_off, const rk_place_entry *entries, rk_assign *placed,
                            float *total);

/* A whole round on nodes (Sec. 5.2, Algorithm 1): rk_schedule_round (with sla ==
 * NULL) or rk_schedule_round_sla against what the nodes hold together, then
 * rk_place_plans with the floors of the guaranteed jobs.  assign [device]
 * n_jobs records receives the amounts the allocation decided, placed what
 * came of them on the nodes; total is that of the placed jobs. */
int32_t rk_schedule_round_placed(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                                 const rk_alloc_grid *grid, const rk_env *env, const rk_nodes *nodes,
                                 const rk_sla *sla_or_null, rk_assign *assign, rk_assign *placed,
                                 uint32_t *place_off, rk_place_entry *entries, uint64_t cap_entries,
                                 uint32_t *status, float *total, rk_place_result *result);

/* Who is privileged when Schedule runs from a running state (Sec. 5.2: the
 * guaranteed jobs whose demands are within their tenant's remaining quota are
 * scheduled first; the quota usage of a job is its minimum demand): turns the
 * service levels into the floors and states rk_reschedule, rk_reschedule_rounds
 * and rk_reschedule_nodes take.  Over all jobs of the table.
 *  - A guaranteed job that holds something (held: state, cur_seg, cur_c) keeps
 *    taking part; its minimum demand (min_seg, min_c as rk_min_res gives them;
 *    none when min_seg is no index of its list or its tenant is unknown) is its
 *    floor and is charged to its tenant's quota before any queued job is looked
 *    at; a quota does not go below zero.
 *  - Queued guaranteed jobs, in job order: a job whose minimum demand (GPUs,
 *    CPUs) fits what is left of its tenant's quota gets it as its floor - the
 *    loop then serves it first - and charges the quota; a job that does not
 *    fit, or has no minimum demand, waits: state 1.
 *  - Best-effort jobs have no floor.  A job whose given state says it takes no
 *    part keeps that state and charges nothing.
 *   sla        guaranteed, tenant, n_tenants, quota_g, quota_c are read
 *   floor_seg, floor_c, state_out   [device] n_jobs entries each (state_out
 *              must not be the array held->state points to) */
int32_t rk_privileged(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid, const rk_sla *sla,
                      const int32_t *min_seg, const uint32_t *min_c, const rk_job_state *held, int32_t *floor_seg,
                      uint32_t *floor_c, uint8_t *state_out);

/* Algorithm 1's Schedule with ScheduleJob searching the cluster node by node
 * (Sec. 5.2, Algorithm 1: ScheduleJob's loop over the nodes, whose
 * GetLowestSlopeOverMinJob takes the node as its argument; and the paragraph
 * on shrinking).  State, order of the jobs, steps,
 * slopes, permit cases and commit rule are those of rk_reschedule; here every
 * job that holds something is somewhere, and the job to shrink on a node is
 * the one with the lowest slope among the jobs on THAT node.
 *  - The grid's CPU levels must be CPUs per GPU (cpu_mode 1, otherwise
 *    RK_ERR_UNSUPPORTED): a part of k GPUs at level l holds cpu_levels[l] * k
 *    CPUs of its node.
 *  - prev_off [device] n_jobs + 1 offsets, prev_entries [device]
 *    n_prev_entries records: where the jobs are now.  The parts of a job that
 *    holds something (jobs_state) must add up to its GPU count, lie on nodes in
 *    strictly ascending order and carry c = cpu_levels[cur_c] * g; no node may
 *    hold more than it has (mem_gb is not read: memory is allocated anew).
 *    Parts of a job that holds nothing are ignored.  Both NULL: nobody holds
 *    anything.  A state that is no such placement schedules nothing: all
 *    records and offsets are zero and stats[4] is 1.
 *  - A GPU step of job j walks the nodes in order.  On a node it takes what is
 *    free (a GPU only with its CPUs at the step's level); while it still lacks
 *    GPUs, the job with the lowest slope among the other jobs on this node
 *    that are above their own floor (lower index on ties) is shrunk if that is
 *    permitted (j's slope is higher, or j is below its floor): it steps down
 *    to its next useful amount, giving up GPUs of its part on this node first
 *    and, if its step is larger than that part, the rest from its other parts,
 *    the last one first; j takes again.  Nobody, or not permitted: next node.
 *    A step to a floor with a higher CPU level needs the additional CPUs of
 *    the parts j already has free on their nodes.
 *  - A CPU step raises the level on every node the job is on: per node what is
 *    free first, then the jobs on that node by lowest CPU slope, each giving
 *    one level (on all its nodes).
 *  - A step is committed when all of it was found and (unless j is below its
 *    floor) j gains more than the others lose; otherwise jobs and nodes are
 *    put back and j's search in that resource ends.
 *  - Memory last, in job order: a tier costs every part its share
 *    (tier * k / g, float32) of its node's memory; among the tiers every part
 *    can pay, the highest throughput, the smallest such tier; none: the job is
 *    dropped and has no parts in the result.
 *   assign     [device] n_jobs records (plan and throughput from best_plan / best_thr)
 *   place_off  [device] n_jobs + 1 offsets; entries [device] cap_entries records,
 *              cap_entries >= n_nodes * gpus_per_node; a job's parts in ascending
 *              node order, c = CPUs, mem_gb = its share of the tier
 *   total      [device] one float: sum of thr / ref_thr
 *   stats      [device] five words or NULL: steps committed, jobs that needed
 *              more than a look, shrinks applied, steps taken back, 1 when the
 *              state was no placement
 * GetBestPlan(j, placement) on the result: rk_best_plan_placed (rk_place_plans,
 * given the result as the earlier placement, keeps it part by part and chooses
 * the same plans).
 * Limits: RK_MAX_JOBS_PER_ROUND jobs, n_nodes * gpus_per_node <= 2^20.  One
 * workgroup runs the loop: the rule is sequential. */
int32_t rk_reschedule_nodes(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                            const rk_alloc_grid *grid, const rk_nodes *nodes, const float *best_thr,
                            const uint32_t *best_plan, const float *curve_thr,
                            const rk_job_state *jobs_state, const uint32_t *prev_off_or_null,
                            const rk_place_entry *prev_entries_or_null, uint64_t n_prev_entries,
                            rk_assign *assign, uint32_t *place_off, rk_place_entry *entries,
                            uint64_t cap_entries, float *total, uint32_t *stats_or_null);

/* A whole round of Algorithm 1 on nodes from the job descriptors, in one call
 * (Sec. 5.2, Algorithm 1: Schedule over the jobs, ScheduleJob over the nodes,
 * GetBestPlan for the placement found, memory last): the plan table and the
 * curves of all jobs (as rk_schedule_round computes them, in the context's
 * buffers), rk_reschedule_nodes from what the jobs hold and where they are,
 * then rk_best_plan_placed on the placement that leaves.  Arguments as for
 * these two; assign receives the loop's records (plans of the packed
 * placement), placed the records with the plans of the actual splits, total
 * the sum of thr / ref_thr over placed. */
int32_t rk_schedule_round_nodes(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                                const rk_alloc_grid *grid, const rk_env *env, const rk_nodes *nodes,
                                const rk_job_state *jobs_state, const uint32_t *prev_off_or_null,
                                const rk_place_entry *prev_entries_or_null, uint64_t n_prev_entries,
                                rk_assign *assign, rk_assign *placed, uint32_t *place_off, rk_place_entry *entries,
                                uint64_t cap_entries, float *total, uint32_t *stats_or_null);

/* ---- measurement helper (no part of the method) --------------------------- */

/* Streams a buffer and nothing else, for the benchmark's roofline context:
 * mode 0 reads the first n_floats (rounded down to a multiple of 4) floats of
 * buf [device, 16-byte aligned] with 16-byte streaming loads (out [device]: one
 * float the kernel may add to), a tile of 64 KiB per workgroup; mode 3 is the
 * same read under a second kernel name (a profile then tells a read that
 * follows a fill from one that follows a read); mode 2 reads them with 4,096
 * workgroups that stride through the buffer together; mode 1 fills them with
 * `value`, mode 4 is the same fill under a second kernel name (a fill that
 * follows a fill).  Any other mode, a null or misaligned buf, or fewer than 4
 * floats: RK_ERR_INVALID_ARG. */
int32_t rk_probe_stream(rk_ctx *ctx, float *buf, uint64_t n_floats, int32_t mode, float value, float *out);

#ifdef __cplusplus
}
#endif
#endif /* RUBICK_H */
