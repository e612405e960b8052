/*
 * CPU oracle for the plan-evaluation path of the Rubick scheduler
 * (arxiv 2408.08586).  TEST INFRASTRUCTURE ONLY: a plain, slow, obviously
 * correct implementation used to check the GPU library and to serve as the
 * reported CPU baseline.  It shares no code with the GPU library and nothing
 * in the product path may call it.
 *
 * All pointers are host pointers.  Times are double precision; the memory
 * feasibility test and the greedy slopes are float32 with one rounding per
 * written operation (build with -ffp-contract=off), because those values
 * decide integers that the GPU library must reproduce bit for bit.
 *
 * Job descriptor: coef[j*17 + k] (float32) with k =
 *   0 P_bytes  1 seq  2 hidden  3 elem_bytes  4 t_fwd_sample  5 k_bwd  6 k_sync
 *   7 k_opt  8 k_opt_off  9 k_off  10 k_swap  11 k_const  12 mem_state
 *   13 mem_act  14 mem_act_gc  15 mem_const  16 ref_thr
 * and ints[j*3 + k] (uint32) with k = 0 layers, 1 global batch, 2 micro-batch size.
 * Symbols follow Table 1 of the paper.
 *
 * Parity status of each function is stated at its definition in rk_oracle.cpp.
 */
#ifndef RK_ORACLE_H
#define RK_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORK_NO_PLAN 0xFFFFFFFFu
#define ORK_N_TERMS 24

typedef struct {
    float B_intra, B_inter, B_pcie;   /* bytes/s */
    float gpu_mem_cap;                /* bytes */
    uint32_t gpus_per_node;
} ork_env;

typedef struct {
    uint32_t n_cpu;
    const uint32_t *cpu_levels;       /* ascending, >= 1 */
    uint32_t cpu_mode;                /* 0: CPUs of the job, 1: CPUs per GPU */
    uint32_t n_mem;
    const float *mem_levels_gb;       /* ascending */
    uint32_t mem_mode;                /* 0: GB of the job, 1: GB per GPU */
} ork_grid;

typedef struct {
    uint32_t g_max, tp_max, pp_max;
    uint32_t zero_mask, gc_mask, off_mask;
    uint32_t mu_mask;                 /* bit v: micro-batches of mu * 2^v samples allowed */
} ork_bounds;

typedef struct {                      /* plan table, filled by ork_enumerate */
    const uint32_t *triple_off;       /* [n_jobs+1] */
    const uint32_t *triples;          /* [n_triples][4] = d,t,p,v (v: micro-batch shift) */
    const uint32_t *seg_off;          /* [n_jobs+1] */
    const uint32_t *seg_g;            /* [n_segs] GPU count of the segment */
    const uint32_t *seg_first;        /* [n_segs] first triple (job-local) */
} ork_table;

typedef struct { uint32_t g, c; float mem_gb; uint32_t plan; float thr; } ork_assign;

/* (x^k + y^k)^(1/k), Sec. 4.3 "Modeling overlapping". */
double ork_f_overlap(double k, double x, double y);

/* Enumerate (d,t,p,v) entries per job in canonical order (g, then t, p, v
 * ascending).  Null output buffers: only the counts are produced. Returns 0,
 * or -1 if a capacity is too small (counts still written).  n_threads host
 * threads share the jobs (0 or 1: the calling thread alone). */
int ork_enumerate(uint32_t n_jobs, const uint32_t *ints, const ork_bounds *bounds,
                  uint32_t *triple_off, uint32_t *triples, uint64_t cap_triples,
                  uint32_t *seg_off, uint32_t *seg_g, uint32_t *seg_first, uint64_t cap_segs,
                  uint64_t *n_triples, uint64_t *n_segs, uint32_t n_threads);

/* std::thread::hardware_concurrency() of the machine. */
uint32_t ork_host_cores(void);

/* One candidate; terms[ORK_N_TERMS] receives every intermediate quantity
 * (order documented in rk_oracle.cpp).  Returns the reason bits
 * (0 = feasible; 1 structural, 2 GPU memory, 4 host memory). */
uint32_t ork_eval_one(const float *coef17, const uint32_t *ints3, const ork_bounds *bounds,
                      const ork_env *env, uint32_t d, uint32_t t, uint32_t p, uint32_t v,
                      uint32_t z, uint32_t gc, uint32_t off, uint32_t c, float host_bytes,
                      double *terms);

/* Predicted throughput (and iteration time, optional) of n_samples measured
 * runs of one model type under the seven fittable parameters th (double:
 * k_bwd, k_sync, k_opt, k_opt_off, k_off, k_swap, k_const); the other
 * coefficients come from coef17.  0 for structurally invalid samples. */
int ork_predict_f64(const float *coef17, const uint32_t *ints3, const ork_env *env, const double *th,
                    uint32_t n_samples, const uint32_t *d, const uint32_t *t, const uint32_t *p,
                    const uint32_t *mu_shift_or_null, const uint32_t *option, const uint32_t *cpus, double *thr,
                    double *t_iter_or_null);

/* Every candidate of jobs [job_begin, job_end): thr (0 when infeasible) and
 * optional reason bits, candidate order [job][cpu level][mem tier][plan],
 * plan = triple*16 + (z*4 + gc*2 + off). */
int ork_eval_jobs(uint32_t n_jobs, const float *coef, const uint32_t *ints,
                  const ork_bounds *bounds, const ork_table *table, const ork_grid *grid,
                  const ork_env *env, uint32_t job_begin, uint32_t job_end,
                  double *thr, uint8_t *reason_or_null, uint32_t n_threads);

/* Per segment x cpu level x mem tier: maximum and lowest-index argmax. */
int ork_best_plan_f64(const ork_table *table, const ork_grid *grid, uint32_t job_begin,
                      uint32_t job_end, const double *thr, double *best_thr, uint32_t *best_plan,
                      uint32_t n_threads);
int ork_best_plan_f32(const ork_table *table, const ork_grid *grid, uint32_t job_begin,
                      uint32_t job_end, const float *thr, float *best_thr, uint32_t *best_plan,
                      uint32_t n_threads);

/* Prefix maximum over a job's GPU counts (resource sensitivity curve). */
int ork_curves_f32(const ork_table *table, const ork_grid *grid, uint32_t job_begin,
                   uint32_t job_end, const float *best_thr, const uint32_t *best_plan,
                   float *curve_thr, uint32_t *curve_plan, uint32_t *curve_g);

/* Greedy marginal-gain allocation over all n_jobs jobs of the table.
 * min_gap (optional) receives the smallest relative gap between a winning
 * slope and its runner-up over all decisions taken. */
int ork_greedy_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *table,
                   const ork_grid *grid, uint32_t G, uint32_t C, float host_mem_gb,
                   const float *best_thr, const uint32_t *best_plan,
                   const float *curve_thr, ork_assign *assign, double *total, double *min_gap);

/* Minimum demand of guaranteed jobs: (segment, CPU level, memory tier), -1 if
 * none; outputs indexed by job - job_begin. */
int ork_min_res_f32(const ork_table *table, const ork_grid *grid, uint32_t job_begin, uint32_t job_end,
                    const float *best_thr, const uint32_t *guaranteed, const uint32_t *req_g,
                    const uint32_t *req_c, const uint32_t *req_m, const float *base_thr,
                    int32_t *min_seg, uint32_t *min_c, uint32_t *min_m);

/* Greedy with service-level floors and tenant quotas (guaranteed == NULL: plain greedy). */
int ork_policy_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *table,
                   const ork_grid *grid, uint32_t G, uint32_t C, float host_mem_gb,
                   const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                   const uint32_t *guaranteed, const uint32_t *tenant, const int32_t *min_seg,
                   const uint32_t *min_c, uint32_t n_tenants, const uint32_t *quota_g,
                   const uint32_t *quota_c, ork_assign *assign, double *total, double *min_gap);

/* A round with per-job state: 0 takes part, 1 takes no part, 2 keeps the
 * allocation (cur_seg, cur_c) it holds and is charged for it first. */
int ork_frozen_round_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *table,
                         const ork_grid *grid, uint32_t G, uint32_t C, float host_mem_gb,
                         const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                         const uint8_t *state, const int32_t *cur_seg, const uint32_t *cur_c,
                         ork_assign *assign, double *total, double *min_gap);

/* Algorithm 1's Schedule as a loop from the jobs' present state: privileged
 * jobs (below their floor) first, the others by slope; every job takes what is
 * free and shrinks the jobs with the lowest slope while that is permitted
 * (rules at the definition).  state[j] = 1: takes no part (may be NULL);
 * cur_seg / cur_c: what the job holds (-1: nothing); floor_seg / floor_c: its
 * minimum demand (-1 or NULL: none). */
int ork_reschedule_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *table, const ork_grid *grid,
                       uint32_t G, uint32_t C, float host_mem_gb, const float *best_thr,
                       const uint32_t *best_plan, const float *curve_thr, const uint8_t *state,
                       const int32_t *cur_seg, const uint32_t *cur_c, const int32_t *floor_seg,
                       const uint32_t *floor_c, ork_assign *assign, double *total, uint32_t *n_moves);

/* Node-level placement of an allocation (Sec. 5.2, Algorithm 1, ScheduleJob:
 * a job walks the nodes in order, takes what each node has free and records
 * {node, resources}; it is placed only if its whole amount is found).  Jobs
 * in index order.  On a node a job takes the most GPUs k (up to what it still
 * needs) such that ceil(c*k/g) CPUs and mem*k/g GiB are free there; the part
 * is booked with CPUs floor(c*(done+k)/g) - floor(c*done/g) (done = GPUs
 * placed on earlier nodes) and mem*k/g GiB (float32).
 * place_off [n_jobs+1], entries [sum of g] at most, status [n_jobs]:
 * 0 = nothing to place, 1 = placed, 2 = could not be placed (no entries). */
typedef struct { uint32_t node, g, c; float mem_gb; } ork_place_entry;
int ork_place_f32(uint32_t n_jobs, const ork_assign *assign, uint32_t n_nodes, uint32_t gpus_per_node,
                  uint32_t cpus_per_node, float mem_per_node_gb, uint32_t *place_off,
                  ork_place_entry *entries, uint32_t *status);

/* ork_eval_one for a job whose GPUs are parts[0..n_parts) on the consecutive
 * nodes of its placement: every communication group gets the intra-node
 * bandwidth only if all its ranks are on one node. */
uint32_t ork_eval_one_placed(const float *coef17, const uint32_t *ints3, const ork_bounds *bounds,
                             const ork_env *env, uint32_t d, uint32_t t, uint32_t p, uint32_t v,
                             uint32_t z, uint32_t gc, uint32_t off, uint32_t c, float host_bytes,
                             uint32_t n_parts, const uint32_t *parts, double *terms);

/* Placement of an allocation that feeds the plan: first fit per job with a
 * fall-back to smaller valid GPU counts (not below min_seg[j], NULL or -1 = no
 * floor), then the best plan of the placed count under the bandwidths of the
 * actual node split.  out[n_jobs] = placed amounts, plan, throughput; status
 * 0 nothing to place, 1 placed as asked, 2 placed with fewer GPUs, 3 not placed.
 * prev_off [n_jobs+1] / prev_entries (or NULL): an earlier placement; a job
 * whose amounts are what its earlier parts add up to keeps them, and the
 * kept jobs are booked before the others look for room.
 * Returns -1 for a record that is no allocation on this table and grid (its
 * GPU count, CPU level or memory tier is not one of the job's, or no plan is
 * feasible there). */
int ork_place_plans(uint32_t n_jobs, const float *coef, const uint32_t *ints, const ork_bounds *bounds,
                    const ork_table *table, const ork_grid *grid, const ork_env *env, const float *best_thr,
                    const ork_assign *assign, const int32_t *min_seg, const uint32_t *prev_off,
                    const ork_place_entry *prev_entries, uint32_t n_nodes, uint32_t gpus_per_node,
                    uint32_t cpus_per_node, float mem_per_node_gb, ork_assign *out, uint32_t *place_off,
                    ork_place_entry *entries, uint32_t *status, double *total);

/* Algorithm 1's Schedule with ScheduleJob searching node by node: the job to
 * shrink on a node is the one with the lowest slope among the jobs on that
 * node.  State as ork_reschedule_f32 plus the earlier placement of the jobs
 * that hold something (parts in ascending node order, CPUs = level * GPUs; the
 * grid's CPU levels must be per GPU).  Results: assign [n_jobs], the new
 * placement (place_off [n_jobs+1], entries at most the cluster's GPUs).
 * Returns 0, -1 when the state is no placement on these nodes, -2 when the
 * CPU levels are not per GPU. */
int ork_reschedule_nodes_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *table, const ork_grid *grid,
                             uint32_t n_nodes, uint32_t gpus_per_node, uint32_t cpus_per_node, float mem_per_node_gb,
                             const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                             const uint8_t *state, const int32_t *cur_seg, const uint32_t *cur_c,
                             const int32_t *floor_seg, const uint32_t *floor_c, const uint32_t *prev_off,
                             const ork_place_entry *prev_entries, ork_assign *assign, uint32_t *place_off,
                             ork_place_entry *entries, double *total, uint32_t *n_moves);

/* Floors and states for the Schedule loops from the service levels: running
 * guaranteed jobs keep their minimum demand as floor and charge their tenant's
 * quota first; queued guaranteed jobs get theirs in job order while the quota
 * lasts, the others wait (state 1). */
int ork_privileged(uint32_t n_jobs, const ork_table *table, const ork_grid *grid, const uint32_t *guaranteed,
                   const uint32_t *tenant, const int32_t *min_seg, const uint32_t *min_c, uint32_t n_tenants,
                   const uint32_t *quota_g, const uint32_t *quota_c, const uint8_t *state_in, const int32_t *cur_seg,
                   const uint32_t *cur_c, int32_t *floor_seg, uint32_t *floor_c, uint8_t *state_out);

/* The slope table of the curves: per row and GPU count the next GPU step (slope,
 * target count or -1) and the next CPU step (slope, target level or n_cpu), and
 * per row the first step from nothing.  Segment layout of jobs [jb, je). */
int ork_curve_slopes(const float *ref_thr, const ork_table *table, const ork_grid *grid, uint32_t jb, uint32_t je,
                     const float *best_thr, const float *curve_thr, float *gpu_slope, int32_t *gpu_next,
                     float *from0_slope, int32_t *from0_next, float *cpu_slope, uint32_t *cpu_next);

#ifdef __cplusplus
}
#endif
#endif
