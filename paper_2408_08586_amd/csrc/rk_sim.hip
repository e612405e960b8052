// Discrete-time simulation of a job trace through the greedy allocation with
// the reconfiguration-penalty gate (paper Sec. 5.2 "Incorporating
// reconfiguration penalty", Sec. 7.4).  The curves are computed once by the
// caller; a tick is
//   k_sim_begin   (one workgroup) advances the tick counter; per-job state of
//                 the tick: inactive, frozen or free to move; floors of the
//                 frozen jobs; capacity left
//   the allocation kernels from these floors
//   k_sim_commit  (thread per job) reconfiguration count and cost, progress,
//                 completion; remembers what every job holds
// The tick counter lives on the device, so every tick is the same sequence of
// launches with the same arguments: the first tick runs eagerly (it also sizes
// the scratch memory), the sequence is then captured once as a HIP graph on a
// stream of the simulation's own and replayed for the remaining ticks.
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int SIM_THREADS = 1024;
constexpr int COMMIT_THREADS = 256;

struct SimState {               // per job, between the ticks
    uint32_t *g, *c, *plan;     // what the job holds (g = 0: nothing)
    int32_t *seg;               // ... as segment index
    uint32_t *lvl;              // ... and CPU level
    double *owed;               // checkpoint-resume seconds still to pay
    uint8_t *done;
};

struct SimArgs {
    TableDev tb;
    GridDev grid;
    rk_cluster cl;
    uint32_t n_jobs;
    const double *arrival, *work, *delta;
    double dt, gate;
    SimState S;
    FloorsDev F;
    const rk_assign *assign;
    uint32_t *tick;             // device counter, advanced by k_sim_begin
    float *tick_total;          // the allocation's total of the current tick
    rk_sim_result out;
    double *held;               // result arrays or scratch when the caller passes none
    double *progress, *finish;
    uint32_t *n_reconf;
    // the search over nodes only: where the jobs are (left by the last tick) and where this tick puts them
    uint32_t *at_off, *now_off;
    rk_place_entry *at_ent, *now_ent;
};

__global__ __launch_bounds__(SIM_THREADS) void k_sim_init(SimArgs A) {
    const uint32_t j = blockIdx.x * SIM_THREADS + threadIdx.x;
    if (j >= A.n_jobs) return;
    A.S.g[j] = 0; A.S.c[j] = 0; A.S.plan[j] = RK_NO_PLAN; A.S.seg[j] = -1; A.S.lvl[j] = 0;
    A.S.owed[j] = 0.0; A.S.done[j] = 0;
    A.held[j] = 0.0; A.progress[j] = 0.0; A.finish[j] = -1.0; A.n_reconf[j] = 0;
    if (j == 0) *A.tick = 0xFFFFFFFFu;                    // the first k_sim_begin makes it 0
    if (A.at_off) { A.at_off[j] = 0u; if (j == 0) A.at_off[A.n_jobs] = 0u; }   // nobody is anywhere yet
}

// the placement this tick made is where the jobs are when the next tick begins
__global__ void k_sim_keep_placement(SimArgs A) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= A.n_jobs) A.at_off[i] = A.now_off[i];
    if (i < A.now_off[A.n_jobs]) A.at_ent[i] = A.now_ent[i];
}

__global__ __launch_bounds__(SIM_THREADS) void k_sim_begin(SimArgs A) {
    __shared__ unsigned long long red_g[SIM_THREADS / 64], red_c[SIM_THREADS / 64];
    __shared__ uint32_t red_f[SIM_THREADS / 64];
    __shared__ uint32_t tick_now;
    const uint32_t tid = threadIdx.x;
    if (tid == 0) { tick_now = *A.tick + 1u; *A.tick = tick_now; }
    __syncthreads();
    const uint32_t tick = tick_now;
    const double t = (double)tick * A.dt;
    unsigned long long held_g = 0, held_c = 0;
    uint32_t n_frozen = 0;
    for (uint32_t j = tid; j < A.n_jobs; j += SIM_THREADS) {
        const bool active = A.arrival[j] <= t && !A.S.done[j];
        const uint32_t g = A.S.g[j];
        uint8_t state = RK_JOB_OUT;
        int32_t gi = -1;
        uint32_t ci = 0;
        if (active) {
            state = RK_JOB_NORMAL;
            if (g > 0) {
                const double T = A.held[j];
                const bool may_move = T - ((double)A.n_reconf[j] + 1.0) * A.delta[j] > A.gate * T;
                if (!may_move) {
                    state = RK_JOB_FROZEN;
                    gi = A.S.seg[j];
                    ci = A.S.lvl[j];
                    held_g += g;
                    held_c += A.grid.cpu_mode ? (unsigned long long)A.grid.cpu_levels[ci] * g
                                              : (unsigned long long)A.grid.cpu_levels[ci];
                    ++n_frozen;
                }
            }
        }
        A.F.state[j] = state;
        A.F.gi[j] = gi;
        A.F.ci[j] = ci;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        held_g += __shfl_xor(held_g, off, 64);
        held_c += __shfl_xor(held_c, off, 64);
        n_frozen += __shfl_xor(n_frozen, off, 64);
    }
    if ((tid & 63u) == 0) { red_g[tid >> 6] = held_g; red_c[tid >> 6] = held_c; red_f[tid >> 6] = n_frozen; }
    __syncthreads();
    if (tid == 0) {
        unsigned long long hg = 0, hc = 0;
        uint32_t nf = 0;
        for (int w = 0; w < SIM_THREADS / 64; ++w) { hg += red_g[w]; hc += red_c[w]; nf += red_f[w]; }
        A.F.cap0[0] = hg < A.cl.G ? A.cl.G - hg : 0ull;       // frozen jobs are charged first
        A.F.cap0[1] = hc < A.cl.C ? A.cl.C - hc : 0ull;
        if (A.out.frozen) A.out.frozen[tick] = nf;
        if (A.out.gpus_in_use) A.out.gpus_in_use[tick] = 0u;  // summed by k_sim_commit
    }
}

__global__ __launch_bounds__(COMMIT_THREADS) void k_sim_commit(SimArgs A) {
    const uint32_t j = blockIdx.x * COMMIT_THREADS + threadIdx.x;
    const uint32_t tick = *A.tick;
    if (j == 0 && A.out.totals) A.out.totals[tick] = *A.tick_total;
    uint32_t g_used = 0;
    if (j < A.n_jobs && A.F.state[j] != RK_JOB_OUT) {
        const double t = (double)tick * A.dt;
        const rk_assign a = A.assign[j];
        uint32_t g = a.g;
        g_used = g;
        const uint32_t g_prev = A.S.g[j];
        if (g_prev > 0 && g > 0 && (g != g_prev || a.c != A.S.c[j] || a.plan != A.S.plan[j])) {
            A.n_reconf[j] += 1;
            A.S.owed[j] = A.S.owed[j] + A.delta[j];
        }
        if (g > 0) {
            A.held[j] = A.held[j] + A.dt;
            const double owed = A.S.owed[j];
            const double paid = owed < A.dt ? owed : A.dt;
            A.S.owed[j] = owed - paid;
            const double train = A.dt - paid;
            const double thr = (double)a.thr;
            const double gain = thr * train;
            const double progress = A.progress[j], work = A.work[j];
            if (progress + gain >= work) {
                A.finish[j] = t + paid + (work - progress) / thr;
                A.progress[j] = work;
                A.S.done[j] = 1;
                g = 0;
            } else {
                A.progress[j] = progress + gain;
            }
        }
        if (g > 0) {
            // segment index of g (the job's counts ascend) and the CPU level that costs a.c
            const uint32_t s0 = A.tb.seg_off[j], ns = A.tb.seg_off[j + 1] - s0;
            uint32_t lo = 0, hi = ns;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (A.tb.seg_g[s0 + mid] < g) lo = mid + 1; else hi = mid;
            }
            uint32_t lvl = 0;
            for (uint32_t i = 0; i < A.grid.n_cpu; ++i)
                if (cpus_of(A.grid, i, g) == a.c) { lvl = i; break; }
            A.S.g[j] = g; A.S.c[j] = a.c; A.S.plan[j] = a.plan; A.S.seg[j] = (int32_t)lo; A.S.lvl[j] = lvl;
        } else {
            A.S.g[j] = 0; A.S.c[j] = 0; A.S.plan[j] = RK_NO_PLAN; A.S.seg[j] = -1; A.S.lvl[j] = 0;
        }
    }
    if (A.out.gpus_in_use) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) g_used += __shfl_xor(g_used, off, 64);
        if ((threadIdx.x & 63u) == 0 && g_used) atomicAdd(&A.out.gpus_in_use[tick], g_used);
    }
}

}  // namespace

extern "C" int32_t rk_simulate(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                               const rk_alloc_grid *grid, const rk_cluster *cluster, const float *best_thr,
                               const uint32_t *best_plan, const float *curve_thr, const rk_trace *trace,
                               const rk_sim_options *options, const rk_sim_result *result) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!table) return rk_fail(ctx, RK_ERR_INVALID_ARG, "table is null");
    if ((rc = rk_check_table(ctx, table, 0, table->n_jobs))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (!cluster || !trace || !options || !result) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    const uint32_t J = table->n_jobs;
    if (J == 0 || options->n_ticks == 0) return RK_OK;
    if (!ref_thr || !best_thr || !best_plan || !curve_thr || !trace->arrival || !trace->work || !trace->delta)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (!(options->dt > 0.0)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "dt must be positive");
    if (options->gate != options->gate) return rk_fail(ctx, RK_ERR_INVALID_ARG, "gate is NaN");
    if (options->policy > 2u)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "policy must be 0 (greedy round), 1 (Schedule loop) or 2 (Schedule loop over nodes)");
    const rk_nodes *nodes = options->policy == 2u ? options->nodes : nullptr;
    uint64_t cap_parts = 0;
    if (options->policy == 2u) {
        if (!nodes) return rk_fail(ctx, RK_ERR_INVALID_ARG, "policy 2 needs the nodes");
        if (nodes->n_nodes == 0 || nodes->n_nodes > RK_MAX_NODES || nodes->gpus_per_node == 0 ||
            nodes->gpus_per_node > 65535u || nodes->cpus_per_node > 65535u || !(nodes->mem_per_node_gb >= 0.f))
            return rk_fail(ctx, RK_ERR_INVALID_ARG, "nodes: 1..%u nodes of 1..65535 GPUs, at most 65535 CPUs, memory >= 0", RK_MAX_NODES);
        if (grid->cpu_mode != 1u)
            return rk_fail(ctx, RK_ERR_UNSUPPORTED, "the search over nodes needs CPU levels per GPU (cpu_mode 1)");
        cap_parts = (uint64_t)nodes->n_nodes * nodes->gpus_per_node;
        if (cap_parts > (1u << 20)) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 2^20 GPUs on the nodes");
    }
    if (!(cluster->host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    if (J > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u jobs, the allocation kernels take up to %u", J, RK_MAX_JOBS_PER_ROUND);
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    RK_HIP(ctx, hipSetDevice(ctx->device));

    // per-job state in one scratch block, carved by alignment
    const size_t n8 = ((size_t)J * 8 + 255) & ~(size_t)255, n4 = ((size_t)J * 4 + 255) & ~(size_t)255;
    const size_t n1 = ((size_t)J + 255) & ~(size_t)255;
    char *blk;
    if ((rc = rk_scratch(ctx, SL_SIM_STATE, 5 * n8 + 8 * n4 + 2 * n1 + 256, (void **)&blk))) return rc;
    rk_assign *assign;
    if ((rc = rk_scratch(ctx, SL_SIM_ASSIGN, (size_t)J * sizeof(rk_assign) + 16, (void **)&assign))) return rc;
    auto take = [&](size_t bytes) { char *p = blk; blk += bytes; return p; };
    SimArgs A;
    A.tb = table_dev(table); A.grid = grid_dev(grid); A.cl = *cluster; A.n_jobs = J;
    A.arrival = trace->arrival; A.work = trace->work; A.delta = trace->delta;
    A.dt = options->dt; A.gate = options->gate;
    A.S.owed = (double *)take(n8);
    double *s_held = (double *)take(n8), *s_prog = (double *)take(n8), *s_fin = (double *)take(n8);
    A.F.cap0 = (unsigned long long *)take(256);
    A.S.g = (uint32_t *)take(n4); A.S.c = (uint32_t *)take(n4); A.S.plan = (uint32_t *)take(n4);
    A.S.seg = (int32_t *)take(n4); A.S.lvl = (uint32_t *)take(n4);
    A.F.gi = (int32_t *)take(n4); A.F.ci = (uint32_t *)take(n4);
    uint32_t *s_nrec = (uint32_t *)take(n4);
    A.S.done = (uint8_t *)take(n1); A.F.state = (uint8_t *)take(n1);
    A.out = *result;
    A.held = result->held ? result->held : s_held;
    A.progress = result->progress ? result->progress : s_prog;
    A.finish = result->finish ? result->finish : s_fin;
    A.n_reconf = result->n_reconf ? result->n_reconf : s_nrec;
    A.assign = assign;

    A.at_off = A.now_off = nullptr; A.at_ent = A.now_ent = nullptr;
    if (nodes) {                                               // two placements: where the jobs are, where they go
        char *pl;
        const size_t off_bytes = (((size_t)J + 1) * 4 + 255) & ~(size_t)255;
        const size_t ent_bytes = ((size_t)cap_parts * sizeof(rk_place_entry) + 255) & ~(size_t)255;
        if ((rc = rk_scratch(ctx, SL_SIM_PLACES, 2 * (off_bytes + ent_bytes), (void **)&pl))) return rc;
        A.at_off = (uint32_t *)pl; A.now_off = (uint32_t *)(pl + off_bytes);
        A.at_ent = (rk_place_entry *)(pl + 2 * off_bytes); A.now_ent = (rk_place_entry *)(pl + 2 * off_bytes + ent_bytes);
    }
    A.tick = reinterpret_cast<uint32_t *>(A.F.cap0 + 4);       // inside the 256-byte capacity block
    A.tick_total = reinterpret_cast<float *>(A.F.cap0 + 5);

    // the simulation's own stream, ordered after what the context's stream holds
    if (!ctx->sim_stream) {
        RK_HIP(ctx, hipStreamCreateWithFlags(&ctx->sim_stream, hipStreamNonBlocking));
        RK_HIP(ctx, hipEventCreateWithFlags(&ctx->sim_ev[0], hipEventDisableTiming));
        RK_HIP(ctx, hipEventCreateWithFlags(&ctx->sim_ev[1], hipEventDisableTiming));
    }
    hipStream_t user = ctx->stream, s = ctx->sim_stream;
    RK_HIP(ctx, hipEventRecord(ctx->sim_ev[0], user));
    RK_HIP(ctx, hipStreamWaitEvent(s, ctx->sim_ev[0], 0));

    auto tick_body = [&]() -> int32_t {
        k_sim_begin<<<1, SIM_THREADS, 0, s>>>(A);
        RK_CHECK_LAUNCH(ctx, "k_sim_begin");
        ctx->stream = s;                                       // the allocation enqueues on the context's stream
        int32_t r;
        if (options->policy == 2u) {                           // ... searching node by node, from where the jobs are
            const rk_job_state held = {A.F.state, A.S.seg, A.S.lvl, nullptr, nullptr};
            r = rk_launch_reschedule_nodes(ctx, ref_thr, table, grid, nodes, best_thr, best_plan, curve_thr, &held, A.at_off,
                                           A.at_ent, cap_parts, assign, A.now_off, A.now_ent, A.tick_total, nullptr);
        } else if (options->policy == 1u) {                    // Algorithm 1's loop from what the jobs hold
            const rk_job_state held = {A.F.state, A.S.seg, A.S.lvl, nullptr, nullptr};
            r = rk_launch_reschedule(ctx, ref_thr, table, grid, cluster, best_thr, best_plan, curve_thr, &held, assign,
                                     A.tick_total, nullptr);
        } else {
            r = rk_launch_allocate(ctx, ref_thr, A.tb, grid, 1, nullptr, nullptr, cluster, 0, J, J,
                                   table->max_segs_per_job, best_thr, best_plan, curve_thr, nullptr, &A.F,
                                   nullptr, assign, A.tick_total);
        }
        ctx->stream = user;
        if (r) return r;
        k_sim_commit<<<(J + COMMIT_THREADS - 1) / COMMIT_THREADS, COMMIT_THREADS, 0, s>>>(A);
        RK_CHECK_LAUNCH(ctx, "k_sim_commit");
        if (nodes) {
            const uint64_t most = cap_parts > J + 1 ? cap_parts : J + 1;
            k_sim_keep_placement<<<(uint32_t)((most + 255) / 256), 256, 0, s>>>(A);
            RK_CHECK_LAUNCH(ctx, "k_sim_keep_placement");
        }
        return RK_OK;
    };

    k_sim_init<<<(J + SIM_THREADS - 1) / SIM_THREADS, SIM_THREADS, 0, s>>>(A);
    RK_CHECK_LAUNCH(ctx, "k_sim_init");
    if ((rc = tick_body())) return rc;                         // tick 0, eagerly
    if (options->n_ticks > 1) {
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
        RK_HIP(ctx, hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed));
        rc = tick_body();
        const hipError_t e_end = hipStreamEndCapture(s, &graph);
        if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
        if (e_end != hipSuccess) return rk_fail(ctx, RK_ERR_DEVICE, "hipStreamEndCapture: %s", hipGetErrorString(e_end));
        hipError_t e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        for (uint32_t k = 1; e == hipSuccess && k < options->n_ticks; ++k) e = hipGraphLaunch(exec, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);      // the graph must outlive its launches
        if (exec) (void)hipGraphExecDestroy(exec);
        (void)hipGraphDestroy(graph);
        if (e != hipSuccess) return rk_fail(ctx, RK_ERR_DEVICE, "simulation graph: %s", hipGetErrorString(e));
    }
    RK_HIP(ctx, hipEventRecord(ctx->sim_ev[1], s));
    RK_HIP(ctx, hipStreamWaitEvent(user, ctx->sim_ev[1], 0));
    return RK_OK;
}
