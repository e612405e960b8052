// Algorithm 1's Schedule with ScheduleJob searching the cluster node by node (paper Sec. 5.2, Algorithm 1 and the
// paragraph on shrinking): on each node the job first takes what is free, then the job with the lowest slope among
// the jobs ON THAT NODE that are above their own minimum is shrunk while that is permitted, then the next node.
// State, order of the jobs, steps, slopes, permit cases and commit rule are those of the loop over the cluster's
// totals (k_reschedule); this kernel adds where things are.
//
// Nodes: per node what is free (GPUs, CPUs) and the list of its residents (job, GPUs of that job here); a node of n
// GPUs has at most n residents, so the lists are a fixed table.  The CPU levels are CPUs per GPU: a part of k GPUs at
// level l holds cpu_levels[l] * k CPUs of its node.  A job's parts are not stored per job; they are found by looking
// the job up on every node (all threads, a node or a few per thread) in the few places that need them.
//
// k_nd_init clears the nodes and k_nd_prepare loads every job on its own, over the whole chip: what it holds, its parts
// booked on the nodes, its cached slopes and next steps.  The loop itself is one workgroup: the rule is sequential.
// Parallel are: the refresh of the jobs a committed step changed (a wavefront per job), the walk over the nodes as
// long as nobody has to be asked (a node per thread: what each offers, a prefix sum that cuts the offers at what the
// job lacks, and the first node where the job still lacks GPUs and somebody may be shrunk), the parts a shrunk job
// gives up elsewhere (a suffix sum over the nodes), the look-ahead that passes over jobs with nothing to do, and
// everything about memory and the records.
// Before a step touches anything the node tables are copied; a step that is not committed copies them back.
#include "rk_internal.h"
#include "rk_model.h"
#include "rk_loop.h"

namespace {

constexpr int ND_THREADS = 1024;
constexpr int ND_WAVES = ND_THREADS / 64;
constexpr uint32_t ND_NONE = 0xFFFFFFFFu;
constexpr uint32_t ND_PER = (RK_MAX_NODES + ND_THREADS - 1) / ND_THREADS;   // nodes per thread, at most
constexpr uint32_t ND_MAX_GPUS = 1u << 20;                                   // nodes x GPUs per node

struct NdCurves {
    const float *ref_thr;
    TableDev tb;
    GridDev grid;
    const float *best_thr;
    const uint32_t *best_plan;
    const float *curve_thr;
};
struct NdHold { int32_t *gi; uint32_t *ci; };

struct NdBody {
    NdHold st;                       // what every job holds: index of its GPU count (-1 nothing), CPU level
    unsigned long long G;            // GPUs of the cluster
    uint32_t n_jobs, n_nodes, gpn, cpn;
    float mem_gb;                    // host memory of a node
    const uint8_t *state;            // may be null
    const int32_t *cur_seg;
    const uint32_t *cur_c;
    const int32_t *floor_seg;        // may be null
    const uint32_t *floor_c;         // may be null
    const uint32_t *prev_off;        // may be null (then nobody may hold anything)
    const rk_place_entry *prev_entries;
    uint64_t n_prev;                 // records in prev_entries
    // nodes: one block of words [free_g | free_c | cnt | res_job | res_k], and its copy
    uint32_t *free_g, *free_c, *cnt, *res_job, *res_k;
    uint32_t *keep_nodes;
    uint32_t nodes_words;
    // per job: cached slopes (see rk_loop.h), the order, what a step touched
    float *ds_g, *ds_c, *ug, *uc, *sg, *sc, *keep_ds;
    float *gain_g, *gain_c;          // ... and of a job's next GPU / CPU step: its gain,
    int32_t *tgt_g;                  // the GPU step's target amount,
    uint32_t *lvl_g, *lvl_c, *any;   // the CPU level each step ends on, bit 0 / 1: there is a GPU / CPU step
    uint32_t *udg, *touched, *stamp, *first, *keep_ci, *np, *tmp_off, *tier;
    int32_t *keep_gi;
    unsigned long long *udc_g, *udc_c;
    uint32_t *plist;                 // parts of one job: (node, GPUs) pairs, ascending node
    uint32_t *tmp_parts;             // parts of all jobs, grouped by job, in no order
    rk_assign *assign;
    uint32_t *place_off;
    rk_place_entry *entries;
    float *total;
    uint32_t *stats;                 // may be null
    uint32_t *flags;                 // one word: non-zero when some job's parts are no placement
};
// What the device code sees: the body by value (registers), the table, grid and curves where the kernel arguments
// hold them (a copy of the grid's level arrays would live in scratch memory).
struct NdArgs : NdBody {
    const NdCurves &X;
    __device__ NdArgs(const NdBody &b, const NdCurves &x) : NdBody(b), X(x) {}
};
struct NdKernArgs { NdCurves X; NdBody b; };       // the kernels' argument

__device__ __forceinline__ uint32_t nd_cpl(const NdArgs &A, uint32_t lvl) { return A.X.grid.cpu_levels[lvl]; }

// where job `job` is in node n's list, -1: not there
__device__ __forceinline__ int nd_find(const NdArgs &A, uint32_t n, uint32_t job) {
    const uint32_t c = A.cnt[n];
    const uint32_t *rj = A.res_job + (size_t)n * A.gpn;
    for (uint32_t i = 0; i < c; ++i)
        if (rj[i] == job) return (int)i;
    return -1;
}
__device__ __forceinline__ uint32_t nd_part(const NdArgs &A, uint32_t n, uint32_t job) {
    const int i = nd_find(A, n, job);
    return i < 0 ? 0u : A.res_k[(size_t)n * A.gpn + (uint32_t)i];
}
// job takes k free GPUs of node n, each with per_gpu CPUs (the caller has checked that they are free)
__device__ __forceinline__ void nd_add(const NdArgs &A, uint32_t n, uint32_t job, uint32_t k, uint32_t per_gpu) {
    A.free_g[n] -= k; A.free_c[n] -= k * per_gpu;
    const size_t base = (size_t)n * A.gpn;
    const int i = nd_find(A, n, job);
    if (i >= 0) { A.res_k[base + (uint32_t)i] += k; return; }
    const uint32_t c = A.cnt[n];
    if (c < A.gpn) { A.res_job[base + c] = job; A.res_k[base + c] = k; A.cnt[n] = c + 1u; }   // (always: a resident holds a GPU)
}
// job gives k GPUs of node n back, each with per_gpu CPUs
__device__ __forceinline__ void nd_drop(const NdArgs &A, uint32_t n, uint32_t job, uint32_t k, uint32_t per_gpu) {
    const int i = nd_find(A, n, job);
    if (i < 0) return;
    const size_t base = (size_t)n * A.gpn;
    A.free_g[n] += k; A.free_c[n] += k * per_gpu;
    const uint32_t left = A.res_k[base + (uint32_t)i] - k;
    if (left) { A.res_k[base + (uint32_t)i] = left; return; }
    const uint32_t c = A.cnt[n] - 1u;
    A.res_job[base + (uint32_t)i] = A.res_job[base + c]; A.res_k[base + (uint32_t)i] = A.res_k[base + c];
    A.cnt[n] = c;
}
// GetLowestSlopeOverMinJob(n, resType): lowest cached slope among the residents of n other than j (infinite: gives
// nothing); lower job index among equal slopes; who = ND_NONE when nobody can give
__device__ __forceinline__ float nd_lowest_on(const NdArgs &A, uint32_t n, uint32_t j, const float *ds, uint32_t &who) {
    const float INF = __int_as_float(0x7F800000);
    float best = INF;
    who = ND_NONE;
    const uint32_t c = A.cnt[n];
    const uint32_t *rj = A.res_job + (size_t)n * A.gpn;
    for (uint32_t i = 0; i < c; ++i) {
        const uint32_t v = rj[i];
        if (v == j) continue;
        const float s = ds[v];
        if (s < best || (s == best && s < INF && v < who)) { best = s; who = v; }
    }
    return best;
}

// The same for a whole wavefront, a resident per lane (64 at a time): the residents' slopes are asked for together.
__device__ __forceinline__ float nd_lowest_on_wave(const NdArgs &A, uint32_t n, uint32_t j, const float *ds, uint32_t &who,
                                                   uint32_t lane) {
    const float INF = __int_as_float(0x7F800000);
    const uint32_t c = A.cnt[n];
    const uint32_t *rj = A.res_job + (size_t)n * A.gpn;
    unsigned long long low = ~0ull;                          // (slope as a word that orders like it, job)
    for (uint32_t b = 0; b < c; b += 64u) {
        const uint32_t i = b + lane;
        const uint32_t v = i < c ? rj[i] : j;
        const float s = v != j ? ds[v] : INF;
        const unsigned long long key = ((unsigned long long)rs_ordered(s) << 32) | v;
        if (s < INF && key < low) low = key;
    }
    low = wave_min_u64_rows(low);
    who = low == ~0ull ? ND_NONE : (uint32_t)low;
    return low == ~0ull ? INF : rs_unordered((uint32_t)(low >> 32));
}

// All cached values of job v from its present state: what it gives (rs_refresh_give) and its next steps in full, so
// that ScheduleJob need not search them again.  `lanes` threads share the search (1, or the 64 of a wavefront).
__device__ __forceinline__ void nd_refresh(const NdArgs &A, uint32_t v, uint32_t lane, uint32_t lanes) {
    const RsGive a = rs_down_gpu(A, v), b = rs_down_cpu(A, v);
    const RsStep ug = rs_up_gpu(A, v, lane, lanes), uc = rs_up_cpu(A, v, lane, lanes);
    if (lane != 0) return;
    A.ds_g[v] = a.any ? a.slope : __int_as_float(0x7F800000);
    A.ds_c[v] = b.any ? b.slope : __int_as_float(0x7F800000);
    A.ug[v] = ug.any ? ug.slope : 0.f; A.udg[v] = (uint32_t)ug.dg; A.udc_g[v] = ug.dc;   // (a step that exists has its slope here)
    A.uc[v] = uc.any ? uc.slope : 0.f; A.udc_c[v] = uc.dc;
    A.gain_g[v] = ug.gain; A.gain_c[v] = uc.gain; A.tgt_g[v] = ug.tgt; A.lvl_g[v] = ug.lvl; A.lvl_c[v] = uc.lvl;
    A.any[v] = (ug.any ? 1u : 0u) | (uc.any ? 2u : 0u);
}
// nd_refresh for a whole wavefront: a job of at most 64 amounts that is not below its floor has its rows loaded at
// once, an amount per lane, and every step comes from the registers (rs_rows)
__device__ __forceinline__ void nd_refresh_wave(const NdArgs &A, uint32_t v, uint32_t lane) {
    const int32_t gi = A.st.gi[v];
    const uint32_t ci = A.st.ci[v];
    const int32_t fl = rs_fl_s(A, v);
    const uint32_t so = A.X.tb.seg_off[v], ns = A.X.tb.seg_off[v + 1] - so;
    if (ns > 64u || (fl >= 0 && gi < fl)) { nd_refresh(A, v, lane, 64); return; }
    const RsRows R = rs_rows(A, v, so, ns, gi, ci, lane);
    const RsGive a = rs_down_gpu_rows(A, R, R.curve, gi, ci, lane);
    const RsGive b = rs_down_cpu_rows(A, R, gi, ci, rs_lane_f(R.best, gi), rs_lane_f(R.best_lo, gi));
    const RsStep ug = rs_up_gpu_rows(A, R, gi, ci, lane), uc = rs_up_cpu_rows(A, R, gi, ci, lane);
    if (lane != 0) return;
    A.ds_g[v] = a.any ? a.slope : __int_as_float(0x7F800000);
    A.ds_c[v] = b.any ? b.slope : __int_as_float(0x7F800000);
    A.ug[v] = ug.any ? ug.slope : 0.f; A.udg[v] = (uint32_t)ug.dg; A.udc_g[v] = ug.dc;
    A.uc[v] = uc.any ? uc.slope : 0.f; A.udc_c[v] = uc.dc;
    A.gain_g[v] = ug.gain; A.gain_c[v] = uc.gain; A.tgt_g[v] = ug.tgt; A.lvl_g[v] = ug.lvl; A.lvl_c[v] = uc.lvl;
    A.any[v] = (ug.any ? 1u : 0u) | (uc.any ? 2u : 0u);
}
// the cached next step of job j: res 0 GPUs, 1 CPU level
__device__ __forceinline__ RsStep nd_cached_step(const NdArgs &A, uint32_t j, uint32_t res) {
    RsStep st;
    if (res == 0) {
        st.any = A.any[j] & 1u; st.tgt = A.tgt_g[j]; st.lvl = A.lvl_g[j]; st.slope = A.ug[j]; st.gain = A.gain_g[j];
        st.dg = A.udg[j]; st.dc = A.udc_g[j];
    } else {
        st.any = (A.any[j] >> 1) & 1u; st.tgt = A.st.gi[j]; st.lvl = A.lvl_c[j]; st.slope = A.uc[j]; st.gain = A.gain_c[j];
        st.dg = 0ull; st.dc = A.udc_c[j];
    }
    return st;
}

// The nodes, all free and empty.
__global__ void k_nd_init(NdKernArgs K) {
    const NdArgs A(K.b, K.X);
    const uint32_t n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n < A.n_nodes) { A.free_g[n] = A.gpn; A.free_c[n] = A.cpn; A.cnt[n] = 0u; }
    if (n == 0) A.flags[0] = 0u;
}

// Every job on its own, any number of workgroups: what it holds, whether it comes first, its parts booked on the
// nodes (atomics; a node that ends up holding more than it has is seen by the main kernel), its cached slopes.
__global__ void k_nd_prepare(NdKernArgs K) {
    const NdArgs A(K.b, K.X);
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= A.n_jobs) return;
    const uint32_t N = A.n_nodes;
    int32_t gi = -1;
    uint32_t ci = 0;
    if (rs_holds(A, j) && A.cur_seg[j] >= 0 && (uint32_t)A.cur_seg[j] < rs_ns(A, j) && A.cur_c[j] < A.X.grid.n_cpu) {
        gi = A.cur_seg[j]; ci = A.cur_c[j];
    }
    A.st.gi[j] = gi; A.st.ci[j] = ci;
    A.stamp[j] = 0u;
    const int32_t fl = rs_fl_s(A, j);
    A.first[j] = (rs_part(A, j) && fl >= 0 && gi < fl) ? 1u : 0u;
    if (gi >= 0) {
        bool good = A.prev_off != nullptr && A.prev_entries != nullptr;
        if (good) {
            const uint32_t per_gpu = nd_cpl(A, ci);
            const uint32_t a = A.prev_off[j], b = A.prev_off[j + 1];
            if (a > b || b > A.n_prev) good = false;
            unsigned long long sum = 0;
            long long last = -1;
            for (uint32_t i = a; i < b && good; ++i) {
                const rk_place_entry e = A.prev_entries[i];
                if (e.node >= N || (long long)e.node <= last || e.g == 0u || e.g > A.gpn || e.c > A.cpn ||
                    (unsigned long long)e.c != (unsigned long long)per_gpu * e.g) { good = false; break; }
                last = e.node; sum += e.g;
            }
            if (good && sum != rs_g(A, j, gi)) good = false;
            for (uint32_t i = a; i < b && good; ++i) {
                const rk_place_entry e = A.prev_entries[i];
                const uint32_t slot = atomicAdd(&A.cnt[e.node], 1u);
                if (slot < A.gpn) {
                    A.res_job[(size_t)e.node * A.gpn + slot] = j; A.res_k[(size_t)e.node * A.gpn + slot] = e.g;
                }
                // (wraps below zero when the node holds more than it has; the main kernel sees that)
                atomicSub(&A.free_g[e.node], e.g);
                atomicSub(&A.free_c[e.node], e.c);
            }
        }
        if (!good) atomicOr(&A.flags[0], 1u);
    }
    nd_refresh(A, j, 0, 1);
}

__global__ __launch_bounds__(ND_THREADS) void k_reschedule_nodes(NdKernArgs K) {
    // what every job loses per GPU / CPU it gives, [2][n_jobs]: read at every look at a node's residents and at every
    // look for the next job, so the kernel keeps them in LDS (k_nd_prepare left them in memory)
    extern __shared__ float sh_ds[];
    NdArgs A(K.b, K.X);
    for (uint32_t j = threadIdx.x; j < A.n_jobs; j += ND_THREADS) {
        sh_ds[j] = K.b.ds_g[j];
        sh_ds[A.n_jobs + j] = K.b.ds_c[j];
    }
    A.ds_g = sh_ds;
    A.ds_c = sh_ds + A.n_jobs;
    __shared__ RsStep sh_step;
    __shared__ float sh_lost;
    __shared__ unsigned long long sh_pick_key[ND_WAVES + 1];
    __shared__ uint32_t sh_pick_j[ND_WAVES + 1];
    __shared__ uint32_t sh_widx[ND_WAVES], sh_scan[ND_WAVES];
    __shared__ uint32_t sh_lack, sh_ok, sh_go, sh_touched, sh_epoch, sh_moves, sh_full, sh_shrinks, sh_undone;
    __shared__ uint32_t sh_vnode, sh_next, sh_v, sh_rest, sh_per_v, sh_flag, sh_np, sh_bad, sh_fit, sh_done, sh_ask;
    __shared__ unsigned long long sh_take[RK_MAX_CPU_LEVELS], sh_free_c;
    __shared__ RsMin sh_min[2];
    __shared__ unsigned long long sh_two_k[2 * (ND_WAVES + 1)];
    __shared__ uint32_t sh_two_s[2 * (ND_WAVES + 1)];
    __shared__ double sh_sum[ND_WAVES];
    __shared__ float sh_mem[RK_MAX_NODES];                  // memory of the nodes: sums of wishes, then what is left
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t J = A.n_jobs, N = A.n_nodes;
    const float INF = __int_as_float(0x7F800000);
    const uint32_t per_thread = (N + ND_THREADS - 1) / ND_THREADS;          // <= ND_PER

    // exclusive prefix sum over the threads of the workgroup (thread order); all threads call it
    auto block_scan = [&](uint32_t val, uint32_t &all) {
        uint32_t inc = val;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(inc, off, 64);
            if ((int)lane >= off) inc += o;
        }
        if (lane == 63) sh_scan[wave] = inc;
        __syncthreads();
        uint32_t base = 0;
        all = 0;
        for (uint32_t w = 0; w < ND_WAVES; ++w) { if (w < wave) base += sh_scan[w]; all += sh_scan[w]; }
        __syncthreads();
        return base + inc - val;
    };

    // ---- the state the jobs are in has been loaded (k_nd_init, k_nd_prepare); no node may hold more than it has
    if (tid == 0) { sh_bad = A.flags[0]; sh_epoch = 0u; sh_moves = 0u; sh_full = 0u; sh_shrinks = 0u; sh_undone = 0u; }
    __syncthreads();
    for (uint32_t n = tid; n < N; n += ND_THREADS)
        if (A.cnt[n] > A.gpn || A.free_g[n] > A.gpn || A.free_c[n] > A.cpn) atomicOr(&sh_bad, 1u);
    __syncthreads();
    if (sh_bad) {                                            // not a placement on these nodes: nothing is scheduled
        for (uint32_t j = tid; j < J; j += ND_THREADS) {
            A.assign[j] = rk_assign{0u, 0u, 0.f, RK_NO_PLAN, 0.f};
            A.place_off[j] = 0u;
        }
        if (tid == 0) {
            A.place_off[J] = 0u; *A.total = 0.f;
            if (A.stats) { A.stats[0] = 0u; A.stats[1] = 0u; A.stats[2] = 0u; A.stats[3] = 0u; A.stats[4] = 1u; }
        }
        return;
    }
    // the node tables and their copy, four words at a time, two pieces in flight (nodes_words is a multiple of four)
    auto copy_nodes = [&](uint32_t *to, const uint32_t *from) {
        const uint4 *src = reinterpret_cast<const uint4 *>(from);
        uint4 *dst = reinterpret_cast<uint4 *>(to);
        const uint32_t n4 = A.nodes_words / 4u;
        for (uint32_t i = tid; i < n4; i += 2 * ND_THREADS) {
            const uint4 a = src[i];
            const bool two = i + ND_THREADS < n4;
            const uint4 b = two ? src[i + ND_THREADS] : a;
            dst[i] = a;
            if (two) dst[i + ND_THREADS] = b;
        }
    };
    auto keep_nodes = [&]() { copy_nodes(A.keep_nodes, A.free_g); };
    auto restore_nodes = [&]() { copy_nodes(A.free_g, A.keep_nodes); };
    // first thread: remember job v as it is before this step changes it
    auto remember = [&](uint32_t v) {
        if (A.stamp[v] == sh_epoch) return;
        A.stamp[v] = sh_epoch;
        A.keep_gi[v] = A.st.gi[v]; A.keep_ci[v] = A.st.ci[v];
        A.keep_ds[2 * v] = A.ds_g[v]; A.keep_ds[2 * v + 1] = A.ds_c[v];
        A.touched[sh_touched++] = v;
    };
    auto put_jobs_back = [&]() {
        for (uint32_t i = 0; i < sh_touched; ++i) {
            const uint32_t v = A.touched[i];
            A.st.gi[v] = A.keep_gi[v]; A.st.ci[v] = A.keep_ci[v];
            A.ds_g[v] = A.keep_ds[2 * v]; A.ds_c[v] = A.keep_ds[2 * v + 1];
        }
        sh_undone += sh_touched ? 1u : 0u;
    };

    // ScheduleJob(j); the same code path for all threads
    auto schedule_job = [&](uint32_t j) {
        for (;;) {                                           // ---- GPUs
            if (tid == 0) {
                const RsStep up = nd_cached_step(A, j, 0);
                sh_step = up;
                sh_lack = (uint32_t)up.dg; sh_lost = 0.f; sh_ok = 1u; sh_touched = 0u; sh_epoch += 1u;
            }
            __syncthreads();
            const RsStep st = sh_step;
            if (!st.any) { __syncthreads(); break; }
            const bool below_min = rs_fl_s(A, j) >= 0 && A.st.gi[j] < rs_fl_s(A, j);
            const uint32_t per_gpu = nd_cpl(A, st.lvl);
            keep_nodes();
            __syncthreads();
            if (A.st.gi[j] >= 0 && st.lvl != A.st.ci[j]) {   // its parts go to the step's level: their CPUs must be free
                const uint32_t more = per_gpu - nd_cpl(A, A.st.ci[j]);
                for (uint32_t n = tid; n < N; n += ND_THREADS) {
                    const uint32_t k = nd_part(A, n, j);
                    if (!k) continue;
                    if (A.free_c[n] < more * k) atomicAnd(&sh_ok, 0u);
                    else A.free_c[n] -= more * k;
                }
                __syncthreads();
            }
            uint32_t n0 = 0;
            bool walking = sh_ok && sh_lack > 0;             // (read here, written again only behind the next barrier)
            __syncthreads();
            while (walking && n0 < N) {                      // the walk over the nodes, a node per thread at a time
                const uint32_t lack = sh_lack;
                const uint32_t n = n0 + tid;
                const bool in = n < N;
                uint32_t offer = 0;
                bool ask = false;                            // somebody here may be shrunk
                if (in) {
                    const uint32_t by_cpu = A.free_c[n] / per_gpu;
                    offer = A.free_g[n] < by_cpu ? A.free_g[n] : by_cpu;
                    uint32_t who;
                    const float low = nd_lowest_on(A, n, j, A.ds_g, who);
                    ask = who != ND_NONE && (below_min || st.slope > low);
                }
                if (tid == 0) { sh_done = ND_THREADS; sh_ask = ND_THREADS; }
                uint32_t all;
                const uint32_t before = block_scan(offer, all);          // (its barriers order the two lines around it)
                if (in && before + offer >= lack) atomicMin(&sh_done, tid);
                if (in && ask && before + offer < lack) atomicMin(&sh_ask, tid);
                __syncthreads();
                const uint32_t done_t = sh_done, ask_t = sh_ask;
                const uint32_t last = done_t < ask_t ? done_t : ask_t;   // the nodes up to here give what they offer
                if (in && tid <= last && offer) nd_add(A, n, j, offer < lack - before ? offer : lack - before, per_gpu);
                if (tid == (last < ND_THREADS ? last : 0u)) {
                    const uint32_t upto = last < ND_THREADS ? before + offer : all;
                    sh_lack = lack - (upto < lack ? upto : lack);
                    sh_vnode = ask_t < done_t ? n0 + ask_t : ND_NONE;
                    sh_next = ask_t < done_t ? n0 + ask_t + 1u : n0 + ND_THREADS;
                }
                __syncthreads();
                const uint32_t f = sh_vnode;
                if (f != ND_NONE) {                          // node f: the job still lacks GPUs and somebody may be shrunk
                    for (;;) {
                        if (wave == 0) {                     // the first wavefront: a resident of node f per lane
                            const uint32_t c = A.cnt[f];
                            const size_t base = (size_t)f * A.gpn;
                            if (c > 64u) {                       // more residents than lanes: the first lane asks them one by one
                                if (lane == 0) {
                                    uint32_t who;
                                    const float low = nd_lowest_on(A, f, j, A.ds_g, who);
                                    if (who == ND_NONE || !(below_min || st.slope > low)) {
                                        sh_v = ND_NONE;
                                    } else {
                                        const RsGive gv = rs_down_gpu(A, who);
                                        remember(who);
                                        const uint32_t per_v = nd_cpl(A, A.st.ci[who]);
                                        const uint32_t here_has = nd_part(A, f, who);
                                        const uint32_t here = (uint32_t)gv.dg < here_has ? (uint32_t)gv.dg : here_has;
                                        nd_drop(A, f, who, here, per_v);
                                        sh_rest = (uint32_t)gv.dg - here; sh_per_v = per_v; sh_v = who;
                                        sh_lost = sh_lost + gv.loss;
                                        A.st.gi[who] = gv.tgt; if (gv.tgt < 0) A.st.ci[who] = 0u;
                                        rs_refresh_give(A, who);
                                        sh_shrinks += 1u;
                                    }
                                }
                            } else {
                                // the node's list and what it has free, asked for together; then the residents' slopes
                                const uint32_t free_g = A.free_g[f], free_c = A.free_c[f];
                                const uint32_t rv = lane < c ? A.res_job[base + lane] : j;
                                const uint32_t rk = lane < c ? A.res_k[base + lane] : 0u;
                                const float sl = rv != j ? A.ds_g[rv] : INF;
                                unsigned long long key = ~0ull;      // (slope as a word that orders like it, job): lower job among equals
                                if (sl < INF) key = ((unsigned long long)rs_ordered(sl) << 32) | rv;
                                key = wave_min_u64_rows(key);
                                const uint32_t who = (uint32_t)key;
                                const float low = rs_unordered((uint32_t)(key >> 32));
                                if (key == ~0ull || !(below_min || st.slope > low)) {
                                    if (lane == 0) sh_v = ND_NONE;
                                } else {
                                    // the job's state and what remembering it reads, together
                                    const int32_t gi0 = A.st.gi[who];
                                    const uint32_t ci0 = A.st.ci[who];
                                    const uint32_t so = A.X.tb.seg_off[who], ns = A.X.tb.seg_off[who + 1] - so;
                                    const uint32_t stamp = A.stamp[who];
                                    const float ds_c0 = A.ds_c[who];
                                    const uint32_t slot = (uint32_t)__ffsll((long long)__ballot(lane < c && rv == who)) - 1u;
                                    const uint32_t here_has = wave_lane_u32(rk, slot);
                                    const float ds_g0 = __uint_as_float(wave_lane_u32(__float_as_uint(sl), slot));
                                    const uint32_t last_v = wave_lane_u32(rv, c - 1u), last_k = wave_lane_u32(rk, c - 1u);
                                    const RsShrunk sk = rs_shrink_wave(A, who, so, ns, 0, gi0, ci0, lane);
                                    if (lane == 0) {
                                        if (stamp != sh_epoch) {     // (remember)
                                            A.stamp[who] = sh_epoch;
                                            A.keep_gi[who] = gi0; A.keep_ci[who] = ci0;
                                            A.keep_ds[2 * who] = ds_g0; A.keep_ds[2 * who + 1] = ds_c0;
                                            A.touched[sh_touched++] = who;
                                        }
                                        const uint32_t per_v = nd_cpl(A, ci0);
                                        const uint32_t here = (uint32_t)sk.gv.dg < here_has ? (uint32_t)sk.gv.dg : here_has;
                                        A.free_g[f] = free_g + here; A.free_c[f] = free_c + here * per_v;      // (nd_drop)
                                        if (here_has - here) A.res_k[base + slot] = here_has - here;
                                        else { A.res_job[base + slot] = last_v; A.res_k[base + slot] = last_k; A.cnt[f] = c - 1u; }
                                        sh_rest = (uint32_t)sk.gv.dg - here; sh_per_v = per_v; sh_v = who;
                                        sh_lost = sh_lost + sk.gv.loss;
                                        A.st.gi[who] = sk.gi; A.st.ci[who] = sk.ci;
                                        A.ds_g[who] = sk.ds_g; A.ds_c[who] = sk.ds_c;
                                        sh_shrinks += 1u;
                                    }
                                }
                            }
                        }
                        __syncthreads();
                        const uint32_t v = sh_v, rest = sh_rest, per_v = sh_per_v;
                        if (v == ND_NONE) break;
                        if (rest > 0) {                      // the rest from its other parts, the last one first
                            uint32_t k[ND_PER], local = 0;
#pragma unroll
                            for (uint32_t i = 0; i < ND_PER; ++i) {
                                const uint32_t r = tid * per_thread + i;     // position from the last node
                                k[i] = (i < per_thread && r < N && N - 1u - r != f) ? nd_part(A, N - 1u - r, v) : 0u;
                                local += k[i];
                            }
                            uint32_t all;
                            uint32_t running = block_scan(local, all);
#pragma unroll
                            for (uint32_t i = 0; i < ND_PER; ++i) {
                                if (k[i] && rest > running) {
                                    const uint32_t give = k[i] < rest - running ? k[i] : rest - running;
                                    nd_drop(A, N - 1u - (tid * per_thread + i), v, give, per_v);
                                }
                                running += k[i];
                            }
                            __syncthreads();
                        }
                        if (tid == 0) {
                            const uint32_t by_cpu = A.free_c[f] / per_gpu;
                            const uint32_t offer = A.free_g[f] < by_cpu ? A.free_g[f] : by_cpu;
                            const uint32_t t = offer < sh_lack ? offer : sh_lack;
                            if (t) nd_add(A, f, j, t, per_gpu);
                            sh_lack -= t;
                        }
                        __syncthreads();
                        if (sh_lack == 0) break;
                    }
                }
                n0 = sh_next;
                walking = sh_lack > 0;
                __syncthreads();
            }
            if (tid == 0) {
                bool ok = sh_ok != 0u && sh_lack == 0u;
                if (ok && !below_min && !(st.gain > sh_lost)) ok = false;
                if (!ok) put_jobs_back();
                else { A.st.gi[j] = st.tgt; A.st.ci[j] = st.lvl; sh_moves += 1u; }
                sh_go = ok ? 1u : 0u;
            }
            __syncthreads();
            const uint32_t go = sh_go;
            if (go) {
                const uint32_t n_changed = sh_touched + 1u;      // a wavefront per job whose state changed
                for (uint32_t i = wave; i < n_changed; i += ND_WAVES) nd_refresh_wave(A, i < sh_touched ? A.touched[i] : j, lane);
            } else {
                restore_nodes();
            }
            __syncthreads();
            if (!go) break;
        }
        for (;;) {                                           // ---- CPUs: on every node the job is on
            if (tid == 0) { sh_step = nd_cached_step(A, j, 1); sh_lost = 0.f; sh_ok = 1u; sh_touched = 0u; sh_epoch += 1u; }
            __syncthreads();
            const RsStep st = sh_step;
            if (!st.any) { __syncthreads(); break; }
            const uint32_t more = nd_cpl(A, st.lvl) - nd_cpl(A, A.st.ci[j]);
            keep_nodes();
            {                                                // its parts, in node order
                uint32_t k[ND_PER], local = 0;
#pragma unroll
                for (uint32_t i = 0; i < ND_PER; ++i) {
                    const uint32_t n = tid * per_thread + i;
                    k[i] = (i < per_thread && n < N) ? nd_part(A, n, j) : 0u;
                    local += k[i] ? 1u : 0u;
                }
                uint32_t all;
                uint32_t at = block_scan(local, all);
#pragma unroll
                for (uint32_t i = 0; i < ND_PER; ++i)
                    if (k[i]) { A.plist[2 * at] = tid * per_thread + i; A.plist[2 * at + 1] = k[i]; ++at; }
                if (tid == 0) sh_np = all;
                __syncthreads();
            }
            const uint32_t np = sh_np;
            bool found = true;                               // every part so far has its CPUs
            for (uint32_t p = 0; p < np && found; ++p) {
                const uint32_t n = A.plist[2 * p], need = more * A.plist[2 * p + 1];
                for (;;) {
                    if (wave == 0) {                         // the first wavefront: its lanes share the job's step down
                        const uint32_t free_here = A.free_c[n];
                        if (free_here >= need) { if (lane == 0) { A.free_c[n] = free_here - need; sh_flag = 0u; } }
                        else {
                            uint32_t who;
                            const float low = nd_lowest_on_wave(A, n, j, A.ds_c, who, lane);
                            if (who == ND_NONE || !(st.slope > low)) { if (lane == 0) { sh_ok = 0u; sh_flag = 0u; } }
                            else {
                                const int32_t gi0 = A.st.gi[who];
                                const uint32_t ci0 = A.st.ci[who];
                                const uint32_t so = A.X.tb.seg_off[who], ns = A.X.tb.seg_off[who + 1] - so;
                                const RsShrunk sk = rs_shrink_wave(A, who, so, ns, 1, gi0, ci0, lane);
                                if (lane == 0) {
                                    remember(who);
                                    sh_per_v = nd_cpl(A, ci0) - nd_cpl(A, ci0 - 1u);
                                    sh_v = who; sh_flag = 1u;
                                    sh_lost = sh_lost + sk.gv.loss;
                                    A.st.ci[who] = sk.ci;
                                    A.ds_g[who] = sk.ds_g; A.ds_c[who] = sk.ds_c;
                                    sh_shrinks += 1u;
                                }
                            }
                        }
                    }
                    __syncthreads();
                    const uint32_t flag = sh_flag, v = sh_v, less = sh_per_v;
                    found = sh_ok != 0u;
                    if (flag)                                 // the job that gives a level gives it on all its nodes
                        for (uint32_t m = tid; m < N; m += ND_THREADS) A.free_c[m] += less * nd_part(A, m, v);
                    __syncthreads();
                    if (!flag) break;
                }
            }
            if (tid == 0) {
                bool ok = sh_ok != 0u;
                if (ok && !(st.gain > sh_lost)) ok = false;
                if (!ok) put_jobs_back();
                else { A.st.ci[j] = st.lvl; sh_moves += 1u; }
                sh_go = ok ? 1u : 0u;
            }
            __syncthreads();
            const uint32_t go = sh_go;
            if (go) {
                const uint32_t n_changed = sh_touched + 1u;      // a wavefront per job whose state changed
                for (uint32_t i = wave; i < n_changed; i += ND_WAVES) nd_refresh_wave(A, i < sh_touched ? A.touched[i] : j, lane);
            } else {
                restore_nodes();
            }
            __syncthreads();
            if (!go) break;
        }
    };

    // ---- privileged jobs (below their floor) come first, in job order: their list (tmp_off serves as the list)
    uint32_t n_first = 0;
    for (uint32_t base = 0; base < J; base += ND_THREADS) {
        const uint32_t j = base + tid;
        const bool is = j < J && A.first[j] != 0u;
        uint32_t all;
        const uint32_t at = block_scan(is ? 1u : 0u, all);
        if (is) A.tmp_off[n_first + at] = j;
        n_first += all;
    }
    __syncthreads();
    // ---- then the others: their order is fixed once (when the privileged jobs are through), by GPU slope, then CPU
    // slope (both descending), then index.
    // Most jobs find nothing to do when their turn comes, and whether that is so follows from values that change
    // only when a step is committed.  A GPU step does nothing when there is none, or when what the nodes can give
    // a job at its level (GPUs with their CPUs) is less than the step needs and no job anywhere has a slope below
    // this job's (then nobody on any node may be shrunk).  A CPU step does nothing when there is none, or when no
    // job anywhere has a lower CPU slope and all free CPUs together are fewer than the step needs.  Passing over
    // such a job changes nothing, so the jobs are not sorted: all threads look for the first job in the order, after
    // the one served last, that is not of that kind; it is served in full and the search starts again.
    auto comes_before = [&](float ga, float ca, uint32_t a, float gb, float cb, uint32_t b) {
        return ga > gb || (ga == gb && (ca > cb || (ca == cb && a < b)));
    };
    float last_g = INF, last_c = INF;
    uint32_t last_j = 0u, moves_seen = ND_NONE, k_first = 0;
    bool others = false;
    for (;;) {                                               // one job per turn; ScheduleJob appears once in the code
        if (k_first < n_first) {
            schedule_job(A.tmp_off[k_first++]);
            continue;
        }
        if (!others) {
            for (uint32_t j = tid; j < J; j += ND_THREADS) {
                const bool in = rs_part(A, j) && !A.first[j];
                A.sg[j] = in ? A.ug[j] : -1.f;               // the cached slopes are current; -1: not in the list
                A.sc[j] = in ? A.uc[j] : -1.f;
            }
            others = true;
        }
        __syncthreads();
        const bool fresh = sh_moves != moves_seen;          // a step was committed since the last look (or this is the first)
        moves_seen = sh_moves;
        __syncthreads();
        if (fresh) {
            if (tid < RK_MAX_CPU_LEVELS) sh_take[tid] = 0ull;
            if (tid == 0) sh_free_c = 0ull;
            {
                RsMin two[2];
                rs_two_lowest<ND_WAVES, ND_THREADS>(sh_ds, J, tid, lane, wave, sh_two_k, sh_two_s, two);
                if (tid == 0) { sh_min[0] = two[0]; sh_min[1] = two[1]; }
            }
            {                                                    // what the nodes can give at every CPU level
                unsigned long long fc = 0;
                for (uint32_t n = tid; n < N; n += ND_THREADS) fc += A.free_c[n];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) fc += __shfl_xor(fc, off, 64);
                if (lane == 0 && fc) atomicAdd(&sh_free_c, fc);
                for (uint32_t l = 0; l < A.X.grid.n_cpu; ++l) {
                    const uint32_t per_gpu = nd_cpl(A, l);
                    unsigned long long t = 0;
                    for (uint32_t n = tid; n < N; n += ND_THREADS) {
                        const uint32_t by_cpu = A.free_c[n] / per_gpu;
                        t += A.free_g[n] < by_cpu ? A.free_g[n] : by_cpu;
                    }
#pragma unroll
                    for (int off = 32; off >= 1; off >>= 1) t += __shfl_xor(t, off, 64);
                    if (lane == 0 && t) atomicAdd(&sh_take[l], t);
                }
            }
        }
        __syncthreads();
        const RsMin mg = sh_min[0], mc = sh_min[1];
        const unsigned long long free_c = sh_free_c;
        float best_g = -1.f, best_c = -1.f;
        uint32_t best_j = ND_NONE;
        for (uint32_t j0 = tid; j0 < J; j0 += 4 * ND_THREADS) {          // four jobs' values in flight
            float kg[4], kc[4], ug[4], uc[4];
            uint32_t dg[4], lv[4];
            unsigned long long dc[4];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint32_t j = j0 + k * ND_THREADS;
                const bool in = j < J;
                kg[k] = in ? A.sg[j] : -1.f; kc[k] = in ? A.sc[j] : -1.f;
                ug[k] = in ? A.ug[j] : 0.f; uc[k] = in ? A.uc[j] : 0.f;
                dg[k] = in ? A.udg[j] : 0u; lv[k] = in ? A.st.ci[j] : 0u; dc[k] = in ? A.udc_c[j] : 0ull;
            }
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint32_t j = j0 + k * ND_THREADS;
                if (kg[k] < 0.f || !comes_before(last_g, last_c, last_j, kg[k], kc[k], j)) continue;
                const float lowest_g = j == mg.i1 ? mg.m2 : mg.m1, lowest_c = j == mc.i1 ? mc.m2 : mc.m1;
                const bool gpu_idle = !(ug[k] > 0.f) || (sh_take[lv[k]] < dg[k] && !(ug[k] > lowest_g));
                const bool cpu_idle = !(uc[k] > 0.f) || (free_c < dc[k] && !(uc[k] > lowest_c));
                if (gpu_idle && cpu_idle) continue;
                if (best_j == ND_NONE || comes_before(kg[k], kc[k], j, best_g, best_c, best_j)) { best_g = kg[k]; best_c = kc[k]; best_j = j; }
            }
        }
        {                                                    // the first of the threads' candidates in the order
            const RsPick pick = rs_pick_first<ND_WAVES>(best_g, best_c, best_j, lane, wave, sh_pick_key, sh_pick_j);
            best_g = pick.g; best_c = pick.c; best_j = pick.j;
        }
        if (best_j == ND_NONE) break;
        if (tid == 0) sh_full += 1u;
        schedule_job(best_j);
        last_g = best_g; last_c = best_c; last_j = best_j;
    }
    __syncthreads();

    // ---- memory, then the records.  Parts of all jobs, grouped by job (in no order yet)
    for (uint32_t j = tid; j < J; j += ND_THREADS) A.np[j] = 0u;
    __syncthreads();
    for (uint32_t n = tid; n < N; n += ND_THREADS)
        for (uint32_t i = 0; i < A.cnt[n]; ++i) atomicAdd(&A.np[A.res_job[(size_t)n * A.gpn + i]], 1u);
    __syncthreads();
    const uint32_t jobs_per_thread = (J + ND_THREADS - 1) / ND_THREADS;
    auto scan_jobs = [&](const uint32_t *count, bool only_kept, uint32_t *off) {       // off[J] = the sum
        uint32_t local = 0;
        for (uint32_t i = 0; i < jobs_per_thread; ++i) {
            const uint32_t j = tid * jobs_per_thread + i;
            if (j < J && (!only_kept || A.tier[j] != ND_NONE)) local += count[j];
        }
        uint32_t all;
        uint32_t at = block_scan(local, all);
        for (uint32_t i = 0; i < jobs_per_thread; ++i) {
            const uint32_t j = tid * jobs_per_thread + i;
            if (j >= J) break;
            off[j] = at;
            if (!only_kept || A.tier[j] != ND_NONE) at += count[j];
        }
        if (tid == 0) off[J] = all;
    };
    scan_jobs(A.np, false, A.tmp_off);
    for (uint32_t j = tid; j < J; j += ND_THREADS) A.stamp[j] = 0u;          // (cursor of the job's parts)
    __syncthreads();
    for (uint32_t n = tid; n < N; n += ND_THREADS)
        for (uint32_t i = 0; i < A.cnt[n]; ++i) {
            const uint32_t job = A.res_job[(size_t)n * A.gpn + i];
            const uint32_t at = A.tmp_off[job] + atomicAdd(&A.stamp[job], 1u);
            A.tmp_parts[2 * (size_t)at] = n; A.tmp_parts[2 * (size_t)at + 1] = A.res_k[(size_t)n * A.gpn + i];
        }
    for (uint32_t n = tid; n < N; n += ND_THREADS) sh_mem[n] = 0.f;
    if (tid == 0) sh_fit = A.gpn <= 4096u ? 1u : 0u;
    __syncthreads();
    const uint64_t rows = (uint64_t)A.X.grid.n_cpu * A.X.grid.n_mem;
    auto tier_cost = [&](uint32_t m, uint32_t g) {
        float v = A.X.grid.mem_levels_gb[m];
        if (A.X.grid.mem_mode) v = v * (float)g;
        return v;
    };
    auto value_at = [&](uint32_t j, uint32_t m) {
        return A.X.best_thr[rows * A.X.tb.seg_off[j] + ((uint64_t)A.st.ci[j] * A.X.grid.n_mem + m) * rs_ns(A, j) + (uint32_t)A.st.gi[j]];
    };
    // the tier every job would like (highest throughput, smallest such tier), and what that asks of the nodes
    for (uint32_t j = tid; j < J; j += ND_THREADS) {
        uint32_t bm = ND_NONE;
        if (A.st.gi[j] >= 0) {
            float bv = 0.f;
            for (uint32_t m = 0; m < A.X.grid.n_mem; ++m) {
                const float v = value_at(j, m);
                if (v > bv) { bv = v; bm = m; }
            }
            if (bm != ND_NONE) {
                const uint32_t g = (uint32_t)rs_g(A, j, A.st.gi[j]);
                const float cost = tier_cost(bm, g);
                for (uint32_t i = 0; i < A.np[j]; ++i) {
                    const size_t at = 2 * (size_t)(A.tmp_off[j] + i);
                    atomicAdd(&sh_mem[A.tmp_parts[at]], (cost * (float)A.tmp_parts[at + 1]) / (float)g);
                }
            }
        }
        A.tier[j] = bm;
    }
    __syncthreads();
    for (uint32_t n = tid; n < N; n += ND_THREADS)
        if (!(sh_mem[n] <= A.mem_gb * 0.999f)) atomicAnd(&sh_fit, 0u);
    __syncthreads();
    if (!sh_fit) {                                           // some node's memory can bind: job by job, in order
        for (uint32_t n = tid; n < N; n += ND_THREADS) sh_mem[n] = A.mem_gb;
        __syncthreads();
        if (wave == 0) {
            for (uint32_t j = 0; j < J; ++j) {
                if (A.st.gi[j] < 0) continue;
                const uint32_t g = (uint32_t)rs_g(A, j, A.st.gi[j]);
                const uint32_t a = A.tmp_off[j], P = A.np[j];
                float bv = 0.f;
                uint32_t bm = ND_NONE;
                for (uint32_t m = 0; m < A.X.grid.n_mem; ++m) {
                    const float cost = tier_cost(m, g);
                    bool bad = false;
                    for (uint32_t i = lane; i < P; i += 64u) {
                        const size_t at = 2 * (size_t)(a + i);
                        if (!((cost * (float)A.tmp_parts[at + 1]) / (float)g <= sh_mem[A.tmp_parts[at]])) bad = true;
                    }
                    if (__ballot(bad)) continue;
                    const float v = value_at(j, m);
                    if (v > bv) { bv = v; bm = m; }
                }
                if (bm != ND_NONE) {
                    const float cost = tier_cost(bm, g);
                    for (uint32_t i = lane; i < P; i += 64u) {
                        const size_t at = 2 * (size_t)(a + i);
                        sh_mem[A.tmp_parts[at]] = sh_mem[A.tmp_parts[at]] - (cost * (float)A.tmp_parts[at + 1]) / (float)g;
                    }
                }
                if (lane == 0) A.tier[j] = bm;
            }
        }
        __syncthreads();
    }
    // the records: a job's parts in node order
    scan_jobs(A.np, true, A.place_off);
    if (tid == 0) sh_np = 0u;                                // jobs with many parts (their list: `touched`)
    __syncthreads();
    double sum = 0.0;
    for (uint32_t j = tid; j < J; j += ND_THREADS) {
        rk_assign out = {0u, 0u, 0.f, RK_NO_PLAN, 0.f};
        const uint32_t m = A.tier[j];
        if (m != ND_NONE) {
            const uint32_t g = (uint32_t)rs_g(A, j, A.st.gi[j]);
            const uint32_t per_gpu = nd_cpl(A, A.st.ci[j]);
            const float cost = tier_cost(m, g);
            out.g = g; out.c = per_gpu * g; out.mem_gb = cost;
            out.plan = A.X.best_plan[rows * A.X.tb.seg_off[j] + ((uint64_t)A.st.ci[j] * A.X.grid.n_mem + m) * rs_ns(A, j) + (uint32_t)A.st.gi[j]];
            out.thr = value_at(j, m);
            sum += (double)out.thr / (double)A.X.ref_thr[j];
            const uint32_t P = A.np[j], a = A.tmp_off[j], to = A.place_off[j];
            if (P <= 8u) {                                   // few parts: this thread ranks them
                for (uint32_t i = 0; i < P; ++i) {
                    const uint32_t node = A.tmp_parts[2 * (size_t)(a + i)], k = A.tmp_parts[2 * (size_t)(a + i) + 1];
                    uint32_t rank = 0;
                    for (uint32_t q = 0; q < P; ++q) rank += A.tmp_parts[2 * (size_t)(a + q)] < node ? 1u : 0u;
                    A.entries[to + rank] = rk_place_entry{node, k, per_gpu * k, (cost * (float)k) / (float)g};
                }
            } else {
                A.touched[atomicAdd(&sh_np, 1u)] = j;
            }
        }
        A.assign[j] = out;
    }
    __syncthreads();
    const uint32_t n_wide = sh_np;
    for (uint32_t w = wave; w < n_wide; w += ND_WAVES) {      // many parts: a wavefront ranks them
        const uint32_t j = A.touched[w];
        const uint32_t m = A.tier[j], P = A.np[j];
        const uint32_t g = (uint32_t)rs_g(A, j, A.st.gi[j]);
        const uint32_t per_gpu = nd_cpl(A, A.st.ci[j]);
        const float cost = tier_cost(m, g);
        const uint32_t a = A.tmp_off[j], to = A.place_off[j];
        for (uint32_t i = lane; i < P; i += 64u) {
            const uint32_t node = A.tmp_parts[2 * (size_t)(a + i)], k = A.tmp_parts[2 * (size_t)(a + i) + 1];
            uint32_t rank = 0;
            for (uint32_t q = 0; q < P; ++q) rank += A.tmp_parts[2 * (size_t)(a + q)] < node ? 1u : 0u;
            A.entries[to + rank] = rk_place_entry{node, k, per_gpu * k, (cost * (float)k) / (float)g};
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) sh_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        double s = 0.0;
        for (uint32_t w = 0; w < ND_WAVES; ++w) s += sh_sum[w];
        *A.total = (float)s;
        if (A.stats) { A.stats[0] = sh_moves; A.stats[1] = sh_full; A.stats[2] = sh_shrinks; A.stats[3] = sh_undone; A.stats[4] = 0u; }
    }
}

}  // namespace

extern "C" int32_t rk_reschedule_nodes(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                       const rk_alloc_grid *grid, const rk_nodes *nodes, const float *best_thr,
                                       const uint32_t *best_plan, const float *curve_thr,
                                       const rk_job_state *jobs_state, const uint32_t *prev_off,
                                       const rk_place_entry *prev_entries, uint64_t n_prev_entries,
                                       rk_assign *assign, uint32_t *place_off,
                                       rk_place_entry *entries, uint64_t cap_entries, float *total, uint32_t *stats) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, 0, table ? table->n_jobs : 0))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (!nodes || !total || !jobs_state || !place_off) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    const uint32_t J = table->n_jobs;
    if (J > 0 && (!ref_thr || !assign || !jobs_state->cur_seg || !jobs_state->cur_c ||
                  (table->n_segs > 0 && (!best_thr || !best_plan || !curve_thr))))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if ((prev_off == nullptr) != (prev_entries == nullptr))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "the earlier placement needs both its offsets and its entries");
    if (nodes->n_nodes == 0 || nodes->n_nodes > RK_MAX_NODES || nodes->gpus_per_node == 0 ||
        nodes->gpus_per_node > 65535u || nodes->cpus_per_node > 65535u || !(nodes->mem_per_node_gb >= 0.f))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "nodes: 1..%u nodes of 1..65535 GPUs, at most 65535 CPUs, memory >= 0", RK_MAX_NODES);
    if (grid->cpu_mode != 1u)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "the search over nodes needs CPU levels per GPU (cpu_mode 1)");
    const uint64_t gpus = (uint64_t)nodes->n_nodes * nodes->gpus_per_node;
    if (gpus > ND_MAX_GPUS) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%llu GPUs, the search over nodes takes up to %u", (unsigned long long)gpus, ND_MAX_GPUS);
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    if (J > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u jobs, the allocation kernels take up to %u", J, RK_MAX_JOBS_PER_ROUND);
    if (cap_entries < gpus && J > 0) return rk_fail(ctx, RK_ERR_CAPACITY, "entries: %llu records, %llu may be needed", (unsigned long long)cap_entries, (unsigned long long)gpus);
    if (J > 0 && !entries) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    return rk_launch_reschedule_nodes(ctx, ref_thr, table, grid, nodes, best_thr, best_plan, curve_thr, jobs_state, prev_off,
                                      prev_entries, n_prev_entries, assign, place_off, entries, total, stats);
}

int32_t rk_launch_reschedule_nodes(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                   const rk_alloc_grid *grid, const rk_nodes *nodes, const float *best_thr,
                                   const uint32_t *best_plan, const float *curve_thr, const rk_job_state *jobs_state,
                                   const uint32_t *prev_off, const rk_place_entry *prev_entries, uint64_t n_prev_entries,
                                   rk_assign *assign, uint32_t *place_off, rk_place_entry *entries, float *total,
                                   uint32_t *stats) {
    const uint32_t J = table->n_jobs;
    const uint64_t gpus = (uint64_t)nodes->n_nodes * nodes->gpus_per_node;
    int32_t rc;
    const size_t n = J ? J : 1, N = nodes->n_nodes;
    const size_t nodes_words = (3 * N + 2 * (size_t)gpus + 3) & ~(size_t)3;      // whole 16-byte pieces: the copy moves four words at a time
    uint32_t *w_nodes, *w_jobs;
    float *f_jobs;
    unsigned long long *u64;
    if ((rc = rk_scratch(ctx, SL_ND_NODES, (2 * nodes_words + 2 * N + 2 * (size_t)gpus) * sizeof(uint32_t), (void **)&w_nodes))) return rc;
    if ((rc = rk_scratch(ctx, SL_ND_U32, (15 * n + 2) * sizeof(uint32_t), (void **)&w_jobs))) return rc;
    if ((rc = rk_scratch(ctx, SL_ND_F32, 10 * n * sizeof(float), (void **)&f_jobs))) return rc;
    if ((rc = rk_scratch(ctx, SL_ND_U64, 2 * n * sizeof(unsigned long long), (void **)&u64))) return rc;
    NdKernArgs K;
    NdBody &A = K.b;
    K.X.ref_thr = ref_thr; K.X.tb = table_dev(table); K.X.grid = grid_dev(grid);
    K.X.best_thr = best_thr; K.X.best_plan = best_plan; K.X.curve_thr = curve_thr;
    A.G = gpus;
    A.n_jobs = J; A.n_nodes = nodes->n_nodes; A.gpn = nodes->gpus_per_node; A.cpn = nodes->cpus_per_node;
    A.mem_gb = nodes->mem_per_node_gb;
    A.state = jobs_state->state; A.cur_seg = jobs_state->cur_seg; A.cur_c = jobs_state->cur_c;
    A.floor_seg = jobs_state->floor_seg; A.floor_c = jobs_state->floor_c;
    A.prev_off = prev_off; A.prev_entries = prev_entries; A.n_prev = n_prev_entries;
    A.free_g = w_nodes; A.free_c = w_nodes + N; A.cnt = w_nodes + 2 * N; A.res_job = w_nodes + 3 * N;
    A.res_k = A.res_job + gpus;
    A.keep_nodes = w_nodes + nodes_words; A.nodes_words = (uint32_t)nodes_words;
    A.plist = w_nodes + 2 * nodes_words; A.tmp_parts = A.plist + 2 * N;
    A.st.gi = reinterpret_cast<int32_t *>(w_jobs); A.st.ci = w_jobs + n; A.udg = w_jobs + 2 * n; A.touched = w_jobs + 3 * n;
    A.stamp = w_jobs + 4 * n; A.first = w_jobs + 5 * n; A.keep_ci = w_jobs + 6 * n;
    A.keep_gi = reinterpret_cast<int32_t *>(w_jobs + 7 * n); A.np = w_jobs + 8 * n; A.tier = w_jobs + 9 * n;
    A.tmp_off = w_jobs + 10 * n;                             // n + 1 words
    A.flags = w_jobs + 11 * n + 1;
    uint32_t *more = w_jobs + 11 * n + 2;
    A.tgt_g = reinterpret_cast<int32_t *>(more); A.lvl_g = more + n; A.lvl_c = more + 2 * n; A.any = more + 3 * n;
    A.ds_g = f_jobs; A.ds_c = f_jobs + n; A.ug = f_jobs + 2 * n; A.uc = f_jobs + 3 * n; A.sg = f_jobs + 4 * n;
    A.sc = f_jobs + 5 * n; A.keep_ds = f_jobs + 6 * n; A.gain_g = f_jobs + 8 * n; A.gain_c = f_jobs + 9 * n;
    A.udc_g = u64; A.udc_c = u64 + n;
    A.assign = assign; A.place_off = place_off; A.entries = entries; A.total = total; A.stats = stats;
    k_nd_init<<<(uint32_t)((N + 255) / 256), 256, 0, ctx->stream>>>(K);
    RK_CHECK_LAUNCH(ctx, "k_nd_init");
    if (J > 0) {
        k_nd_prepare<<<(J + 255) / 256, 256, 0, ctx->stream>>>(K);
        RK_CHECK_LAUNCH(ctx, "k_nd_prepare");
    }
    const size_t lds = (size_t)2 * n * sizeof(float);                           // at most 96 KiB
    if (lds > 64 * 1024 && !ctx->nodes_lds_raised) {
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_reschedule_nodes),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 2 * RK_MAX_JOBS_PER_ROUND * sizeof(float)));
        ctx->nodes_lds_raised = true;
    }
    k_reschedule_nodes<<<1, ND_THREADS, lds, ctx->stream>>>(K);
    RK_CHECK_LAUNCH(ctx, "k_reschedule_nodes");
    return RK_OK;
}
