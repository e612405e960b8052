// Greedy marginal-gain allocation over the resource sensitivity curves
// (paper Sec. 5.2: prefer the jobs that gain the most per unit of resource,
// GPU slopes before CPU slopes; memory is granted last from the chosen plan's
// estimate).
//
// The rule is sequential: repeatedly take the (job, larger amount) with the
// highest float32 slope ((v1 - v0) / ref_thr) / delta among the steps that
// still fit; ties go to the smaller amount, then to the lower job index.
// It is evaluated without running every step in sequence.  Per pass (GPUs,
// then CPUs):
//
//  k_hull   Each job's steps, were capacity never short, form a fixed walk
//           over the upper hull of its curve (one wavefront per job; two or
//           four jobs per wavefront when none has more than 32 or 16 amounts:
//           k_hull_groups).  With
//           each slope replaced by the running minimum of the walk, the
//           sequential order is the descending order of these keys (then job,
//           then position in the walk).
//  k_hist   Any key threshold whose whole set of steps {key > threshold} fits
//           the capacity selects a prefix of the sequential order.  Two
//           histogram levels over the top 12 + 12 key bits (cost per bin) find
//           the largest such threshold at 24-bit resolution.
//  k_apply  applies that prefix to every job at once and caches each job's
//           next step (the walk's next step if it still fits, otherwise a fresh
//           search within the capacity that is left).
//  k_tail   the plain step-by-step loop on the little capacity that is left:
//           one workgroup per round, argmax over the cached steps, which each
//           thread keeps in registers for the jobs it owns.
//  When no job's CPU walk has a step, the CPU pass's k_hist, k_apply and k_tail
//  return at once (a per-round flag raised by its k_hull).
//
// Memory (k_mem_wish / k_mem_finish): when the tiers every job would like fit
// with margin, all are granted in parallel; otherwise one wavefront takes the
// decisions in job order.
//
// Service-level floors (k_floors, optional): before the passes, guaranteed
// jobs are granted their minimum demand in job order while their tenant's
// quota and the free capacity last; the passes then start from these floors
// and leave out the guaranteed jobs that have to wait.
#include "rk_internal.h"
#include "rk_model.h"
#include "rk_loop.h"

namespace {

constexpr int TAIL_THREADS = 1024;
constexpr int HULL_THREADS = 256;
constexpr int JOB_THREADS = 256;           // kernels with one thread per job
constexpr uint32_t BINS = 4096;            // 12 key bits per histogram level

struct HullBuf {             // walk steps, entry (k, job) at k*stride + job (job relative to the call's first job)
    uint32_t *key;           // float bits of the running-minimum slope; 0 from the end of the walk on
    float *raw;              // the step's own slope
    uint16_t *tgt;           // target: segment index (GPU pass) or CPU level (CPU pass)
    uint32_t *dg;            // GPUs the step adds
    unsigned long long *dc;  // CPUs the step adds
    uint32_t stride, width;
};

struct Hist {                // per round, pass and level: cost of the steps per key bin
    uint32_t *g;             // [n_rounds][2 passes][2 levels][BINS]
    unsigned long long *c;
};

struct JobState {            // per job of the call, between the kernels
    int32_t *gi;             // granted segment index, -1 = no GPUs
    uint32_t *g;             // granted GPUs
    uint32_t *ci;            // granted CPU level
    float *step_slope;       // cached best next step: slope (0 = none), target, GPUs it adds
    uint16_t *step_tgt, *step_dg;
    unsigned long long *free_g, *free_c;   // per round: capacity left (after apply; after the tail)
    uint32_t *cpu_steps;     // per round: non-zero when some job's CPU walk has a step (else the CPU pass has nothing to do)
    double *partial;         // per round and block of k_mem_wish: {sum of wish GiB, sum of thr/ref}
    uint32_t blocks_per_round;
    // floors, all null without them: the state a job starts from (segment index
    // or -1, CPU level), whether it takes part (RK_JOB_NORMAL), sits the round
    // out (RK_JOB_OUT) or keeps exactly its floor (RK_JOB_FROZEN), and per round
    // the capacity left after the floors ([free G | free C])
    int32_t *fl_gi;
    uint32_t *fl_ci;
    uint8_t *waits;
    unsigned long long *cap0;
};

struct Floor { int32_t gi; uint32_t ci; uint32_t state; };

__device__ __forceinline__ Floor floor_of(const JobState &st, uint32_t jrel) {
    Floor f = {-1, 0u, RK_JOB_NORMAL};
    if (st.fl_gi) { f.gi = st.fl_gi[jrel]; f.ci = st.fl_ci[jrel]; f.state = st.waits[jrel]; }
    return f;
}

// Rounds: job ranges and cluster capacities, either device arrays or, for a
// single round, values carried in the kernel arguments.
struct RoundArgs {
    const uint32_t *round_off;
    const rk_cluster *clusters;
    uint32_t n_rounds, inline_one;
    uint32_t off0, off1;
    rk_cluster cl;
};

struct Ctx {                 // what every kernel of the allocation needs
    const float *ref_thr;
    TableDev tb;
    GridDev grid;
    RoundArgs R;
    uint32_t jb;             // first job of the call (origin of the segment-layout arrays)
    const uint32_t *jmap;    // optional: the job whose curves slot j of the call uses (rounds that share jobs)
    const float *best_thr;
    const uint32_t *best_plan;
    const float *curve_thr;
};

// The job whose plan table, curves and reference throughput slot j uses.
__device__ __forceinline__ uint32_t job_of(const Ctx &X, uint32_t j) { return X.jmap ? X.jmap[j] : j; }

__device__ __forceinline__ void round_of(const RoundArgs &R, uint32_t r, uint32_t &j0, uint32_t &j1, rk_cluster &cl) {
    if (R.inline_one) { j0 = R.off0; j1 = R.off1; cl = R.cl; }
    else { j0 = R.round_off[r]; j1 = R.round_off[r + 1]; cl = R.clusters[r]; }
}

__device__ __forceinline__ uint32_t round_index_of(const RoundArgs &R, uint32_t j) {
    uint32_t lo = 0, hi = R.n_rounds;                     // last r with round_off[r] <= j
    while (!R.inline_one && hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (R.round_off[mid] <= j) lo = mid; else hi = mid;
    }
    return lo;
}


__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ size_t hist_at(uint32_t rnd, int pass, int level) {
    return (((size_t)rnd * 2 + pass) * 2 + level) * BINS;
}

// capacities a pass starts from
template <int PASS>
__device__ __forceinline__ void pass_caps(const RoundArgs &R, const rk_cluster &cl, const JobState &st, uint32_t rnd,
                                          unsigned long long &capG, unsigned long long &capC) {
    if (PASS == 0) {
        if (st.cap0) { capG = st.cap0[rnd]; capC = st.cap0[R.n_rounds + rnd]; }
        else { capG = cl.G; capC = cl.C; }
    } else { capG = 0; capC = st.free_c[rnd]; }
}

// ------------------------------------------------------------------ hull walks
// One wavefront per job; lanes hold the candidate amounts.  PASS 0: GPU counts
// of the job (CPU level of its floor, the lowest without one; highest memory
// tier; values from the curves); PASS 1: CPU levels at the granted GPU count
// (values from the per-segment maxima).  Amounts that the whole round could
// never afford are left out.
template <int PASS>
__global__ __launch_bounds__(HULL_THREADS) void k_hull(Ctx X, JobState st, HullBuf H, Hist zero, size_t zero_bins) {
    // the histograms of the kernels that follow start at zero (zero_bins = 0: nothing to clear)
    for (size_t i = (size_t)blockIdx.x * HULL_THREADS + threadIdx.x; i < zero_bins; i += (size_t)gridDim.x * HULL_THREADS) {
        zero.g[i] = 0u;
        zero.c[i] = 0ull;
        if (i < X.R.n_rounds) st.cpu_steps[i] = 0u;       // (there are more bins than rounds)
    }
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t jrel = blockIdx.x * (HULL_THREADS / 64) + (threadIdx.x >> 6);
    if (jrel >= H.stride) return;                         // whole wavefront
    const uint32_t j = X.jb + jrel;
    const uint32_t rnd = round_index_of(X.R, j);
    uint32_t rj0, rj1;
    rk_cluster cl;
    round_of(X.R, rnd, rj0, rj1, cl);
    const GridDev &grid = X.grid;
    const float *__restrict__ vals = PASS == 0 ? X.curve_thr : X.best_thr;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    const uint32_t ju = job_of(X, j);
    const uint32_t s0 = X.tb.seg_off[ju], ns = X.tb.seg_off[ju + 1] - s0;
    const uint64_t jbase = (uint64_t)n_rows * (s0 - X.tb.seg_off[X.jb]);
    const float ref = X.ref_thr[ju];

    uint32_t npts, g_fixed = 0, c_fixed = 0;
    int32_t cur_i;
    unsigned long long cost_cur, cap_c, cap_g = 0;
    float cur;
    int32_t gi = -1;
    if (PASS == 0) {
        const Floor fl = floor_of(st, jrel);
        unsigned long long startG, startC;
        pass_caps<0>(X.R, cl, st, rnd, startG, startC);
        c_fixed = fl.ci;
        npts = fl.state != RK_JOB_NORMAL ? 0u : ns;
        cur_i = fl.gi;
        cost_cur = fl.gi < 0 ? 0ull : (unsigned long long)X.tb.seg_g[s0 + fl.gi];
        cur = fl.gi < 0 ? 0.f : vals[jbase + (uint64_t)(c_fixed * n_mem + n_mem - 1) * ns + fl.gi];
        cap_g = startG + cost_cur;                       // the floor is already paid for
        cap_c = startC + (fl.gi < 0 ? 0ull : cpu_cost(grid, c_fixed, (uint32_t)cost_cur));
    } else {
        gi = st.gi[jrel];
        npts = (gi < 0 || (st.waits && st.waits[jrel] != RK_JOB_NORMAL)) ? 0u : grid.n_cpu;
        g_fixed = gi < 0 ? 0u : st.g[jrel];
        cur_i = (int32_t)st.ci[jrel];
        cost_cur = cpu_cost(grid, (uint32_t)cur_i, g_fixed);
        cap_c = st.free_c[rnd] + cost_cur;               // the level held is already paid for
        cur = gi < 0 ? 0.f : vals[jbase + (uint64_t)((uint32_t)cur_i * n_mem + n_mem - 1) * ns + gi];
    }
    // amount s: its cost in the pass's resource and its value
    auto cost_of = [&](uint32_t s) -> unsigned long long {
        return PASS == 0 ? (unsigned long long)X.tb.seg_g[s0 + s] : cpu_cost(grid, s, g_fixed);
    };
    auto value_of = [&](uint32_t s) -> float {
        return PASS == 0 ? vals[jbase + (uint64_t)(c_fixed * n_mem + n_mem - 1) * ns + s]
                         : vals[jbase + (uint64_t)(s * n_mem + n_mem - 1) * ns + gi];
    };
    auto affordable = [&](unsigned long long cost) -> bool {
        if (PASS == 0) return cost <= cap_g && cpu_cost(grid, c_fixed, (uint32_t)cost) <= cap_c;
        return cost <= cap_c;
    };

    // the first 64 amounts stay in registers over the whole walk (most jobs have no more)
    unsigned long long cost0 = 0;
    float val0 = 0.f;
    if (lane < npts) { cost0 = cost_of(lane); val0 = value_of(lane); }

    uint32_t k = 0;
    float prev = __uint_as_float(0x7F800000u);
    while (k < H.width) {
        unsigned long long best = 0;
        for (uint32_t base = 0; base < npts; base += 64) {
            const uint32_t s = base + lane;
            if (s < npts && (int32_t)s > cur_i) {
                const unsigned long long cost = base == 0 ? cost0 : cost_of(s);
                if (affordable(cost)) {
                    const float v = base == 0 ? val0 : value_of(s);
                    if (v > cur) {
                        float sl = (v - cur) / ref;
                        sl = sl / (float)(cost - cost_cur);
                        const unsigned long long c = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - s);
                        best = c > best ? c : best;
                    }
                }
            }
        }
        best = wave_max_u64_rows(best);                   // all lanes are here: the loops above run the same number of times
        if (!(best >> 32)) break;
        const float top = __uint_as_float((uint32_t)(best >> 32));
        const uint32_t top_s = 0xFFFFFFFFu - (uint32_t)best;
        // cost and value of the chosen amount: from its lane's registers when it is among the first 64
        unsigned long long top_cost;
        float top_val;
        if (top_s < 64u) {
            const int src = __builtin_amdgcn_readfirstlane((int)top_s);
            top_cost = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(cost0 >> 32), src) << 32) |
                       (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)cost0, src);
            top_val = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(val0), src));
        } else {
            top_cost = cost_of(top_s);
            top_val = value_of(top_s);
        }
        prev = top < prev ? top : prev;
        if (lane == 0) {
            const size_t e = (size_t)k * H.stride + jrel;
            H.key[e] = __float_as_uint(prev);
            H.raw[e] = top;
            H.tgt[e] = (uint16_t)top_s;
            if (PASS == 0) {
                H.dg[e] = (uint32_t)(top_cost - cost_cur);
                H.dc[e] = cpu_cost(grid, c_fixed, (uint32_t)top_cost) - (cost_cur ? cpu_cost(grid, c_fixed, (uint32_t)cost_cur) : 0ull);
            } else {
                H.dg[e] = 0u;
                H.dc[e] = top_cost - cost_cur;
            }
        }
        cur = top_val;
        cur_i = (int32_t)top_s;
        cost_cur = top_cost;
        ++k;
    }
    for (uint32_t kk = k + lane; kk < H.width; kk += 64) H.key[(size_t)kk * H.stride + jrel] = 0u;   // unused positions
    if (PASS == 1 && k > 0 && lane == 0) st.cpu_steps[rnd] = 1u;
}

// The same walks with several jobs per wavefront, for calls in which no job has
// more than LANES amounts (LANES = 16 or 32): a job takes LANES neighbouring
// lanes, the wavefront loops until the last of its jobs has finished, and a
// job's maximum is taken over its own lanes only.
template <int LANES>
__device__ __forceinline__ unsigned long long group_max_u64(unsigned long long v, uint32_t lane) {
    unsigned long long o;
    o = dpp_u64<0xB1>(v);  v = o > v ? o : v;                   // quad_perm [1,0,3,2]
    o = dpp_u64<0x4E>(v);  v = o > v ? o : v;                   // quad_perm [2,3,0,1]
    o = dpp_u64<0x141>(v); v = o > v ? o : v;                   // row_half_mirror
    o = dpp_u64<0x140>(v); v = o > v ? o : v;                   // row_mirror: every row of 16 lanes holds its maximum
    if (LANES == 16) return v;
    unsigned long long row[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
        row[r] = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), 16 * r) << 32) |
                 (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 16 * r);
    const unsigned long long lo = row[0] > row[1] ? row[0] : row[1], hi = row[2] > row[3] ? row[2] : row[3];
    return lane < 32 ? lo : hi;
}

template <int PASS, int LANES>
__global__ __launch_bounds__(HULL_THREADS) void k_hull_groups(Ctx X, JobState st, HullBuf H, Hist zero, size_t zero_bins) {
    for (size_t i = (size_t)blockIdx.x * HULL_THREADS + threadIdx.x; i < zero_bins; i += (size_t)gridDim.x * HULL_THREADS) {
        zero.g[i] = 0u;
        zero.c[i] = 0ull;
        if (i < X.R.n_rounds) st.cpu_steps[i] = 0u;
    }
    constexpr uint32_t PER_WAVE = 64 / LANES;
    const uint32_t lane = threadIdx.x & 63u, sub = lane % LANES, group_base = lane - sub;
    const uint32_t slot = (blockIdx.x * (HULL_THREADS / 64) + (threadIdx.x >> 6)) * PER_WAVE + lane / LANES;
    const bool valid = slot < H.stride;                    // lanes of a slot past the end stay for the shuffles
    const uint32_t jrel = valid ? slot : H.stride - 1;
    const uint32_t j = X.jb + jrel;
    const uint32_t rnd = round_index_of(X.R, j);
    uint32_t rj0, rj1;
    rk_cluster cl;
    round_of(X.R, rnd, rj0, rj1, cl);
    const GridDev &grid = X.grid;
    const float *__restrict__ vals = PASS == 0 ? X.curve_thr : X.best_thr;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    const uint32_t ju = job_of(X, j);
    const uint32_t s0 = X.tb.seg_off[ju], ns = X.tb.seg_off[ju + 1] - s0;
    const uint64_t jbase = (uint64_t)n_rows * (s0 - X.tb.seg_off[X.jb]);
    const float ref = X.ref_thr[ju];

    uint32_t npts, g_fixed = 0, c_fixed = 0;
    int32_t cur_i;
    unsigned long long cost_cur, cap_c, cap_g = 0;
    float cur;
    int32_t gi = -1;
    if (PASS == 0) {
        const Floor fl = floor_of(st, jrel);
        unsigned long long startG, startC;
        pass_caps<0>(X.R, cl, st, rnd, startG, startC);
        c_fixed = fl.ci;
        npts = fl.state != RK_JOB_NORMAL ? 0u : ns;
        cur_i = fl.gi;
        cost_cur = fl.gi < 0 ? 0ull : (unsigned long long)X.tb.seg_g[s0 + fl.gi];
        cur = fl.gi < 0 ? 0.f : vals[jbase + (uint64_t)(c_fixed * n_mem + n_mem - 1) * ns + fl.gi];
        cap_g = startG + cost_cur;                       // the floor is already paid for
        cap_c = startC + (fl.gi < 0 ? 0ull : cpu_cost(grid, c_fixed, (uint32_t)cost_cur));
    } else {
        gi = st.gi[jrel];
        npts = (gi < 0 || (st.waits && st.waits[jrel] != RK_JOB_NORMAL)) ? 0u : grid.n_cpu;
        g_fixed = gi < 0 ? 0u : st.g[jrel];
        cur_i = (int32_t)st.ci[jrel];
        cost_cur = cpu_cost(grid, (uint32_t)cur_i, g_fixed);
        cap_c = st.free_c[rnd] + cost_cur;               // the level held is already paid for
        cur = gi < 0 ? 0.f : vals[jbase + (uint64_t)((uint32_t)cur_i * n_mem + n_mem - 1) * ns + gi];
    }
    if (!valid) npts = 0;
    // the lane's amount: cost in the pass's resource, value, and whether the round could ever afford it
    unsigned long long cost0 = 0;
    float val0 = 0.f;
    bool can = false;
    if (sub < npts) {
        cost0 = PASS == 0 ? (unsigned long long)X.tb.seg_g[s0 + sub] : cpu_cost(grid, sub, g_fixed);
        val0 = PASS == 0 ? vals[jbase + (uint64_t)(c_fixed * n_mem + n_mem - 1) * ns + sub]
                         : vals[jbase + (uint64_t)(sub * n_mem + n_mem - 1) * ns + gi];
        can = PASS == 0 ? (cost0 <= cap_g && cpu_cost(grid, c_fixed, (uint32_t)cost0) <= cap_c) : cost0 <= cap_c;
    }

    uint32_t k = 0;
    float prev = __uint_as_float(0x7F800000u);
    bool walking = npts > 0;                               // the same in all lanes of a job
    while (__ballot(walking && k < H.width)) {             // until the wavefront's last job has finished
        unsigned long long best = 0;
        if (walking && k < H.width && can && (int32_t)sub > cur_i && val0 > cur) {
            float sl = (val0 - cur) / ref;
            sl = sl / (float)(cost0 - cost_cur);
            best = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - sub);
        }
        best = group_max_u64<LANES>(best, lane);
        const bool step = walking && k < H.width && (best >> 32) != 0;
        const float top = __uint_as_float((uint32_t)(best >> 32));
        const uint32_t top_s = step ? 0xFFFFFFFFu - (uint32_t)best : 0u;
        const int src = (int)(group_base + top_s);        // the lane that holds the chosen amount
        const unsigned long long top_cost = ((unsigned long long)(uint32_t)__shfl((int)(uint32_t)(cost0 >> 32), src, 64) << 32) |
                                            (uint32_t)__shfl((int)(uint32_t)cost0, src, 64);
        const float top_val = __shfl(val0, src, 64);
        if (step) {
            prev = top < prev ? top : prev;
            if (sub == 0) {
                const size_t e = (size_t)k * H.stride + jrel;
                H.key[e] = __float_as_uint(prev);
                H.raw[e] = top;
                H.tgt[e] = (uint16_t)top_s;
                if (PASS == 0) {
                    H.dg[e] = (uint32_t)(top_cost - cost_cur);
                    H.dc[e] = cpu_cost(grid, c_fixed, (uint32_t)top_cost) - (cost_cur ? cpu_cost(grid, c_fixed, (uint32_t)cost_cur) : 0ull);
                } else {
                    H.dg[e] = 0u;
                    H.dc[e] = top_cost - cost_cur;
                }
            }
            cur = top_val;
            cur_i = (int32_t)top_s;
            cost_cur = top_cost;
            ++k;
        } else {
            walking = false;
        }
    }
    if (valid) {
        for (uint32_t kk = k + sub; kk < H.width; kk += LANES) H.key[(size_t)kk * H.stride + jrel] = 0u;   // unused positions
        if (PASS == 1 && k > 0 && sub == 0) st.cpu_steps[rnd] = 1u;
    }
}

// ------------------------------------------------------------------ threshold search
// Highest bin whose steps, added to everything above it, no longer fit.
// bin = -1: all bins fit.  base*: cost of the bins above `bin`.
struct Cut { int32_t bin; unsigned long long baseG, baseC; };

struct CutScratch {
    unsigned long long wave_g[JOB_THREADS / 64], wave_c[JOB_THREADS / 64];   // totals of the wavefronts
    unsigned long long mask[JOB_THREADS / 64];                               // lanes that found a failing bin
    int32_t cand[JOB_THREADS];
    unsigned long long candG[JOB_THREADS], candC[JOB_THREADS];
};

// Workgroup-wide: the first JOB_THREADS threads do the work (thread t owns the
// bins BINS-1-16t downwards), every thread of the workgroup must call it
// (barriers) and gets the result.
__device__ Cut find_cut(const uint32_t *__restrict__ hG, const unsigned long long *__restrict__ hC,
                        unsigned long long baseG, unsigned long long baseC, unsigned long long capG,
                        unsigned long long capC, CutScratch &S) {
    constexpr uint32_t PER = BINS / JOB_THREADS, NW = JOB_THREADS / 64;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const bool part = tid < JOB_THREADS;
    const uint32_t top = BINS - 1 - (part ? tid : 0u) * PER;
    uint32_t vg[PER];
    unsigned long long vc[PER];
    unsigned long long sg = 0, sc = 0;
#pragma unroll
    for (uint32_t i = 0; i < PER; ++i) {
        vg[i] = part ? hG[top - i] : 0u;
        vc[i] = part ? hC[top - i] : 0ull;
        sg += vg[i]; sc += vc[i];
    }
    // inclusive scan over the threads: inside the wavefront by shuffles, then the wavefronts' totals
    unsigned long long ig = sg, ic = sc;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long ag = __shfl_up(ig, off, 64), ac = __shfl_up(ic, off, 64);
        if ((int)lane >= off) { ig += ag; ic += ac; }
    }
    if (part && lane == 63u) { S.wave_g[tid >> 6] = ig; S.wave_c[tid >> 6] = ic; }
    __syncthreads();
    unsigned long long allG = 0, allC = 0, beforeG = 0, beforeC = 0;
#pragma unroll
    for (uint32_t w = 0; w < NW; ++w) {
        if (w < (tid >> 6)) { beforeG += S.wave_g[w]; beforeC += S.wave_c[w]; }
        allG += S.wave_g[w]; allC += S.wave_c[w];
    }
    unsigned long long cg = baseG + beforeG + ig - sg, cc = baseC + beforeC + ic - sc;   // everything above this thread's bins
    int32_t cand = -1;
#pragma unroll
    for (uint32_t i = 0; i < PER; ++i) {
        if (cand < 0) {
            if (cg + vg[i] > capG || cc + vc[i] > capC) cand = (int32_t)(top - i);
            else { cg += vg[i]; cc += vc[i]; }
        }
    }
    const unsigned long long found = __ballot(part && cand >= 0);
    if (part) {
        if (cand >= 0) { S.cand[tid] = cand; S.candG[tid] = cg; S.candC[tid] = cc; }
        if (lane == 0) S.mask[tid >> 6] = found;
    }
    __syncthreads();
    Cut out;
    out.bin = -1;
    out.baseG = baseG + allG;
    out.baseC = baseC + allC;
    int32_t first = -1;                                   // the first thread (highest bins) with a failing bin
#pragma unroll
    for (uint32_t w = 0; w < NW; ++w) {
        const unsigned long long m = S.mask[w];
        if (first < 0 && m) first = (int32_t)(w * 64 + (uint32_t)__ffsll((long long)m) - 1u);
    }
    if (first >= 0) { out.bin = S.cand[first]; out.baseG = S.candG[first]; out.baseC = S.candC[first]; }
    __syncthreads();
    return out;
}

template <int PASS>
__device__ __forceinline__ uint32_t walk_width(const Ctx &X, const HullBuf &H) {
    return PASS == 0 ? H.width : (X.grid.n_cpu - 1 < H.width ? X.grid.n_cpu - 1 : H.width);
}

// Adds the steps of one job's walk to a histogram in LDS.  The walk is read
// four steps at a time (all twelve loads go out together; positions past the
// walk's end are inside the buffers and ignored).
template <int PASS, int LEVEL>
__device__ __forceinline__ void hist_add(const Ctx &X, const HullBuf &H, uint32_t jrel, int32_t want_top, uint32_t *lg,
                                         unsigned long long *lc) {
    const uint32_t width = walk_width<PASS>(X, H);
    for (uint32_t k0 = 0; k0 < width; k0 += 4) {
        uint32_t key[4], dg[4];
        unsigned long long dc[4];
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
            const uint32_t k = k0 + u < width ? k0 + u : width - 1;
            const size_t e = (size_t)k * H.stride + jrel;
            key[u] = H.key[e];
            dg[u] = PASS == 0 ? H.dg[e] : 0u;
            dc[u] = H.dc[e];
        }
#pragma unroll
        for (uint32_t u = 0; u < 4; ++u) {
            if (k0 + u >= width || !key[u]) return;
            uint32_t bin;
            if (LEVEL == 0) bin = key[u] >> 20;
            else {
                if ((int32_t)(key[u] >> 20) > want_top) continue;
                if ((int32_t)(key[u] >> 20) < want_top) return;   // keys only decrease along a walk
                bin = (key[u] >> 8) & (BINS - 1);
            }
            if (dg[u]) atomicAdd(&lg[bin], dg[u]);
            if (dc[u]) atomicAdd(&lc[bin], dc[u]);
        }
    }
}

// Cost histogram of one level.  Level 0: bin = key bits 31..20 of every step.
// Level 1: key bits 19..8 of the steps inside the bin where level 0 was cut.
template <int PASS, int LEVEL>
__global__ __launch_bounds__(JOB_THREADS) void k_hist(Ctx X, JobState st, HullBuf H, Hist hist) {
    __shared__ uint32_t lg[BINS];
    __shared__ unsigned long long lc[BINS];
    __shared__ CutScratch cs;
    const uint32_t rnd = blockIdx.y, tid = threadIdx.x;
    if (PASS == 1 && st.cpu_steps[rnd] == 0u) return;       // no job can use more CPUs: the whole pass is empty
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    int32_t want_top = 0;
    if (LEVEL == 1) {
        unsigned long long capG, capC;
        pass_caps<PASS>(X.R, cl, st, rnd, capG, capC);
        const size_t h0 = hist_at(rnd, PASS, 0);
        const Cut c0 = find_cut(hist.g + h0, hist.c + h0, 0, 0, capG, capC, cs);
        if (c0.bin < 0) return;                           // everything fits: no second level needed
        want_top = c0.bin;
    }
    for (uint32_t i = tid; i < BINS; i += JOB_THREADS) { lg[i] = 0; lc[i] = 0; }
    __syncthreads();
    const uint32_t jl = blockIdx.x * JOB_THREADS + tid;
    if (J0 + jl < J1) hist_add<PASS, LEVEL>(X, H, J0 + jl - X.jb, want_top, lg, lc);
    __syncthreads();
    const size_t h = hist_at(rnd, PASS, LEVEL);
    for (uint32_t i = tid; i < BINS; i += JOB_THREADS) {
        if (lg[i]) atomicAdd(&hist.g[h + i], lg[i]);
        if (lc[i]) atomicAdd(&hist.c[h + i], lc[i]);
    }
}

// ------------------------------------------------------------------ best step from scratch
struct Step { float slope; uint32_t tgt, dg; };

// Best step of job j from its current state under the free capacity.  The
// candidates are read four at a time, so that their loads (and those of the
// current state) are in flight together; positions past the end repeat the
// last one and are ignored.
template <int PASS>
__device__ __forceinline__ Step best_step(const Ctx &X, uint32_t j, int32_t gi, uint32_t g_held, uint32_t ci,
                                          unsigned long long freeG, unsigned long long freeC) {
    const GridDev &grid = X.grid;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem, m_top = n_mem - 1;
    const uint32_t ju = job_of(X, j);
    const uint32_t s0 = X.tb.seg_off[ju], ns = X.tb.seg_off[ju + 1] - s0;
    const uint64_t jbase = (uint64_t)n_rows * (s0 - X.tb.seg_off[X.jb]);
    const float ref = X.ref_thr[ju];
    Step out = {0.f, 0u, 0u};
    if (PASS == 0) {
        const uint64_t row = jbase + (uint64_t)(ci * n_mem + m_top) * ns;      // the CPU level the job holds
        const uint32_t g_cur = gi < 0 ? 0u : X.tb.seg_g[s0 + gi];
        const float cur = gi < 0 ? 0.f : X.curve_thr[row + gi];
        const unsigned long long c_cur = gi < 0 ? 0ull : cpu_cost(grid, ci, g_cur);
        for (uint32_t b = (uint32_t)(gi + 1); b < ns; b += 4) {
            uint32_t gs[4];
            float vs[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t s = b + u < ns ? b + u : ns - 1;
                gs[u] = X.tb.seg_g[s0 + s];
                vs[u] = X.curve_thr[row + s];
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t s = b + u;
                if (s >= ns) return out;
                const uint32_t dg = gs[u] - g_cur;
                if (dg > freeG) return out;                    // amounts ascend: nothing further on fits
                const float v = vs[u];
                if (!(v > cur)) continue;
                if (cpu_cost(grid, ci, g_cur + dg) - c_cur > freeC) continue;
                float sl = (v - cur) / ref;
                sl = sl / (float)dg;
                if (sl > out.slope) { out.slope = sl; out.tgt = s; out.dg = dg; }
            }
        }
    } else if (gi >= 0) {
        const float cur = X.best_thr[jbase + (uint64_t)(ci * n_mem + m_top) * ns + gi];
        const unsigned long long have = cpu_cost(grid, ci, g_held);
        for (uint32_t b = ci + 1; b < grid.n_cpu; b += 4) {
            float vs[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t c = b + u < grid.n_cpu ? b + u : grid.n_cpu - 1;
                vs[u] = X.best_thr[jbase + (uint64_t)(c * n_mem + m_top) * ns + gi];
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t c = b + u;
                if (c >= grid.n_cpu) return out;
                const unsigned long long dc = cpu_cost(grid, c, g_held) - have;
                if (dc > freeC) return out;                    // levels ascend
                const float v = vs[u];
                if (!(v > cur)) continue;
                float sl = (v - cur) / ref;
                sl = sl / (float)dc;
                if (sl > out.slope) { out.slope = sl; out.tgt = c; }
            }
        }
    }
    return out;
}

// ------------------------------------------------------------------ apply the selected prefix
// The threshold from the two histogram levels: steps with (key >> 8) > thr24
// are applied; freeG / freeC = what is left after them.  Workgroup-wide.
struct Selection { long long thr24; unsigned long long freeG, freeC; };

__device__ Selection select_threshold(const uint32_t *h0g, const unsigned long long *h0c, const uint32_t *h1g,
                                      const unsigned long long *h1c, unsigned long long capG, unsigned long long capC,
                                      CutScratch &cs) {
    const Cut c0 = find_cut(h0g, h0c, 0, 0, capG, capC, cs);
    Selection sel;
    sel.thr24 = -1;
    unsigned long long usedG = c0.baseG, usedC = c0.baseC;
    if (c0.bin >= 0) {
        const Cut c1 = find_cut(h1g, h1c, c0.baseG, c0.baseC, capG, capC, cs);
        sel.thr24 = ((long long)c0.bin << 12) + (long long)c1.bin;   // c1.bin = -1: the whole of c0.bin fits as well
        usedG = c1.baseG; usedC = c1.baseC;
    }
    sel.freeG = capG - usedG;
    sel.freeC = capC - usedC;
    return sel;
}

// Applies the selected prefix (steps with key >> 8 above thr24) to job j and
// caches its best next step under what is left.
template <int PASS>
__device__ __forceinline__ void apply_job(const Ctx &X, const JobState &st, const HullBuf &H, uint32_t j, long long thr24,
                                          unsigned long long freeG, unsigned long long freeC) {
    {
        const uint32_t jrel = j - X.jb;
        const uint32_t width = walk_width<PASS>(X, H);
        const Floor fl = PASS == 0 ? floor_of(st, jrel) : Floor{-1, 0u, RK_JOB_NORMAL};
        int32_t gi = PASS == 0 ? fl.gi : st.gi[jrel];
        uint32_t g_held = PASS == 0 ? 0u : st.g[jrel];
        uint32_t ci = PASS == 0 ? fl.ci : st.ci[jrel];
        uint32_t k = 0, key = 0;
        size_t e = 0;
        bool open_end = true;                                      // no step left out so far
        for (uint32_t k0 = 0; k0 < width && open_end; k0 += 4) {   // four steps per round of loads
            uint32_t keys[4], tgts[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t kk = k0 + u < width ? k0 + u : width - 1;
                keys[u] = H.key[(size_t)kk * H.stride + jrel];
                tgts[u] = H.tgt[(size_t)kk * H.stride + jrel];
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                if (!open_end || k0 + u >= width) continue;
                k = k0 + u;
                e = (size_t)k * H.stride + jrel;
                key = keys[u];
                if (!key || (long long)(key >> 8) <= thr24) { open_end = false; continue; }
                if (PASS == 0) gi = (int32_t)tgts[u]; else ci = tgts[u];
                k = k0 + u + 1;
            }
        }
        if (k == width) key = 0;
        if (PASS == 0) {
            g_held = gi < 0 ? 0u : X.tb.seg_g[X.tb.seg_off[job_of(X, j)] + gi];
            st.gi[jrel] = gi;
            st.g[jrel] = g_held;
        }
        st.ci[jrel] = ci;
        // the job's best next step: the walk's next step if it still fits, else a fresh search
        Step nx = {0.f, 0u, 0u};
        if (key) {
            if (H.dg[e] <= freeG && H.dc[e] <= freeC) { nx.slope = H.raw[e]; nx.tgt = H.tgt[e]; nx.dg = H.dg[e]; }
            else nx = best_step<PASS>(X, j, gi, g_held, ci, freeG, freeC);
        }
        st.step_slope[jrel] = nx.slope;
        st.step_tgt[jrel] = (uint16_t)nx.tgt;
        st.step_dg[jrel] = (uint16_t)nx.dg;
    }
}

// One thread per job.  Every workgroup derives the threshold from the two
// histogram levels (same inputs, same result in all of them).
template <int PASS>
__global__ __launch_bounds__(JOB_THREADS) void k_apply(Ctx X, JobState st, HullBuf H, Hist hist) {
    __shared__ CutScratch cs;
    const uint32_t rnd = blockIdx.y, tid = threadIdx.x;
    if (PASS == 1 && st.cpu_steps[rnd] == 0u) return;       // empty pass: every job keeps the CPU level it has
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    unsigned long long capG, capC;
    pass_caps<PASS>(X.R, cl, st, rnd, capG, capC);
    const size_t h0 = hist_at(rnd, PASS, 0), h1 = hist_at(rnd, PASS, 1);
    const Selection sel = select_threshold(hist.g + h0, hist.c + h0, hist.g + h1, hist.c + h1, capG, capC, cs);

    const uint32_t jl = blockIdx.x * JOB_THREADS + tid;
    if (J0 + jl < J1) apply_job<PASS>(X, st, H, J0 + jl, sel.thr24, sel.freeG, sel.freeC);
    // the capacity left goes to the tail through a second pair of words: the
    // pass's starting capacity (free_c) is still being read by other workgroups
    if (blockIdx.x == 0 && tid == 0) { st.free_g[rnd] = sel.freeG; st.free_g[X.R.n_rounds + rnd] = sel.freeC; }
}

// ------------------------------------------------------------------ step by step on what is left
// The same search as best_step, by a whole wavefront: every lane passes the
// same arguments and gets the same result.  Lanes take one candidate target
// each, so the loads of a job's amounts and values go out together instead of
// one after the other.
template <int PASS>
__device__ __forceinline__ Step best_step_wave(const Ctx &X, uint32_t j, int32_t gi, uint32_t g_held, uint32_t ci,
                                               unsigned long long freeG, unsigned long long freeC) {
    const GridDev &grid = X.grid;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem, m_top = n_mem - 1;
    const uint32_t ju = job_of(X, j);
    const uint32_t s0 = X.tb.seg_off[ju], ns = X.tb.seg_off[ju + 1] - s0;
    const uint64_t jbase = (uint64_t)n_rows * (s0 - X.tb.seg_off[X.jb]);
    const float ref = X.ref_thr[ju];
    unsigned long long mine = 0;                                // (slope bits, inverted target): lowest target wins ties
    uint32_t mine_dg = 0;
    if (PASS == 0) {
        const uint32_t g_cur = gi < 0 ? 0u : X.tb.seg_g[s0 + gi];
        const uint64_t row = jbase + (uint64_t)(ci * n_mem + m_top) * ns;
        const float cur = gi < 0 ? 0.f : X.curve_thr[row + gi];
        const unsigned long long c_cur = gi < 0 ? 0ull : cpu_cost(grid, ci, g_cur);
        for (uint32_t b = (uint32_t)(gi + 1); b < ns; b += 64) {
            const uint32_t s = b + lane;
            const bool in = s < ns;
            uint32_t dg = 0;
            float v = 0.f;
            if (in) { dg = X.tb.seg_g[s0 + s] - g_cur; v = X.curve_thr[row + s]; }
            const bool fits = in && dg <= freeG;
            if (fits && v > cur && cpu_cost(grid, ci, g_cur + dg) - c_cur <= freeC) {
                float sl = (v - cur) / ref;
                sl = sl / (float)dg;
                const unsigned long long key = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - s);
                if (key > mine) { mine = key; mine_dg = dg; }
            }
            if (__ballot(in && !fits)) break;                   // amounts ascend: nothing further on fits
        }
    } else if (gi >= 0) {
        const float cur = X.best_thr[jbase + (uint64_t)(ci * n_mem + m_top) * ns + gi];
        const unsigned long long have = cpu_cost(grid, ci, g_held);
        for (uint32_t b = ci + 1; b < grid.n_cpu; b += 64) {
            const uint32_t c = b + lane;
            const bool in = c < grid.n_cpu;
            unsigned long long dc = 0;
            float v = 0.f;
            if (in) {
                dc = cpu_cost(grid, c, g_held) - have;
                v = X.best_thr[jbase + (uint64_t)(c * n_mem + m_top) * ns + gi];
            }
            const bool fits = in && dc <= freeC;
            if (fits && v > cur) {
                float sl = (v - cur) / ref;
                sl = sl / (float)dc;
                const unsigned long long key = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - c);
                if (key > mine) mine = key;
            }
            if (__ballot(in && !fits)) break;                   // levels ascend
        }
    }
    const unsigned long long best = wave_max_u64_rows(mine);
    Step out = {0.f, 0u, 0u};
    if (best >> 32) {                                           // a positive slope
        out.slope = __uint_as_float((uint32_t)(best >> 32));
        out.tgt = 0xFFFFFFFFu - (uint32_t)best;
        if (PASS == 0) {
            const unsigned long long holder = __ballot(mine == best);   // one lane: keys differ in the target
            out.dg = (uint32_t)__builtin_amdgcn_readlane((int)mine_dg, __builtin_amdgcn_readfirstlane((int)__ffsll((long long)holder) - 1));
        }
    }
    return out;
}

// LDS words tail_run needs beside its per-job scratch: the two key maxima in
// three copies used in turn, the winner's two costs, and the CPU levels.
constexpr int TAIL_RED_WORDS = 3 * 2 + 2 + RK_MAX_CPU_LEVELS / 2;

// Workgroup of TAIL_THREADS threads; lds = max_jobs * 12 bytes of scratch, red =
// TAIL_RED_WORDS words; at most KMAX * TAIL_THREADS jobs.  Starts from the
// state k_apply / apply_job left in st.  Thread t owns jobs t, t +
// TAIL_THREADS, ...: their cached steps stay in its registers, and only it
// (and, for the winner's new search, its wavefront) touches their LDS entries,
// so a step needs two barriers: one for the maxima, one for the winner's costs.
template <int PASS, int KMAX>
__device__ __forceinline__ void tail_run(const Ctx &X, const JobState &st, uint32_t rnd, uint32_t J0, uint32_t J1,
                                         unsigned long long freeG, unsigned long long freeC, uint32_t max_jobs,
                                         float *lds, unsigned long long *red) {
    uint16_t *tgt = reinterpret_cast<uint16_t *>(lds);             // target of the cached step (segment index or CPU level)
    int16_t *gi = reinterpret_cast<int16_t *>(tgt + max_jobs);     // granted segment index, -1 = none
    uint16_t *ci = reinterpret_cast<uint16_t *>(gi + max_jobs);    // granted CPU level
    uint16_t *gh = ci + max_jobs;                                  // GPUs held (CPU pass); GPUs of a new step (GPU pass)
    float *found = reinterpret_cast<float *>(gh + max_jobs);       // slope of a new step on its way to the registers
    unsigned long long *win = red + 6;                             // GPUs and CPUs the winning step costs
    uint32_t *lvl = reinterpret_cast<uint32_t *>(red + 8);         // CPU levels, for indexing by lane

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t nj = J1 - J0, jrel0 = J0 - X.jb;
    const GridDev &grid = X.grid;

    // CPUs a step costs (saturated to 32 bits: the free CPUs fit in 32)
    auto need_cpus = [&](int32_t g_i, uint32_t c_i, uint32_t target, uint32_t gpus) -> uint32_t {
        unsigned long long c;
        if (PASS == 0) {
            const unsigned long long times = grid.cpu_mode ? gpus : (g_i < 0 ? 1u : 0u);
            c = (unsigned long long)lvl[c_i] * times;
        } else {
            const unsigned long long times = grid.cpu_mode ? gpus : 1u;
            c = (unsigned long long)lvl[target] * times - (unsigned long long)lvl[c_i] * times;
        }
        return c > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)c;
    };

    if (nj == 0) {                                                 // the same in all threads
        if (PASS == 0 && tid == 0) st.free_c[rnd] = freeC;
        return;
    }
    if (tid < RK_MAX_CPU_LEVELS) lvl[tid] = grid.cpu_levels[tid];
    if (tid < 6) red[tid] = 0ull;
    float slope[KMAX];                                             // cached best step of the thread's jobs:
    uint32_t dg[KMAX], dc[KMAX];                                   // > 0 exact, < 0 an upper bound, 0 none; its GPUs, CPUs
    {
        int32_t g_i[KMAX];
        uint32_t c_i[KMAX], target[KMAX], gpus[KMAX];
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {                           // all loads go out before the first is used
            const uint32_t jl = tid + (uint32_t)k * TAIL_THREADS;
            const uint32_t at = jrel0 + (jl < nj ? jl : nj - 1u);
            g_i[k] = st.gi[at];
            c_i[k] = st.ci[at];
            target[k] = st.step_tgt[at];
            gpus[k] = PASS == 0 ? st.step_dg[at] : st.g[at];
            slope[k] = st.step_slope[at];
        }
        __syncthreads();                                           // the levels are in LDS
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const uint32_t jl = tid + (uint32_t)k * TAIL_THREADS;
            const bool have = jl < nj;
            const uint32_t need = need_cpus(g_i[k], c_i[k], target[k], gpus[k]);
            slope[k] = have ? slope[k] : 0.f;
            dg[k] = PASS == 0 && have ? gpus[k] : 0u;
            dc[k] = have ? need : 0u;
            if (have) {
                tgt[jl] = (uint16_t)target[k];
                gi[jl] = (int16_t)g_i[k];
                ci[jl] = (uint16_t)c_i[k];
                if (PASS == 1) gh[jl] = (uint16_t)gpus[k];
            }
        }
    }

    // A cached step that stops fitting is not searched anew at once: it is
    // kept, negated, as an upper bound of whatever the job can still do (the
    // job's state is unchanged and the capacity only shrank).  A step is
    // taken when the best exact entry beats every such bound under the tie
    // rule (lower job index first); bounds that could win are made exact
    // first, all of them in one go.
    auto key_of = [](float v, uint32_t jl) -> unsigned long long {
        return ((unsigned long long)__float_as_uint(v) << 32) | (0xFFFFFFFFu - jl);
    };
    uint32_t turn = 0, moved = 0;                               // moved: bit k = the thread's k-th job took a step here
    for (;;) {
        if (PASS == 0 ? freeG == 0 : freeC == 0) break;         // nothing can fit any more
        // the thread's best exact step and best bound: plain float compares (its jobs come in rising order, so the
        // first of equal slopes is the lower job), the two keys are built once at the end
        const uint32_t roomG = freeG > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)freeG;
        const uint32_t roomC = freeC > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)freeC;
        float vf = 0.f, vs = 0.f;
        uint32_t jf = 0, js = 0;
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const uint32_t jl = tid + (uint32_t)k * TAIL_THREADS;
            float v = slope[k];
            const bool stopped = v > 0.f && ((PASS == 0 && dg[k] > roomG) || dc[k] > roomC);
            v = stopped ? -v : v;
            slope[k] = v;
            if (v > vf) { vf = v; jf = jl; }
            if (-v > vs) { vs = -v; js = jl; }
        }
        unsigned long long kf = vf > 0.f ? key_of(vf, jf) : 0ull, ks = vs > 0.f ? key_of(vs, js) : 0ull;
        kf = wave_max_u64_rows(kf);
        ks = wave_max_u64_rows(ks);
        unsigned long long *both = red + 2 * turn;              // three copies in turn: the next one is cleared meanwhile
        turn = turn == 2 ? 0u : turn + 1u;
        if (lane == 0) {
            if (kf) atomicMax(&both[0], kf);
            if (ks) atomicMax(&both[1], ks);
        }
        if (tid == TAIL_THREADS - 1) { red[2 * turn] = 0ull; red[2 * turn + 1] = 0ull; }
        __syncthreads();
        kf = both[0];
        ks = both[1];
        if (ks > kf) {                                          // a bound could still win: make those exact
            uint32_t todo = 0;
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const float v = slope[k];
                if (v < 0.f && key_of(-v, tid + (uint32_t)k * TAIL_THREADS) > kf) todo |= 1u << k;
            }
            // the searches go through LDS so that the register arrays are only ever indexed by constants
            for (uint32_t rest = todo; rest; rest &= rest - 1u) {
                const uint32_t jl = tid + ((uint32_t)__ffs((int)rest) - 1u) * TAIL_THREADS;
                const Step nx = best_step<PASS>(X, J0 + jl, gi[jl], PASS == 0 ? 0u : gh[jl], ci[jl], freeG, freeC);
                found[jl] = nx.slope;
                tgt[jl] = (uint16_t)nx.tgt;
                if (PASS == 0) gh[jl] = (uint16_t)nx.dg;
            }
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                if (todo >> k & 1u) {
                    const uint32_t jl = tid + (uint32_t)k * TAIL_THREADS;
                    slope[k] = found[jl];
                    if (PASS == 0) dg[k] = gh[jl];
                    dc[k] = need_cpus(gi[jl], ci[jl], tgt[jl], gh[jl]);
                }
            }
            continue;
        }
        if (!(kf >> 32)) break;                                 // no positive slope left
        const uint32_t jw = 0xFFFFFFFFu - (uint32_t)kf;
        const uint32_t owner = jw % TAIL_THREADS;
        const uint32_t kw = (uint32_t)__builtin_amdgcn_readfirstlane((int)(jw / TAIL_THREADS));   // same in all lanes
        if (tid == owner) {
            uint32_t a = 0, b = 0;
#pragma unroll
            for (int k = 0; k < KMAX; ++k) if ((uint32_t)k == kw) { a = dg[k]; b = dc[k]; }
            win[0] = a;
            win[1] = b;
        }
        __syncthreads();
        if (PASS == 0) freeG -= win[0];
        freeC -= win[1];
        if (wave == owner / 64u) {                              // the owner's wavefront searches the winner's next step
            int32_t g_i = gi[jw];
            uint32_t c_i = ci[jw];
            if (PASS == 0) g_i = (int32_t)tgt[jw]; else c_i = tgt[jw];
            const uint32_t held = PASS == 0 ? 0u : gh[jw];
            const Step nx = best_step_wave<PASS>(X, J0 + jw, g_i, held, c_i, freeG, freeC);
            if (tid == owner) {
                if (PASS == 0) gi[jw] = (int16_t)g_i; else ci[jw] = (uint16_t)c_i;
                moved |= 1u << kw;
                tgt[jw] = (uint16_t)nx.tgt;
                const uint32_t need = need_cpus(g_i, c_i, nx.tgt, PASS == 0 ? nx.dg : held);
#pragma unroll
                for (int k = 0; k < KMAX; ++k)
                    if ((uint32_t)k == kw) { slope[k] = nx.slope; dg[k] = PASS == 0 ? nx.dg : 0u; dc[k] = need; }
            }
        }
    }
    for (; moved; moved &= moved - 1u) {                        // only the jobs that took a step here changed since k_apply
        const uint32_t jl = tid + ((uint32_t)__ffs((int)moved) - 1u) * TAIL_THREADS;
        if (PASS == 0) {
            const int32_t s_i = gi[jl];
            st.gi[jrel0 + jl] = s_i;
            st.g[jrel0 + jl] = s_i < 0 ? 0u : X.tb.seg_g[X.tb.seg_off[job_of(X, J0 + jl)] + s_i];
        } else {
            st.ci[jrel0 + jl] = ci[jl];
        }
    }
    if (PASS == 0 && tid == 0) st.free_c[rnd] = freeC;          // what the CPU pass starts from
}

constexpr int TAIL_KMAX = (RK_MAX_JOBS_PER_ROUND + TAIL_THREADS - 1) / TAIL_THREADS;

template <int PASS>
__global__ __launch_bounds__(TAIL_THREADS) void k_tail(Ctx X, uint32_t max_jobs, JobState st) {
    extern __shared__ float lds_dyn[];
    __shared__ unsigned long long red[TAIL_RED_WORDS];
    const uint32_t rnd = blockIdx.x;
    if (PASS == 1 && st.cpu_steps[rnd] == 0u) return;       // empty pass
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    tail_run<PASS, TAIL_KMAX>(X, st, rnd, J0, J1, st.free_g[rnd], st.free_g[X.R.n_rounds + rnd], max_jobs, lds_dyn, red);
}

// ------------------------------------------------------------------ selection of a pass in one workgroup
// For rounds of at most SMALL_ROUND_JOBS jobs the histograms, the threshold,
// the application and the step-by-step tail of a pass run in one workgroup per
// round, with the histograms in LDS: one launch instead of six (KMAX = jobs per
// thread = 2).  The workgroup of the CPU pass also takes the memory step that
// ends the round.  Larger rounds use the same kernel for their CPU pass
// (KMAX = TAIL_KMAX, without the memory step) as long as all CPU walks together
// are short, which the host can tell from the grid:
// (CPU levels - 1) * jobs <= CPU_ONE_WG_STEPS.
// The histogram (48 KiB) and the tail's scratch (12 bytes per job) share the
// dynamic LDS: the tail starts when the threshold is known.
constexpr uint32_t SMALL_ROUND_JOBS = 2048;
constexpr uint64_t CPU_ONE_WG_STEPS = 65536;
constexpr size_t SELECT_HIST_BYTES = (size_t)BINS * 12;

__device__ __forceinline__ void mem_wish_job(const Ctx &X, const JobState &st, uint32_t j, rk_assign *__restrict__ assign,
                                             double &cost_d, double &val_d);
__device__ void mem_close_round(const Ctx &X, const JobState &st, uint32_t rnd, double wish, double val,
                                rk_assign *__restrict__ assign, float *__restrict__ totals);

template <int PASS, int KMAX>
__global__ __launch_bounds__(TAIL_THREADS) void k_select_small(Ctx X, uint32_t max_jobs, JobState st, HullBuf H,
                                                              rk_assign *__restrict__ assign, float *__restrict__ totals) {
    extern __shared__ unsigned long long lds_sel[];             // the histogram, then the tail's scratch
    unsigned long long *hc = lds_sel;                           // one histogram, used for level 0 and then level 1
    uint32_t *hg = reinterpret_cast<uint32_t *>(hc + BINS);
    __shared__ CutScratch cs;
    __shared__ unsigned long long red[TAIL_RED_WORDS];
    __shared__ double sums[2 * (TAIL_THREADS / 64)];
    const uint32_t rnd = blockIdx.x, tid = threadIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    const uint32_t nj = J1 - J0;
    // a large round knows whether any job's CPU walk has a step at all (same in all threads)
    const bool empty_pass = PASS == 1 && KMAX == TAIL_KMAX && st.cpu_steps[rnd] == 0u;
    if (!empty_pass) {
        unsigned long long capG, capC;
        pass_caps<PASS>(X.R, cl, st, rnd, capG, capC);
        for (uint32_t i = tid; i < BINS; i += TAIL_THREADS) { hg[i] = 0; hc[i] = 0; }
        __syncthreads();
        for (uint32_t jl = tid; jl < nj; jl += TAIL_THREADS) hist_add<PASS, 0>(X, H, J0 + jl - X.jb, 0, hg, hc);
        __syncthreads();
        const Cut c0 = find_cut(hg, hc, 0, 0, capG, capC, cs);
        Selection sel;
        sel.thr24 = -1;
        unsigned long long usedG = c0.baseG, usedC = c0.baseC;
        if (c0.bin >= 0) {                                      // uniform over the workgroup
            for (uint32_t i = tid; i < BINS; i += TAIL_THREADS) { hg[i] = 0; hc[i] = 0; }
            __syncthreads();
            for (uint32_t jl = tid; jl < nj; jl += TAIL_THREADS) hist_add<PASS, 1>(X, H, J0 + jl - X.jb, c0.bin, hg, hc);
            __syncthreads();
            const Cut c1 = find_cut(hg, hc, c0.baseG, c0.baseC, capG, capC, cs);
            sel.thr24 = ((long long)c0.bin << 12) + (long long)c1.bin;
            usedG = c1.baseG; usedC = c1.baseC;
        }
        sel.freeG = capG - usedG;
        sel.freeC = capC - usedC;
        for (uint32_t jl = tid; jl < nj; jl += TAIL_THREADS) apply_job<PASS>(X, st, H, J0 + jl, sel.thr24, sel.freeG, sel.freeC);
        __syncthreads();                                        // the state in st is read back by the whole workgroup; the
                                                                // histogram's LDS passes to the tail
        tail_run<PASS, KMAX>(X, st, rnd, J0, J1, sel.freeG, sel.freeC, max_jobs, reinterpret_cast<float *>(lds_sel), red);
    }
    if (PASS == 0 || KMAX == TAIL_KMAX) return;                 // (large rounds: a thread per job does it faster, k_mem_wish)
    // memory: every thread writes the wishes of its jobs, the first wavefront closes the round
    __syncthreads();                                            // the granted amounts are in st
    double cost_d = 0.0, val_d = 0.0;
    for (uint32_t jl = tid; jl < nj; jl += TAIL_THREADS) mem_wish_job(X, st, J0 + jl, assign, cost_d, val_d);
    cost_d = wave_sum_f64(cost_d);
    val_d = wave_sum_f64(val_d);
    if ((tid & 63u) == 0) { sums[tid >> 6] = cost_d; sums[TAIL_THREADS / 64 + (tid >> 6)] = val_d; }
    __syncthreads();                                            // also: the wishes are stored before anything replaces them
    if (tid < 64u) {
        const bool has = tid < TAIL_THREADS / 64;
        const double wish = wave_sum_f64(has ? sums[tid] : 0.0), val = wave_sum_f64(has ? sums[TAIL_THREADS / 64 + tid] : 0.0);
        mem_close_round(X, st, rnd, wish, val, assign, totals);
    }
}

// ------------------------------------------------------------------ memory
// Wish of a job: the smallest tier that reaches its best throughput over all
// tiers.  The wishes are written as the result; they are kept when all of them
// together stay 1 % below the round's host memory (then every job finds its
// wish still free when its turn comes: the float32 running remainder of the
// in-order rule drifts by far less), otherwise the round is redone in job order.
// Large rounds: k_mem_wish (a thread per job) and k_mem_finish (a wavefront per
// round); small rounds: the workgroup of the CPU pass's selection does both.

// the wish of job j, written to its record; adds its cost and its normalised throughput to the two sums
__device__ __forceinline__ void mem_wish_job(const Ctx &X, const JobState &st, uint32_t j, rk_assign *__restrict__ assign,
                                             double &cost_d, double &val_d) {
    const GridDev &grid = X.grid;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    const uint32_t jrel = j - X.jb;
    rk_assign out = {0u, 0u, 0.f, RK_NO_PLAN, 0.f};
    const int32_t gi = st.gi[jrel];
    if (gi >= 0) {
        const uint32_t g = st.g[jrel], c_lvl = st.ci[jrel];
        const uint32_t ju = job_of(X, j);
        const uint32_t s0 = X.tb.seg_off[ju], ns = X.tb.seg_off[ju + 1] - s0;
        const uint64_t base = (uint64_t)n_rows * (s0 - X.tb.seg_off[X.jb]) + (uint64_t)(c_lvl * n_mem) * ns + gi;
        float bv = 0.f;
        uint32_t bm = 0;
        for (uint32_t m = 0; m < n_mem; ++m) {
            const float v = X.best_thr[base + (uint64_t)m * ns];
            if (v > bv) { bv = v; bm = m; }
        }
        if (bv > 0.f) {
            float cost = grid.mem_levels_gb[bm];
            if (grid.mem_mode) cost = cost * (float)g;
            out.g = g;
            out.c = (uint32_t)cpu_cost(grid, c_lvl, g);
            out.mem_gb = cost;
            out.plan = X.best_plan[base + (uint64_t)bm * ns];
            out.thr = bv;
            cost_d += (double)cost;
            val_d += (double)bv / (double)X.ref_thr[job_of(X, j)];
        }
    }
    assign[jrel] = out;
}

__global__ __launch_bounds__(JOB_THREADS) void k_mem_wish(Ctx X, JobState st, rk_assign *__restrict__ assign) {
    __shared__ double red[2][JOB_THREADS / 64];
    const uint32_t rnd = blockIdx.y, tid = threadIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    const uint32_t jl = blockIdx.x * JOB_THREADS + tid;
    double cost_d = 0.0, val_d = 0.0;
    if (J0 + jl < J1) mem_wish_job(X, st, J0 + jl, assign, cost_d, val_d);
    cost_d = wave_sum_f64(cost_d);
    val_d = wave_sum_f64(val_d);
    if ((tid & 63u) == 0) { red[0][tid >> 6] = cost_d; red[1][tid >> 6] = val_d; }
    __syncthreads();
    if (tid == 0) {
        double a = 0.0, b = 0.0;
        for (int w = 0; w < JOB_THREADS / 64; ++w) { a += red[0][w]; b += red[1][w]; }
        st.partial[((size_t)rnd * st.blocks_per_round + blockIdx.x) * 2 + 0] = a;
        st.partial[((size_t)rnd * st.blocks_per_round + blockIdx.x) * 2 + 1] = b;
    }
}

// One wavefront (threadIdx.x = lane) closes a round whose wishes sum to `wish` GiB and `val` normalised throughput.
__device__ void mem_close_round(const Ctx &X, const JobState &st, uint32_t rnd, double wish, double val,
                                rk_assign *__restrict__ assign, float *__restrict__ totals) {
    const uint32_t tid = threadIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    const GridDev &grid = X.grid;
    const uint32_t nj = J1 - J0, jrel0 = J0 - X.jb;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    if (wish <= 0.99 * (double)cl.host_mem_gb) {
        if (tid == 0) totals[rnd] = (float)val;
        return;
    }
    // in job order: lanes load a batch of 64 jobs, then take their decisions one after the other
    float freeM = cl.host_mem_gb;
    double sum = 0.0;
    for (uint32_t base = 0; base < nj; base += 64) {
        const uint32_t jl = base + tid;
        const bool have = jl < nj && st.gi[jrel0 + jl] >= 0;
        uint32_t g = 0, c_lvl = 0, ns = 0;
        uint64_t at0 = 0;
        unsigned long long choice = 0;      // 4 bits per prefix length: best tier among tiers 0..k
        uint32_t valid = 0;                 // bit k: that best throughput is positive
        float thr_m[RK_MAX_MEM_LEVELS];
#pragma unroll
        for (uint32_t m = 0; m < RK_MAX_MEM_LEVELS; ++m) thr_m[m] = 0.f;
        if (have) {
            const uint32_t j = J0 + jl;
            g = st.g[jrel0 + jl]; c_lvl = st.ci[jrel0 + jl];
            const uint32_t ju = job_of(X, j);
            const uint32_t s0 = X.tb.seg_off[ju];
            ns = X.tb.seg_off[ju + 1] - s0;
            at0 = (uint64_t)n_rows * (s0 - X.tb.seg_off[X.jb]) + (uint64_t)(c_lvl * n_mem) * ns + (uint32_t)st.gi[jrel0 + jl];
            float bv = 0.f;
            uint32_t bm = 0;
#pragma unroll
            for (uint32_t m = 0; m < RK_MAX_MEM_LEVELS; ++m) {
                if (m < n_mem) {
                    const float v = X.best_thr[at0 + (uint64_t)m * ns];
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
                    out.plan = X.best_plan[at0 + (uint64_t)bm * ns];
                    out.thr = v;
                    sum += (double)v / (double)X.ref_thr[job_of(X, J0 + jl)];
                }
            }
            spent = __shfl(spent, (int)turn, 64);
            freeM = freeM - spent;
        }
        if (jl < nj) assign[jrel0 + jl] = out;
    }
    sum = wave_sum_f64(sum);
    if (tid == 0) totals[rnd] = (float)sum;
}

// One wavefront per round.
__global__ __launch_bounds__(64) void k_mem_finish(Ctx X, JobState st, rk_assign *__restrict__ assign,
                                                   float *__restrict__ totals) {
    const uint32_t rnd = blockIdx.x, tid = threadIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    const uint32_t used_blocks = (J1 - J0 + JOB_THREADS - 1) / JOB_THREADS;
    double wish = 0.0, val = 0.0;
    for (uint32_t b = tid; b < used_blocks; b += 64) {
        wish += st.partial[((size_t)rnd * st.blocks_per_round + b) * 2 + 0];
        val += st.partial[((size_t)rnd * st.blocks_per_round + b) * 2 + 1];
    }
    wish = wave_sum_f64(wish);
    val = wave_sum_f64(val);
    mem_close_round(X, st, rnd, wish, val, assign, totals);
}

// ------------------------------------------------------------------ service-level floors
// One workgroup per round.  All threads first stage every job's demand in LDS
// (one word: GPUs, tenant, flags; one word: CPUs), so that the global-memory
// latency is paid once.  The first wavefront then takes the decisions in job
// order, 64 jobs at a time: demands that do not fit what is left right now can
// never fit later and drop out in parallel; the others are decided one after
// the other with wavefront-uniform arithmetic (the demand is broadcast from its
// lane, the quotas of tenant t live in lane t % 64, register t / 64, the free
// capacity in uniform registers).  All threads then write the floors.
constexpr int FLOOR_THREADS = 1024;
constexpr uint32_t FL_CAND = 1u << 24, FL_GUAR = 1u << 25, FL_GRANTED = 1u << 31;

__device__ __forceinline__ uint32_t lane_value(uint32_t v, uint32_t lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)lane);
}

__global__ __launch_bounds__(FLOOR_THREADS) void k_floors(Ctx X, JobState st, SlaDev S, uint32_t max_jobs) {
    extern __shared__ uint32_t lds_floor[];
    uint32_t *word = lds_floor;                 // GPUs (16 bits) | tenant (8 bits) | flags
    uint32_t *cpus = lds_floor + max_jobs;
    constexpr uint32_t QREGS = RK_MAX_TENANTS / 64;
    const uint32_t rnd = blockIdx.x, tid = threadIdx.x, lane = tid & 63u;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(X.R, rnd, J0, J1, cl);
    const GridDev &grid = X.grid;
    const uint32_t nj = J1 - J0;

    for (uint32_t jl = tid; jl < nj; jl += FLOOR_THREADS) {
        const uint32_t j = J0 + jl;
        uint32_t w = 0, c = 0;
        // loaded for every job, so that the loads do not wait for one another
        const bool guar = S.guaranteed[j] != 0;
        const int32_t ms = S.min_seg[j - X.jb];
        const uint32_t mc = S.min_c[j - X.jb], t = S.tenant[j];
        const uint32_t s0 = X.tb.seg_off[j], ns = X.tb.seg_off[j + 1] - s0;
        if (guar) {
            w = FL_GUAR;
            if (ms >= 0 && (uint32_t)ms < ns && mc < grid.n_cpu && t < S.n_tenants) {
                const uint32_t g = X.tb.seg_g[s0 + ms];
                const unsigned long long c64 = cpu_cost(grid, mc, g);
                if (g <= 0xFFFFu && c64 <= 0xFFFFFFFFull) {          // more can never fit a 32-bit capacity
                    w |= FL_CAND | g | (t << 16);
                    c = (uint32_t)c64;
                }
            }
        }
        word[jl] = w;
        cpus[jl] = c;
    }
    __syncthreads();

    if (tid < 64) {
        uint32_t qg[QREGS], qc[QREGS];
#pragma unroll
        for (uint32_t r = 0; r < QREGS; ++r) {
            const uint32_t t = r * 64 + lane;
            qg[r] = t < S.n_tenants ? S.quota_g[t] : 0u;
            qc[r] = t < S.n_tenants ? S.quota_c[t] : 0u;
        }
        const uint32_t n_qregs = (S.n_tenants + 63u) / 64u;
        uint32_t freeG = cl.G, freeC = cl.C;
        for (uint32_t base = 0; base < nj; base += 64) {
            if (freeG == 0) break;                            // every demand asks for at least one GPU
            const uint32_t jl = base + lane;
            const uint32_t w = jl < nj ? word[jl] : 0u;
            const uint32_t c = jl < nj ? cpus[jl] : 0u;
            const uint32_t g = w & 0xFFFFu, t = (w >> 16) & 0xFFu;
            bool cand = (w & FL_CAND) != 0;
            if (__ballot(cand) == 0ull) continue;
            {   // what does not fit now cannot fit later
                uint32_t vg = 0, vc = 0;
#pragma unroll
                for (uint32_t r = 0; r < QREGS; ++r) {
                    if (r < n_qregs) {
                        const uint32_t a = (uint32_t)__shfl((int)qg[r], (int)(t & 63u), 64);
                        const uint32_t b = (uint32_t)__shfl((int)qc[r], (int)(t & 63u), 64);
                        if (r == (t >> 6)) { vg = a; vc = b; }
                    }
                }
                cand = cand && g <= vg && c <= vc && g <= freeG && c <= freeC;
            }
            bool granted = false;
            unsigned long long todo = __ballot(cand);
            while (todo) {
                const uint32_t turn = (uint32_t)__ffsll((long long)todo) - 1u;
                todo &= todo - 1;
                const uint32_t tg = lane_value(g, turn), tc = lane_value(c, turn), tt = lane_value(t, turn);
                const uint32_t ql = tt & 63u, qr = tt >> 6;
                uint32_t vg = 0, vc = 0;
#pragma unroll
                for (uint32_t r = 0; r < QREGS; ++r) {
                    const uint32_t a = lane_value(qg[r], ql), b = lane_value(qc[r], ql);
                    if (r == qr) { vg = a; vc = b; }
                }
                if (tg <= vg && tc <= vc && tg <= freeG && tc <= freeC) {
                    freeG -= tg; freeC -= tc;
#pragma unroll
                    for (uint32_t r = 0; r < QREGS; ++r)
                        if (r == qr && lane == ql) { qg[r] -= tg; qc[r] -= tc; }
                    if (lane == turn) granted = true;
                }
            }
            if (granted) word[jl] = w | FL_GRANTED;
            if (__ballot(granted)) {                          // quotas changed: is any GPU quota left at all?
                bool left = false;
#pragma unroll
                for (uint32_t r = 0; r < QREGS; ++r) left = left || qg[r] > 0;
                if (__ballot(left) == 0ull) break;
            }
        }
        if (lane == 0) { st.cap0[rnd] = freeG; st.cap0[X.R.n_rounds + rnd] = freeC; }
    }
    __syncthreads();

    for (uint32_t jl = tid; jl < nj; jl += FLOOR_THREADS) {
        const uint32_t jrel = J0 + jl - X.jb, w = word[jl];
        const bool granted = (w & FL_GRANTED) != 0;
        st.fl_gi[jrel] = granted ? S.min_seg[jrel] : -1;
        st.fl_ci[jrel] = granted ? S.min_c[jrel] : 0u;
        st.waits[jrel] = ((w & FL_GUAR) && !granted) ? RK_JOB_OUT : RK_JOB_NORMAL;
    }
}


// ------------------------------------------------------------------ Algorithm 1's Schedule as a loop
// From the state the jobs are in (paper Sec. 5.2, Algorithm 1 and the paragraph on shrinking): privileged jobs
// (below their floor) first in job order, then the others sorted once by GPU slope, CPU slope, index.  A job takes
// its next step (to its floor while below it, else the larger amount with the highest slope) when the amount can be
// gathered from what is free and from the jobs with the lowest slope among those above their own floor, each of
// which steps down to its next useful amount; a job may be shrunk when the taker's slope is higher than its own or
// the taker is below its floor, and the step is committed when all was found and (unless the taker is below its
// floor) the taker gains more than the others lose; otherwise everything is put back.
//
// One workgroup: the rule is sequential.  What is parallel is the search for a job's next step and the step down of
// the job that gives (a wavefront over its amounts, the job's rows in its registers), the search for the job to
// shrink (all threads over the cached give-slopes, which the round keeps in LDS) and the look for the next job that
// has something to do (all threads; no sort).  Control flow is the same for all threads; the first wavefront takes
// the decisions, LDS and barriers carry them.  A phase between two barriers costs its longest chain of dependent
// loads plus its instructions on one wavefront, so the phases ask for what they read in as few rounds as they can.
constexpr int RS_THREADS = 1024;

struct RsRound {                 // what a round of the loop works on
    JobState st;                 // gi, g, ci: the state the loop works on (and the memory step reads)
    uint32_t n_jobs;
    unsigned long long G, C;
    const uint8_t *state;        // may be null
    const int32_t *cur_seg;
    const uint32_t *cur_c;
    const int32_t *floor_seg;    // may be null
    const uint32_t *floor_c;     // may be null
    float *ds_g, *ds_c;          // per job: what it loses per GPU / CPU it gives (infinite: gives nothing)
    float *sg, *sc;              // per job: slopes the order is taken from
    float *ug, *uc;              // per job, kept current: slope of its next GPU / CPU step (0: none)
    uint32_t *udg;               // ... GPUs its next GPU step adds
    unsigned long long *udc_g, *udc_c;   // ... CPUs its next GPU step / CPU step adds
    uint32_t *order, *touched, *stamp, *first;
    int32_t *keep_gi;
    uint32_t *keep_ci;
    float *keep_ds;              // the two give-slopes of a job before a step touched it
    uint32_t *stats;             // may be null: steps committed, jobs on the full path, shrinks applied, steps taken back
};

struct RsArgs {                  // the kernels' argument
    Ctx X;
    RsRound r;
    // several independent rounds over the same jobs (a workgroup per round): round k works on the slice [k * n_jobs, ...)
    // of every per-job array of r, reads the state arrays from k * state_stride on and its cluster from d_clusters[k]
    uint32_t state_stride;
    const rk_cluster *d_clusters;    // null: the single round's G and C
};

// What the code of a round sees: its own slice of the per-job arrays, and the table, grid and curves where the kernel
// arguments hold them (a copy of the grid's level arrays would live in scratch memory).
struct RsView : RsRound {
    const Ctx &X;
    __device__ RsView(const RsRound &r, const Ctx &x) : RsRound(r), X(x) {}
};

// The view of round k: every per-job array moved to the round's slice.
__device__ __forceinline__ RsView rs_round(const RsArgs &K, uint32_t r) {
    RsView A(K.r, K.X);
    const RsRound &B = K.r;
    const size_t at = (size_t)r * (B.n_jobs ? B.n_jobs : 1u), from = (size_t)r * K.state_stride;
    A.st.gi += at; A.st.g += at; A.st.ci += at;
    if (B.state) A.state += from;
    A.cur_seg += from; A.cur_c += from;
    if (B.floor_seg) A.floor_seg += from;
    if (B.floor_c) A.floor_c += from;
    A.ds_g += at; A.ds_c += at; A.sg += at; A.sc += at; A.ug += at; A.uc += at; A.udg += at; A.udc_g += at; A.udc_c += at;
    A.order += at; A.touched += at; A.stamp += at; A.first += at; A.keep_gi += at; A.keep_ci += at; A.keep_ds += 2 * at;
    if (B.stats) A.stats += 4 * (size_t)r;
    if (K.d_clusters) { A.G = K.d_clusters[r].G; A.C = K.d_clusters[r].C; }
    return A;
}

// rounds that share their jobs: where every round's slots begin, and the job of every slot
__global__ void k_rs_meta(uint32_t n_rounds, uint32_t n_jobs, uint32_t *round_off, uint32_t *jmap) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= n_rounds) round_off[i] = (uint32_t)(i * n_jobs);
    if (i < (size_t)n_rounds * n_jobs) jmap[i] = (uint32_t)(i % n_jobs);
}

// Every job on its own, any number of workgroups: what it holds, whether it comes first (a floor it is below), its
// cached slopes and steps.
__global__ void k_rs_prepare(RsArgs B) {
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= B.r.n_jobs) return;
    const RsView A = rs_round(B, blockIdx.y);
    int32_t gi = -1;
    uint32_t ci = 0;
    if (rs_holds(A, j) && A.cur_seg[j] >= 0 && (uint32_t)A.cur_seg[j] < rs_ns(A, j) && A.cur_c[j] < A.X.grid.n_cpu) {
        gi = A.cur_seg[j]; ci = A.cur_c[j];
    }
    A.st.gi[j] = gi; A.st.ci[j] = ci; A.st.g[j] = (uint32_t)rs_g(A, j, gi);
    A.stamp[j] = 0u;
    const int32_t fl = rs_fl_s(A, j);
    A.first[j] = (rs_part(A, j) && fl >= 0 && gi < fl) ? 1u : 0u;
    rs_refresh(A, j);
}

__global__ __launch_bounds__(RS_THREADS) void k_reschedule(RsArgs B) {
    // what every job loses per GPU / CPU it gives, [2][n_jobs]: read by all threads at every search for a job to
    // shrink, so the round keeps them in LDS (k_rs_prepare left them in memory)
    extern __shared__ float sh_ds[];
    RsView A = rs_round(B, blockIdx.x);
    for (uint32_t j = threadIdx.x; j < A.n_jobs; j += RS_THREADS) {
        sh_ds[j] = A.ds_g[j];
        sh_ds[A.n_jobs + j] = A.ds_c[j];
    }
    A.ds_g = sh_ds;
    A.ds_c = sh_ds + A.n_jobs;
    __shared__ RsStep sh_step, sh_next[2];
    __shared__ unsigned long long sh_free[2], sh_avail[2], sh_held[2][RS_THREADS / 64];
    __shared__ float sh_lost;
    __shared__ unsigned long long sh_pick_key[RS_THREADS / 64 + 1];
    __shared__ uint32_t sh_pick_j[RS_THREADS / 64 + 1];
    __shared__ unsigned long long sh_wlow[RS_THREADS / 64];
    __shared__ uint32_t sh_below, sh_next_below;
    __shared__ uint32_t sh_widx[RS_THREADS / 64];
    __shared__ uint32_t sh_ok, sh_go, sh_touched, sh_epoch, sh_moves, sh_nb, sh_full, sh_shrinks, sh_undone;
    __shared__ RsMin sh_min[2];
    __shared__ unsigned long long sh_two_k[2 * (RS_THREADS / 64 + 1)];
    __shared__ uint32_t sh_two_s[2 * (RS_THREADS / 64 + 1)];
    constexpr uint32_t RS_LIST = 2048;                     // jobs with something to do, as the last look over all jobs found them
    __shared__ uint32_t sh_listed, sh_list_j[RS_LIST];
    __shared__ float sh_list_g[RS_LIST], sh_list_c[RS_LIST];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t J = A.n_jobs;
    const float INF = __int_as_float(0x7F800000);

    // the state the jobs are in has been loaded (k_rs_prepare); what they hold together
    unsigned long long hg = 0, hc = 0;
    for (uint32_t j = tid; j < J; j += RS_THREADS) {
        const uint32_t g = A.st.g[j];
        if (g) { hg += g; hc += cpu_cost(A.X.grid, A.st.ci[j], g); }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { hg += __shfl_xor(hg, off, 64); hc += __shfl_xor(hc, off, 64); }
    if (lane == 0) { sh_held[0][wave] = hg; sh_held[1][wave] = hc; }
    __syncthreads();
    if (tid == 0) {
        unsigned long long g = 0, c = 0;
        for (uint32_t w = 0; w < RS_THREADS / 64; ++w) { g += sh_held[0][w]; c += sh_held[1][w]; }
        sh_free[0] = g < A.G ? A.G - g : 0ull;
        sh_free[1] = c < A.C ? A.C - c : 0ull;
        sh_epoch = 0u; sh_moves = 0u; sh_full = 0u; sh_shrinks = 0u; sh_undone = 0u;
    }
    __syncthreads();

    // ScheduleJob(j); the same code path for all threads
    auto schedule_job = [&](uint32_t j) {
        // The job's next steps (GPUs, CPUs) and whether it is below its floor are kept in LDS: found here for the job as
        // it is (its cached values are written again, unchanged), and again by the refresh after every committed step.
        if (wave == 0) rs_refresh_wave(A, j, lane, sh_next, &sh_next_below, true);
        rs_lds_barrier();
        for (uint32_t res = 0; res < 2; ++res) {
            for (;;) {
                if (wave == 0) {
                    const RsStep st = sh_next[res];
                    const bool below = res == 0 && sh_next_below != 0u;     // below its floor: it takes at a loss
                    if (lane == 0) {
                        sh_step = st;
                        sh_below = below ? 1u : 0u;
                        sh_avail[0] = sh_free[0]; sh_avail[1] = sh_free[1];
                        sh_lost = 0.f; sh_ok = 1u; sh_touched = 0u; sh_epoch += 1u;
                    }
                }
                __syncthreads();
                const RsStep st = sh_step;
                if (!st.any) { __syncthreads(); break; }
                const bool below_min = sh_below != 0u;
                const unsigned long long need = res == 0 ? st.dg : st.dc;
                while (sh_ok && sh_avail[res] < need) {
                    // the job with the lowest slope among those that can give (GetLowestSlopeOverMinJob); ties: lower index
                    const float *ds = sh_ds + res * J;
                    float best = INF;
                    uint32_t who = 0xFFFFFFFFu;
                    for (uint32_t v0 = tid; v0 < J; v0 += 4 * RS_THREADS) {      // four loads in flight
                        float x[4];
#pragma unroll
                        for (uint32_t k = 0; k < 4; ++k) x[k] = v0 + k * RS_THREADS < J ? ds[v0 + k * RS_THREADS] : INF;
#pragma unroll
                        for (uint32_t k = 0; k < 4; ++k) {                        // ascending: the lower job stays among equal slopes
                            const uint32_t v = v0 + k * RS_THREADS;
                            if (v != j && x[k] < best) { best = x[k]; who = v; }
                        }
                    }
                    // (slope, job) as one key, the slope as a word that orders like it
                    unsigned long long low = who == 0xFFFFFFFFu ? ~0ull : ((unsigned long long)rs_ordered(best) << 32) | who;
                    low = wave_min_u64_rows(low);
                    if (lane == 0) sh_wlow[wave] = low;
                    rs_lds_barrier();
                    if (wave == 0) {                           // the first wavefront takes the decision and the step down
                        const unsigned long long k2 = wave_min_u64_rows(lane < RS_THREADS / 64 ? sh_wlow[lane] : ~0ull);
                        const uint32_t w2 = (uint32_t)k2;
                        const float b2 = rs_unordered((uint32_t)(k2 >> 32));
                        // what the step down reads first, asked for together
                        const bool some = k2 != ~0ull;
                        const uint32_t stamp2 = some ? A.stamp[w2] : 0u;
                        const int32_t gi0 = some ? A.st.gi[w2] : -1;
                        const uint32_t ci0 = some ? A.st.ci[w2] : 0u;
                        const uint32_t so2 = some ? A.X.tb.seg_off[w2] : 0u, ns2 = some ? A.X.tb.seg_off[w2 + 1] - so2 : 0u;
                        if (!some || !(below_min || st.slope > b2)) {
                            if (lane == 0) sh_ok = 0u;
                        } else {
                            const RsShrunk sk = rs_shrink_wave(A, w2, so2, ns2, res, gi0, ci0, lane);
                            if (lane == 0) {
                                if (stamp2 != sh_epoch) {           // first time this job gives in this step: remember its state
                                    A.stamp[w2] = sh_epoch;
                                    A.keep_gi[w2] = gi0; A.keep_ci[w2] = ci0;
                                    A.keep_ds[2 * w2] = A.ds_g[w2]; A.keep_ds[2 * w2 + 1] = A.ds_c[w2];
                                    A.touched[sh_touched++] = w2;
                                }
                                sh_avail[0] += sk.gv.dg; sh_avail[1] += sk.gv.dc;
                                sh_lost = sh_lost + sk.gv.loss;
                                A.st.gi[w2] = sk.gi; A.st.ci[w2] = sk.ci;
                                A.ds_g[w2] = sk.ds_g; A.ds_c[w2] = sk.ds_c;   // (its own next steps are brought up to date on commit)
                                sh_shrinks += 1u;
                            }
                        }
                    }
                    // (what the first wavefront wrote to memory, the state of the job that gave, is read again by itself only,
                    // until the barrier that follows the loop)
                    rs_lds_barrier();
                }
                if (tid == 0) {
                    bool ok = sh_ok != 0u;
                    if (ok && (sh_avail[0] < st.dg || sh_avail[1] < st.dc)) ok = false;
                    if (ok && !below_min && !(st.gain > sh_lost)) ok = false;
                    if (!ok) {
                        for (uint32_t i = 0; i < sh_touched; ++i) {         // everything back as it was
                            const uint32_t v = A.touched[i];
                            A.st.gi[v] = A.keep_gi[v]; A.st.ci[v] = A.keep_ci[v];
                            A.ds_g[v] = A.keep_ds[2 * v]; A.ds_c[v] = A.keep_ds[2 * v + 1];
                        }
                        sh_undone += sh_touched ? 1u : 0u;
                    } else {
                        sh_free[0] = sh_avail[0] - st.dg; sh_free[1] = sh_avail[1] - st.dc;
                        if (res == 0) A.st.gi[j] = st.tgt;
                        A.st.ci[j] = st.lvl;
                        sh_moves += 1u;
                    }
                    sh_go = ok ? 1u : 0u;
                }
                __syncthreads();
                const uint32_t go = sh_go;
                if (go) {                                       // the jobs whose state changed: all their cached values
                    const uint32_t n_touched = sh_touched;           // a wavefront per job
                    for (uint32_t i = wave; i < n_touched + 1u; i += RS_THREADS / 64)
                        rs_refresh_wave(A, i < n_touched ? A.touched[i] : j, lane, sh_next, &sh_next_below, i >= n_touched);
                }
                __syncthreads();
                if (!go) break;
            }
        }
    };

    // privileged jobs, in job order.  Who they are is known from the start: a job never gives below its floor, so
    // only a job that begins below it can be below it.
    if (tid == 0) sh_nb = 0u;
    __syncthreads();
    for (uint32_t base = 0; base < J; base += RS_THREADS) {       // their list, in job order: 1,024 jobs at a time
        const uint32_t j = base + tid;
        const bool is = j < J && A.first[j] != 0u;
        const unsigned long long in_wave = __ballot(is);
        if (lane == 0) sh_widx[wave] = (uint32_t)__popcll(in_wave);
        __syncthreads();
        uint32_t before = sh_nb, all = 0;
        for (uint32_t w = 0; w < RS_THREADS / 64; ++w) {
            if (w < wave) before += sh_widx[w];
            all += sh_widx[w];
        }
        if (is) A.order[before + (uint32_t)__popcll(in_wave & ((1ull << lane) - 1ull))] = j;
        __syncthreads();
        if (tid == 0) sh_nb += all;
    }
    __syncthreads();
    const uint32_t na = sh_nb;
    for (uint32_t k = 0; k < na; ++k) schedule_job(A.order[k]);
    __syncthreads();
    // the others: their order is fixed once, by GPU slope, then CPU slope (both descending), then index
    for (uint32_t j = tid; j < J; j += RS_THREADS) {
        const bool in = rs_part(A, j) && !A.first[j];
        A.sg[j] = in ? A.ug[j] : -1.f;                          // the cached slopes are current; -1: not in the list
        A.sc[j] = in ? A.uc[j] : -1.f;
    }
    __syncthreads();
    // Most jobs of a large round find nothing to do when their turn comes: no step, or a step that needs more than is
    // free while no other job's slope is lower than theirs.  Whether that is so follows from values that change only
    // when a step is committed: the job's own next steps (kept current for every job), what is free, and the two
    // lowest slopes among the jobs that can give.  Passing over such a job changes nothing, so the jobs need not be
    // sorted: all threads look for the first job in the order, after the one served last, that is not of that kind,
    // it is served in full, and the search starts again from the new state.
    auto comes_before = [&](float ga, float ca, uint32_t a, float gb, float cb, uint32_t b) {
        return ga > gb || (ga == gb && (ca > cb || (ca == cb && a < b)));
    };
    float last_g = INF, last_c = INF;                     // key of the job served last (before every job at first)
    uint32_t last_j = 0u, moves_seen = 0xFFFFFFFFu;
    for (;;) {
        __syncthreads();
        const bool fresh = sh_moves != moves_seen;        // a step was committed since the last look (or this is the first)
        moves_seen = sh_moves;
        __syncthreads();
        if (fresh) {                                      // otherwise the lowest slopes are what they were
            RsMin two[2];
            rs_two_lowest<RS_THREADS / 64, RS_THREADS>(sh_ds, J, tid, lane, wave, sh_two_k, sh_two_s, two);
            if (tid == 0) { sh_min[0] = two[0]; sh_min[1] = two[1]; }
            if (tid == 2) sh_listed = 0u;
        }
        __syncthreads();
        const unsigned long long free_g = sh_free[0], free_c = sh_free[1];
        const RsMin mg = sh_min[0], mc = sh_min[1];
        float best_g = -1.f, best_c = -1.f;                // -1: none found
        uint32_t best_j = 0xFFFFFFFFu;
        // A look after a committed step goes over all jobs and lists those that have something to do; until the next
        // committed step the later looks go over that list only (if it held them all): nothing they depend on changes.
        if (fresh || sh_listed > RS_LIST) {
            for (uint32_t j0 = tid; j0 < J; j0 += 4 * RS_THREADS) {      // four jobs' values in flight
                float kg[4], kc[4], ug[4], uc[4];
                uint32_t dg[4];
                unsigned long long dcg[4], dcc[4];
#pragma unroll
                for (uint32_t k = 0; k < 4; ++k) {
                    const uint32_t j = j0 + k * RS_THREADS;
                    const bool in = j < J;
                    kg[k] = in ? A.sg[j] : -1.f; kc[k] = in ? A.sc[j] : -1.f;
                    ug[k] = in ? A.ug[j] : 0.f; uc[k] = in ? A.uc[j] : 0.f;
                    dg[k] = in ? A.udg[j] : 0u; dcg[k] = in ? A.udc_g[j] : 0ull; dcc[k] = in ? A.udc_c[j] : 0ull;
                }
#pragma unroll
                for (uint32_t k = 0; k < 4; ++k) {
                    const uint32_t j = j0 + k * RS_THREADS;
                    if (kg[k] < 0.f || !comes_before(last_g, last_c, last_j, kg[k], kc[k], j)) continue;   // not in the list, or served
                    const float lowest_g = j == mg.i1 ? mg.m2 : mg.m1, lowest_c = j == mc.i1 ? mc.m2 : mc.m1;
                    // GPU step: none; or GPUs are short and nobody may be shrunk for it; or the GPUs are there and its CPUs are not
                    const bool gpu_idle = !(ug[k] > 0.f) || (free_g < dg[k] ? !(ug[k] > lowest_g) : free_c < dcg[k]);
                    const bool cpu_idle = !(uc[k] > 0.f) || (free_c < dcc[k] && !(uc[k] > lowest_c));
                    if (gpu_idle && cpu_idle) continue;
                    if (fresh) {
                        const uint32_t at = atomicAdd(&sh_listed, 1u);
                        if (at < RS_LIST) { sh_list_j[at] = j; sh_list_g[at] = kg[k]; sh_list_c[at] = kc[k]; }
                    }
                    if (best_j == 0xFFFFFFFFu || comes_before(kg[k], kc[k], j, best_g, best_c, best_j)) { best_g = kg[k]; best_c = kc[k]; best_j = j; }
                }
            }
        } else {
            const uint32_t listed = sh_listed;
            for (uint32_t i = tid; i < listed; i += RS_THREADS) {
                const uint32_t j = sh_list_j[i];
                const float kg = sh_list_g[i], kc = sh_list_c[i];
                if (!comes_before(last_g, last_c, last_j, kg, kc, j)) continue;                            // served
                if (best_j == 0xFFFFFFFFu || comes_before(kg, kc, j, best_g, best_c, best_j)) { best_g = kg; best_c = kc; best_j = j; }
            }
        }
        {                                                    // the first of the threads' candidates in the order
            const RsPick pick = rs_pick_first<RS_THREADS / 64>(best_g, best_c, best_j, lane, wave, sh_pick_key, sh_pick_j);
            best_g = pick.g; best_c = pick.c; best_j = pick.j;
        }
        if (best_j == 0xFFFFFFFFu) break;
        if (tid == 0) sh_full += 1u;
        schedule_job(best_j);
        last_g = best_g; last_c = best_c; last_j = best_j;
    }
    __syncthreads();
    for (uint32_t j = tid; j < J; j += RS_THREADS) A.st.g[j] = (uint32_t)rs_g(A, j, A.st.gi[j]);
    if (tid == 0 && A.stats) { A.stats[0] = sh_moves; A.stats[1] = sh_full; A.stats[2] = sh_shrinks; A.stats[3] = sh_undone; }
}

// Scratch of rk_allocate_static: one array in the library's image, so every device the library is loaded on holds
// its own copy at its own address for as long as the process lives.  The name is a host-side stand-in only: host
// code uses the address that hipGetSymbolAddress returned for the context's device (rk_ctx::static_scratch).
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)12 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// Where the working buffers of a call come from: the context's grow-only device buffers (base == nullptr), or
// consecutive 256-byte aligned pieces of a fixed block (no allocation; a call that needs more fails).
struct Arena {
    unsigned char *base;
    size_t used, cap;
};

template <typename T>
int32_t scratch_typed(rk_ctx *ctx, Arena &arena, int slot, size_t count, T **out) {
    if (!arena.base) return rk_scratch(ctx, slot, count * sizeof(T), reinterpret_cast<void **>(out));
    size_t bytes = count * sizeof(T);
    bytes = ((bytes ? bytes : 1) + 255) & ~(size_t)255;
    if (arena.used + bytes > arena.cap)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "the round needs more than the %zu bytes of static scratch memory", arena.cap);
    *out = reinterpret_cast<T *>(arena.base + arena.used);
    arena.used += bytes;
    return RK_OK;
}

// *closed: the pass also took the memory step that ends the round
template <int PASS>
int32_t launch_pass(rk_ctx *ctx, const Ctx &X, const JobState &st, const HullBuf &H, const Hist &hist,
                    uint32_t n_rounds, uint32_t n_jobs, uint32_t mj, uint32_t max_segs, size_t tail_lds, size_t zero_bins,
                    rk_assign *assign, float *totals, bool *closed) {
    hipStream_t s = ctx->stream;
    const uint32_t hull_blocks = (n_jobs + (HULL_THREADS / 64) - 1) / (HULL_THREADS / 64);
    const dim3 job_grid(st.blocks_per_round, n_rounds);
    *closed = false;
    if (n_jobs > 0) {
        // amounts per job: GPU counts (at most max_segs) in the GPU pass, CPU levels in the CPU pass
        const uint32_t amounts = PASS == 0 ? max_segs : X.grid.n_cpu;
        const uint32_t waves = HULL_THREADS / 64;
        if (amounts <= 16) {
            k_hull_groups<PASS, 16><<<(n_jobs + 4 * waves - 1) / (4 * waves), HULL_THREADS, 0, s>>>(X, st, H, hist, zero_bins);
        } else if (amounts <= 32) {
            k_hull_groups<PASS, 32><<<(n_jobs + 2 * waves - 1) / (2 * waves), HULL_THREADS, 0, s>>>(X, st, H, hist, zero_bins);
        } else {
            k_hull<PASS><<<hull_blocks, HULL_THREADS, 0, s>>>(X, st, H, hist, zero_bins);
        }
        RK_CHECK_LAUNCH(ctx, "k_hull");
    }
    const size_t sel_lds = tail_lds > SELECT_HIST_BYTES ? tail_lds : SELECT_HIST_BYTES;
    if (mj <= SMALL_ROUND_JOBS) {
        k_select_small<PASS, SMALL_ROUND_JOBS / TAIL_THREADS><<<n_rounds, TAIL_THREADS, sel_lds, s>>>(X, mj, st, H, assign, totals);
        RK_CHECK_LAUNCH(ctx, "k_select_small");
        *closed = PASS == 1;
        return RK_OK;
    }
    if constexpr (PASS == 1) {
        if ((uint64_t)(X.grid.n_cpu - 1u) * mj <= CPU_ONE_WG_STEPS) {
            k_select_small<1, TAIL_KMAX><<<n_rounds, TAIL_THREADS, sel_lds, s>>>(X, mj, st, H, assign, totals);
            RK_CHECK_LAUNCH(ctx, "k_select_small");
            return RK_OK;
        }
    }
    if (n_jobs > 0) {
        k_hist<PASS, 0><<<job_grid, JOB_THREADS, 0, s>>>(X, st, H, hist);
        RK_CHECK_LAUNCH(ctx, "k_hist<0>");
        k_hist<PASS, 1><<<job_grid, JOB_THREADS, 0, s>>>(X, st, H, hist);
        RK_CHECK_LAUNCH(ctx, "k_hist<1>");
    }
    k_apply<PASS><<<job_grid, JOB_THREADS, 0, s>>>(X, st, H, hist);
    RK_CHECK_LAUNCH(ctx, "k_apply");
    k_tail<PASS><<<n_rounds, TAIL_THREADS, tail_lds, s>>>(X, mj, st);
    RK_CHECK_LAUNCH(ctx, "k_tail");
    return RK_OK;
}

}  // namespace

// Once per context, with its device current: the address of this device's copy of the static scratch array, and
// the dynamic LDS limits of the kernels that may need more than the default (large rounds keep per-job state in LDS;
// the single-workgroup selection adds dynamic to static LDS).  Done here so that no later call has to.
int32_t rk_allocate_setup(rk_ctx *ctx) {
    void *p = nullptr;
    RK_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    ctx->static_scratch = static_cast<unsigned char *>(p);
    const void *big[] = {reinterpret_cast<const void *>(k_tail<0>), reinterpret_cast<const void *>(k_tail<1>),
                         reinterpret_cast<const void *>(k_floors),
                         reinterpret_cast<const void *>(k_select_small<1, TAIL_KMAX>)};
    for (const void *f : big) RK_HIP(ctx, hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024));
    const void *small[] = {reinterpret_cast<const void *>(k_select_small<0, SMALL_ROUND_JOBS / TAIL_THREADS>),
                           reinterpret_cast<const void *>(k_select_small<1, SMALL_ROUND_JOBS / TAIL_THREADS>)};
    for (const void *f : small) RK_HIP(ctx, hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
    return RK_OK;
}

int32_t rk_launch_allocate(rk_ctx *ctx, const float *ref_thr, const TableDev &tb, const rk_alloc_grid *grid,
                           uint32_t n_rounds, const uint32_t *d_round_off, const rk_cluster *d_clusters,
                           const rk_cluster *one_cluster, uint32_t jb, uint32_t n_jobs, uint32_t max_jobs,
                           uint32_t max_segs_per_job, const float *best_thr, const uint32_t *best_plan,
                           const float *curve_thr, const SlaDev *sla, const FloorsDev *given, const uint32_t *d_jmap,
                           rk_assign *assign, float *totals, bool static_scratch) {
    if (n_rounds == 0) return RK_OK;
    Arena arena = {nullptr, 0, 0};
    if (static_scratch) {
        if (!ctx->static_scratch) return rk_fail(ctx, RK_ERR_DEVICE, "the static scratch memory was not set up");
        arena = Arena{ctx->static_scratch, 0, STATIC_SCRATCH_BYTES};
    }
    if (d_jmap && (sla || given || jb != 0))
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "rounds that share jobs take neither floors nor a job range");
    if (max_jobs > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "a round has %u jobs, the allocation kernels take up to %u", max_jobs,
                       RK_MAX_JOBS_PER_ROUND);
    int32_t rc;
    HullBuf H;
    H.stride = n_jobs ? n_jobs : 1;
    H.width = max_segs_per_job > grid->n_cpu ? max_segs_per_job : grid->n_cpu;   // the longest walk of either pass
    if (H.width == 0) H.width = 1;
    const size_t entries = (size_t)H.stride * H.width;
    if ((rc = scratch_typed(ctx, arena, SL_HULL_KEY, entries, &H.key))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_HULL_RAW, entries, &H.raw))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_HULL_TGT, entries, &H.tgt))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_HULL_DG, entries, &H.dg))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_HULL_DC, entries, &H.dc))) return rc;
    JobState st;
    st.blocks_per_round = (max_jobs + JOB_THREADS - 1) / JOB_THREADS;
    if (st.blocks_per_round == 0) st.blocks_per_round = 1;
    if ((rc = scratch_typed(ctx, arena, SL_ST_GI, (size_t)H.stride, &st.gi))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_G, (size_t)H.stride, &st.g))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_CI, (size_t)H.stride, &st.ci))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_STEP_SLOPE, (size_t)H.stride, &st.step_slope))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_STEP_TGT, (size_t)H.stride, &st.step_tgt))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_STEP_DG, (size_t)H.stride, &st.step_dg))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_FREEG, (size_t)n_rounds * 2, &st.free_g))) return rc;   // [free G | free C] after apply
    if ((rc = scratch_typed(ctx, arena, SL_ST_FREEC, (size_t)n_rounds + ((size_t)n_rounds + 1) / 2, &st.free_c))) return rc;
    st.cpu_steps = reinterpret_cast<uint32_t *>(st.free_c + n_rounds);
    if ((rc = scratch_typed(ctx, arena, SL_ST_PARTIAL, (size_t)n_rounds * st.blocks_per_round * 2, &st.partial))) return rc;
    st.fl_gi = nullptr; st.fl_ci = nullptr; st.waits = nullptr; st.cap0 = nullptr;
    if (given) {
        st.fl_gi = given->gi; st.fl_ci = given->ci; st.waits = given->state; st.cap0 = given->cap0;
    } else if (sla) {
        if ((rc = scratch_typed(ctx, arena, SL_FL_GI, (size_t)H.stride, &st.fl_gi))) return rc;
        if ((rc = scratch_typed(ctx, arena, SL_FL_CI, (size_t)H.stride, &st.fl_ci))) return rc;
        if ((rc = scratch_typed(ctx, arena, SL_FL_WAITS, (size_t)H.stride, &st.waits))) return rc;
        if ((rc = scratch_typed(ctx, arena, SL_FL_CAP0, (size_t)n_rounds * 2, &st.cap0))) return rc;
    }
    Hist hist;
    const size_t hist_bins = (size_t)n_rounds * 4 * BINS;
    if ((rc = scratch_typed(ctx, arena, SL_HIST_G, hist_bins, &hist.g))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_HIST_C, hist_bins, &hist.c))) return rc;

    Ctx X;
    X.ref_thr = ref_thr; X.tb = tb; X.grid = grid_dev(grid); X.jb = jb; X.jmap = d_jmap;
    X.best_thr = best_thr; X.best_plan = best_plan; X.curve_thr = curve_thr;
    X.R.round_off = d_round_off; X.R.clusters = d_clusters; X.R.n_rounds = n_rounds;
    X.R.inline_one = one_cluster ? 1u : 0u;
    X.R.off0 = jb; X.R.off1 = jb + n_jobs;
    X.R.cl = one_cluster ? *one_cluster : rk_cluster{0u, 0u, 0.f};

    const uint32_t mj = max_jobs ? ((max_jobs + 1u) & ~1u) : 2u;
    const size_t lds = (size_t)mj * (2 + 2 + 2 + 2 + 4);
    // (the kernels' dynamic LDS limits were raised when the context was made: rk_allocate_setup)
    hipStream_t s = ctx->stream;
    // Histograms start at zero: the first walk kernel clears them for both passes on its way (fill code, no
    // memset, so the sequence can be captured in a graph).  Rounds large enough to use them have jobs, so that
    // kernel always runs.
    const bool hists = mj > SMALL_ROUND_JOBS;
    if (sla && !given) {
        k_floors<<<n_rounds, FLOOR_THREADS, (size_t)mj * 8, s>>>(X, st, *sla, mj);
        RK_CHECK_LAUNCH(ctx, "k_floors");
    }
    bool closed = false;
    if ((rc = launch_pass<0>(ctx, X, st, H, hist, n_rounds, n_jobs, mj, max_segs_per_job, lds, hists ? hist_bins : 0, assign,
                             totals, &closed))) return rc;
    if ((rc = launch_pass<1>(ctx, X, st, H, hist, n_rounds, n_jobs, mj, max_segs_per_job, lds, 0, assign, totals,
                             &closed))) return rc;
    if (closed) return RK_OK;                                   // the CPU pass's selection took the memory step
    if (max_jobs > 0) {
        k_mem_wish<<<dim3(st.blocks_per_round, n_rounds), JOB_THREADS, 0, s>>>(X, st, assign);
        RK_CHECK_LAUNCH(ctx, "k_mem_wish");
    }
    k_mem_finish<<<n_rounds, 64, 0, s>>>(X, st, assign, totals);
    RK_CHECK_LAUNCH(ctx, "k_mem_finish");
    return RK_OK;
}

extern "C" int32_t rk_reschedule(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                 const rk_alloc_grid *grid, const rk_cluster *cluster, const float *best_thr,
                                 const uint32_t *best_plan, const float *curve_thr, const rk_job_state *jobs_state,
                                 rk_assign *assign, float *total, uint32_t *stats) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, 0, table ? table->n_jobs : 0))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (!cluster || !total || !jobs_state) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    const uint32_t J = table->n_jobs;
    if (J > 0 && (!ref_thr || !assign || !jobs_state->cur_seg || !jobs_state->cur_c ||
                  (table->n_segs > 0 && (!best_thr || !best_plan || !curve_thr))))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (!(cluster->host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    if (J > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u jobs, the allocation kernels take up to %u", J, RK_MAX_JOBS_PER_ROUND);
    RK_HIP(ctx, hipSetDevice(ctx->device));
    return rk_launch_reschedule(ctx, ref_thr, table, grid, cluster, best_thr, best_plan, curve_thr, jobs_state, assign, total,
                                stats);
}

// n_rounds independent rounds over the same jobs (clusters [host] n_rounds entries; round r reads the state arrays from
// r * state_stride on and writes assign[r * n_jobs ...], totals[r], stats[4 r ...]); one round: the plain loop
static int32_t launch_reschedule_rounds(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                        const rk_alloc_grid *grid, uint32_t n_rounds, const rk_cluster *clusters,
                                        const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                                        const rk_job_state *jobs_state, uint32_t state_stride, rk_assign *assign,
                                        float *totals, uint32_t *stats) {
    const uint32_t J = table->n_jobs;
    int32_t rc;
    Arena arena = {nullptr, 0, 0};
    const size_t n = J ? J : 1, all = n * n_rounds;
    RsArgs K;
    RsRound &A = K.r;
    JobState &st = A.st;
    st = JobState{};
    st.blocks_per_round = (J + JOB_THREADS - 1) / JOB_THREADS;
    if (st.blocks_per_round == 0) st.blocks_per_round = 1;
    if ((rc = scratch_typed(ctx, arena, SL_ST_GI, all, &st.gi))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_G, all, &st.g))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_CI, all, &st.ci))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_ST_PARTIAL, (size_t)st.blocks_per_round * 2 * n_rounds, &st.partial))) return rc;
    float *f32;
    uint32_t *u32;
    unsigned long long *u64;
    if ((rc = scratch_typed(ctx, arena, SL_RS_F32, all * 8, &f32))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_RS_U32, all * 7, &u32))) return rc;
    if ((rc = scratch_typed(ctx, arena, SL_RS_U64, all * 2, &u64))) return rc;
    A.ds_g = f32; A.ds_c = f32 + all; A.sg = f32 + 2 * all; A.sc = f32 + 3 * all; A.ug = f32 + 4 * all; A.uc = f32 + 5 * all;
    A.keep_ds = f32 + 6 * all;
    A.order = u32; A.touched = u32 + all; A.stamp = u32 + 2 * all; A.first = u32 + 3 * all;
    A.keep_gi = reinterpret_cast<int32_t *>(u32 + 4 * all); A.keep_ci = u32 + 5 * all; A.udg = u32 + 6 * all;
    A.udc_g = u64; A.udc_c = u64 + all;
    Ctx &X = K.X;
    X.ref_thr = ref_thr; X.tb = table_dev(table); X.grid = grid_dev(grid); X.jb = 0; X.jmap = nullptr;
    X.best_thr = best_thr; X.best_plan = best_plan; X.curve_thr = curve_thr;
    X.R.round_off = nullptr; X.R.clusters = nullptr; X.R.n_rounds = n_rounds; X.R.inline_one = 1u;
    X.R.off0 = 0; X.R.off1 = J; X.R.cl = clusters[0];
    A.n_jobs = J; A.G = clusters[0].G; A.C = clusters[0].C;
    A.state = jobs_state->state; A.cur_seg = jobs_state->cur_seg; A.cur_c = jobs_state->cur_c;
    A.floor_seg = jobs_state->floor_seg; A.floor_c = jobs_state->floor_c;
    A.stats = stats;
    K.state_stride = state_stride; K.d_clusters = nullptr;
    hipStream_t s = ctx->stream;
    if (n_rounds > 1) {                                        // the rounds' slots, the job of every slot, the clusters
        const size_t off_bytes = (((size_t)n_rounds + 1) * 4 + 15) & ~(size_t)15;
        char *d_meta;
        uint32_t *d_jmap;
        if ((rc = rk_scratch(ctx, SL_ROUND_META, off_bytes + (size_t)n_rounds * sizeof(rk_cluster), (void **)&d_meta))) return rc;
        if ((rc = rk_scratch(ctx, SL_JMAP, all * 4, (void **)&d_jmap))) return rc;
        RK_HIP(ctx, hipMemcpyAsync(d_meta + off_bytes, clusters, (size_t)n_rounds * sizeof(rk_cluster), hipMemcpyHostToDevice, s));
        const size_t most = all > (size_t)n_rounds + 1 ? all : (size_t)n_rounds + 1;
        k_rs_meta<<<(uint32_t)((most + 255) / 256), 256, 0, s>>>(n_rounds, J, reinterpret_cast<uint32_t *>(d_meta), d_jmap);
        RK_CHECK_LAUNCH(ctx, "k_rs_meta");
        X.R.round_off = reinterpret_cast<const uint32_t *>(d_meta);
        X.R.clusters = reinterpret_cast<const rk_cluster *>(d_meta + off_bytes);
        X.R.inline_one = 0u;
        X.jmap = d_jmap;
        K.d_clusters = X.R.clusters;
    }
    if (J > 0) {
        k_rs_prepare<<<dim3((J + 255) / 256, n_rounds), 256, 0, s>>>(K);
        RK_CHECK_LAUNCH(ctx, "k_rs_prepare");
    }
    const size_t lds = (size_t)2 * (J ? J : 1u) * sizeof(float);                // at most 96 KiB
    if (lds > 64 * 1024 && !ctx->loop_lds_raised) {
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_reschedule),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 2 * RK_MAX_JOBS_PER_ROUND * sizeof(float)));
        ctx->loop_lds_raised = true;
    }
    k_reschedule<<<n_rounds, RS_THREADS, lds, s>>>(K);
    RK_CHECK_LAUNCH(ctx, "k_reschedule");
    if (J > 0) {
        k_mem_wish<<<dim3(st.blocks_per_round, n_rounds), JOB_THREADS, 0, s>>>(X, st, assign);
        RK_CHECK_LAUNCH(ctx, "k_mem_wish");
    }
    k_mem_finish<<<n_rounds, 64, 0, s>>>(X, st, assign, totals);
    RK_CHECK_LAUNCH(ctx, "k_mem_finish");
    return RK_OK;
}

int32_t rk_launch_reschedule(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table, const rk_alloc_grid *grid,
                             const rk_cluster *cluster, const float *best_thr, const uint32_t *best_plan,
                             const float *curve_thr, const rk_job_state *jobs_state, rk_assign *assign, float *total,
                             uint32_t *stats) {
    return launch_reschedule_rounds(ctx, ref_thr, table, grid, 1, cluster, best_thr, best_plan, curve_thr, jobs_state, 0, assign,
                                    total, stats);
}

extern "C" int32_t rk_reschedule_rounds(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                        const rk_alloc_grid *grid, uint32_t n_rounds, const rk_cluster *clusters,
                                        const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                                        const rk_job_state *jobs_state, uint32_t state_stride, rk_assign *assign,
                                        float *totals, uint32_t *stats) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, 0, table ? table->n_jobs : 0))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (!clusters || !totals || !jobs_state) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (n_rounds == 0) return RK_OK;
    const uint32_t J = table->n_jobs;
    if (J > 0 && (!ref_thr || !assign || !jobs_state->cur_seg || !jobs_state->cur_c ||
                  (table->n_segs > 0 && (!best_thr || !best_plan || !curve_thr))))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (state_stride != 0 && state_stride != J)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "state_stride must be 0 (one state for all rounds) or n_jobs (one per round)");
    for (uint32_t r = 0; r < n_rounds; ++r)
        if (!(clusters[r].host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    if (J > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u jobs, the allocation kernels take up to %u", J, RK_MAX_JOBS_PER_ROUND);
    if ((uint64_t)n_rounds * (J ? J : 1) > (1ull << 26) || n_rounds > 65535u)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "rounds x jobs above 2^26, or more than 65535 rounds");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    return launch_reschedule_rounds(ctx, ref_thr, table, grid, n_rounds, clusters, best_thr, best_plan, curve_thr, jobs_state,
                                    state_stride, assign, totals, stats);
}

static int32_t allocate_one_round(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                  const rk_alloc_grid *grid, const rk_cluster *cluster, uint32_t jb, uint32_t je,
                                  const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                                  rk_assign *assign, float *total, bool static_scratch) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (!cluster || !total) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    // (a table without any segment has empty value arrays, which may be null)
    if (je > jb && (!ref_thr || !assign || (table->n_segs > 0 && (!best_thr || !best_plan || !curve_thr))))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (!(cluster->host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    if (static_scratch) {
        const uint64_t width = table->max_segs_per_job > grid->n_cpu ? table->max_segs_per_job : grid->n_cpu;
        if ((uint64_t)(je - jb) * width > RK_STATIC_MAX_STEPS)
            return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u jobs x %llu amounts per job: rk_allocate_static takes up to %u",
                           je - jb, (unsigned long long)width, RK_STATIC_MAX_STEPS);
    }
    RK_HIP(ctx, hipSetDevice(ctx->device));
    return rk_launch_allocate(ctx, ref_thr, table_dev(table), grid, 1, nullptr, nullptr, cluster, jb, je - jb, je - jb,
                              table->max_segs_per_job, best_thr, best_plan, curve_thr, nullptr, nullptr, nullptr, assign,
                              total, static_scratch);
}

extern "C" int32_t rk_allocate(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                               const rk_alloc_grid *grid, const rk_cluster *cluster, uint32_t jb, uint32_t je,
                               const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                               rk_assign *assign, float *total) {
    return allocate_one_round(ctx, ref_thr, table, grid, cluster, jb, je, best_thr, best_plan, curve_thr, assign, total,
                              false);
}

extern "C" int32_t rk_allocate_static(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                      const rk_alloc_grid *grid, const rk_cluster *cluster, uint32_t jb, uint32_t je,
                                      const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                                      rk_assign *assign, float *total) {
    return allocate_one_round(ctx, ref_thr, table, grid, cluster, jb, je, best_thr, best_plan, curve_thr, assign, total,
                              true);
}

int32_t rk_check_sla(rk_ctx *ctx, const rk_sla *sla, bool need_request) {
    if (!sla) return rk_fail(ctx, RK_ERR_INVALID_ARG, "sla is null");
    if (!sla->guaranteed || !sla->tenant) return rk_fail(ctx, RK_ERR_INVALID_ARG, "sla: guaranteed or tenant is null");
    if (sla->n_tenants > RK_MAX_TENANTS)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "%u tenants, at most %u", sla->n_tenants, RK_MAX_TENANTS);
    if (sla->n_tenants > 0 && (!sla->quota_g || !sla->quota_c)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "sla: quota array is null");
    if (need_request && (!sla->req_g || !sla->req_c || !sla->req_m || !sla->base_thr))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "sla: request or baseline array is null");
    return RK_OK;
}

extern "C" int32_t rk_allocate_sla(rk_ctx *ctx, const float *ref_thr, const rk_plan_table *table,
                                   const rk_alloc_grid *grid, const rk_cluster *cluster, uint32_t jb, uint32_t je,
                                   const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                                   const rk_sla *sla, const int32_t *min_seg, const uint32_t *min_c,
                                   rk_assign *assign, float *total) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if (!cluster || !total) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (je > jb && (!ref_thr || !assign || !min_seg || !min_c ||
                    (table->n_segs > 0 && (!best_thr || !best_plan || !curve_thr))))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (je > jb && (rc = rk_check_sla(ctx, sla, false))) return rc;
    if (!(cluster->host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    SlaDev S = {};
    if (je > jb) S = SlaDev{sla->guaranteed, sla->tenant, min_seg, min_c, sla->n_tenants, sla->quota_g, sla->quota_c};
    return rk_launch_allocate(ctx, ref_thr, table_dev(table), grid, 1, nullptr, nullptr, cluster, jb, je - jb, je - jb,
                              table->max_segs_per_job, best_thr, best_plan, curve_thr, je > jb ? &S : nullptr, nullptr,
                              nullptr, assign, total, false);
}
