// Greedy marginal-gain allocation over the resource sensitivity curves
// (paper Sec. 5.2: prefer the jobs that gain the most per unit of resource,
// GPU slopes before CPU slopes; memory is granted last from the chosen plan's
// estimate).
//
// The rule is sequential: repeatedly take the (job, larger amount) with the
// highest float32 slope ((v1 - v0) / ref_thr) / delta among the steps that
// still fit; ties go to the smaller amount, then to the lower job index.
// It is evaluated without running every step in sequence:
//
//  1. Each job's steps, were capacity never short, form a fixed walk over the
//     upper hull of its curve (k_hull, one wavefront per job).  With each
//     slope replaced by the running minimum of the walk, the sequential order
//     is the descending order of these keys (then job, then walk position).
//  2. A radix select over the key bits finds the largest key threshold whose
//     whole set of steps fits the capacity; that set is a prefix of the
//     sequential order and is applied at once (k_pass, one workgroup per round).
//  3. From there the plain step-by-step loop runs on the little capacity that
//     is left: a workgroup-wide argmax over cached per-job best steps.
//
// The same three stages run for the GPU pass and then for the CPU pass.
// Memory (k_mem_wish / k_mem_finish): when the tiers every job would like fit
// with margin, all are granted in parallel; otherwise one wavefront takes the
// decisions in job order.
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int PASS_THREADS = 1024;
constexpr int PASS_WAVES = PASS_THREADS / 64;
constexpr int HULL_THREADS = 256;
constexpr int WISH_THREADS = 256;

struct HullBuf {             // walk steps, entry (k, job) at k*stride + job (job relative to the call's first job)
    uint32_t *key;           // float bits of the running-minimum slope; 0 ends a walk
    float *raw;              // the step's own slope
    uint16_t *tgt;           // target: segment index (GPU pass) or CPU level (CPU pass)
    uint32_t *dg;            // GPUs the step adds
    unsigned long long *dc;  // CPUs the step adds
    uint32_t stride, width;
};

struct JobState {            // per job of the call, between the kernels
    int32_t *gi;             // granted segment index, -1 = no GPUs
    uint32_t *g;             // granted GPUs
    uint32_t *ci;            // granted CPU level
    unsigned long long *free_c;   // per round: CPUs left after the GPU pass
    double *partial;         // per round and block of k_mem_wish: {sum of wish GiB, sum of thr/ref}
    uint32_t blocks_per_round;
};

// Rounds: job ranges and cluster capacities, either device arrays or, for a
// single round, values carried in the kernel arguments.
struct RoundArgs {
    const uint32_t *round_off;
    const rk_cluster *clusters;
    uint32_t n_rounds, inline_one;
    uint32_t off0, off1;
    rk_cluster cl;
};

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

__device__ __forceinline__ unsigned long long cpu_cost(const GridDev &G, uint32_t ci, uint32_t g) {
    return G.cpu_mode ? (unsigned long long)G.cpu_levels[ci] * g : (unsigned long long)G.cpu_levels[ci];
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ------------------------------------------------------------------ hull walks
// One wavefront per job; lanes hold the candidate amounts.  PASS 0: GPU counts
// of the job (lowest CPU level, highest memory tier, values from the curves);
// PASS 1: CPU levels at the granted GPU count (values from the per-segment
// maxima).  Amounts that the whole round could never afford are left out.
template <int PASS>
__global__ __launch_bounds__(HULL_THREADS) void k_hull(const float *__restrict__ ref_thr, TableDev tb, GridDev grid,
                                                       RoundArgs R, uint32_t jb, const float *__restrict__ vals,
                                                       JobState st, HullBuf H) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t jrel = blockIdx.x * (HULL_THREADS / 64) + (threadIdx.x >> 6);
    if (jrel >= H.stride) return;                         // whole wavefront
    const uint32_t j = jb + jrel;
    const uint32_t rnd = round_index_of(R, j);
    uint32_t rj0, rj1;
    rk_cluster cl;
    round_of(R, rnd, rj0, rj1, cl);
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
    const uint64_t jbase = (uint64_t)n_rows * (s0 - tb.seg_off[jb]);
    const float ref = ref_thr[j];

    uint32_t npts, g_fixed = 0;
    int32_t cur_i;
    unsigned long long cost_cur, cap_c;
    float cur;
    int32_t gi = -1;
    if (PASS == 0) {
        npts = ns; cur_i = -1; cost_cur = 0; cur = 0.f; cap_c = cl.C;
    } else {
        gi = st.gi[jrel];
        npts = gi < 0 ? 0u : grid.n_cpu;
        g_fixed = gi < 0 ? 0u : st.g[jrel];
        cur_i = 0;
        cost_cur = cpu_cost(grid, 0, g_fixed);
        cap_c = st.free_c[rnd] + cost_cur;               // level 0 is already paid for
        cur = gi < 0 ? 0.f : vals[jbase + (uint64_t)(n_mem - 1) * ns + gi];
    }
    // amount s: its cost in the pass's resource and its value
    auto cost_of = [&](uint32_t s) -> unsigned long long {
        return PASS == 0 ? (unsigned long long)tb.seg_g[s0 + s] : cpu_cost(grid, s, g_fixed);
    };
    auto value_of = [&](uint32_t s) -> float {
        return PASS == 0 ? vals[jbase + (uint64_t)(n_mem - 1) * ns + s]
                         : vals[jbase + (uint64_t)(s * n_mem + n_mem - 1) * ns + gi];
    };
    auto affordable = [&](uint32_t s, unsigned long long cost) -> bool {
        if (PASS == 0) return cost <= cl.G && cpu_cost(grid, 0, (uint32_t)cost) <= cap_c;
        return cost <= cap_c;
    };

    uint32_t k = 0;
    float prev = __uint_as_float(0x7F800000u);
    while (k < H.width) {
        unsigned long long best = 0;
        for (uint32_t base = 0; base < npts; base += 64) {
            const uint32_t s = base + lane;
            if (s < npts && (int32_t)s > cur_i) {
                const unsigned long long cost = cost_of(s);
                if (affordable(s, cost)) {
                    const float v = value_of(s);
                    if (v > cur) {
                        float sl = (v - cur) / ref;
                        sl = sl / (float)(cost - cost_cur);
                        const unsigned long long c = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - s);
                        best = c > best ? c : best;
                    }
                }
            }
        }
        best = wave_max_u64(best);
        if (!(best >> 32)) break;
        const float top = __uint_as_float((uint32_t)(best >> 32));
        const uint32_t top_s = 0xFFFFFFFFu - (uint32_t)best;
        const unsigned long long top_cost = cost_of(top_s);
        prev = top < prev ? top : prev;
        if (lane == 0) {
            const size_t e = (size_t)k * H.stride + jrel;
            H.key[e] = __float_as_uint(prev);
            H.raw[e] = top;
            H.tgt[e] = (uint16_t)top_s;
            if (PASS == 0) {
                H.dg[e] = (uint32_t)(top_cost - cost_cur);
                H.dc[e] = cpu_cost(grid, 0, (uint32_t)top_cost) - (cost_cur ? cpu_cost(grid, 0, (uint32_t)cost_cur) : 0ull);
            } else {
                H.dg[e] = 0u;
                H.dc[e] = top_cost - cost_cur;
            }
        }
        cur = value_of(top_s);
        cur_i = (int32_t)top_s;
        cost_cur = top_cost;
        ++k;
    }
    if (k < H.width && lane == 0) H.key[(size_t)k * H.stride + jrel] = 0u;
}

// ------------------------------------------------------------------ one pass of a round
struct SelectShared {
    unsigned long long baseG, baseC;
    unsigned int prefix, done, thr;
    unsigned int histG[256];
    unsigned long long histC[256];
    unsigned long long red[PASS_WAVES];
};

// workgroup-wide maximum of a key; every thread gets the result
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long *red) {
    v = wave_max_u64(v);
    if ((threadIdx.x & 63u) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long m = red[0];
#pragma unroll
    for (int w = 1; w < PASS_WAVES; ++w) m = red[w] > m ? red[w] : m;
    __syncthreads();
    return m;
}

template <int PASS>
__global__ __launch_bounds__(PASS_THREADS) void k_pass(const float *__restrict__ ref_thr, TableDev tb, GridDev grid,
                                                       RoundArgs R, uint32_t jb, uint32_t max_jobs,
                                                       const float *__restrict__ vals, HullBuf H, JobState st) {
    extern __shared__ float lds_dyn[];
    __shared__ SelectShared sel;
    float *slope = lds_dyn;                                        // cached best step of each job (0 = none)
    uint16_t *tgt = reinterpret_cast<uint16_t *>(slope + max_jobs);   // its target (segment index or CPU level)
    uint16_t *aux = tgt + max_jobs;                                // PASS 0: GPUs the step adds; PASS 1: GPUs held
    int16_t *gi = reinterpret_cast<int16_t *>(aux + max_jobs);     // granted segment index, -1 = none
    uint16_t *ci = reinterpret_cast<uint16_t *>(gi + max_jobs);    // granted CPU level

    const uint32_t tid = threadIdx.x, rnd = blockIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(R, rnd, J0, J1, cl);
    const uint32_t nj = J1 - J0;
    const uint32_t jrel0 = J0 - jb;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem, m_top = n_mem - 1;
    const uint32_t seg_base = tb.seg_off[jb];
    unsigned long long freeG = PASS == 0 ? cl.G : 0ull;
    unsigned long long freeC = PASS == 0 ? cl.C : st.free_c[rnd];
    const uint32_t width = PASS == 0 ? H.width : (grid.n_cpu - 1 < H.width ? grid.n_cpu - 1 : H.width);

    for (uint32_t jl = tid; jl < nj; jl += PASS_THREADS) {
        if (PASS == 0) { gi[jl] = -1; ci[jl] = 0; }
        else { gi[jl] = (int16_t)st.gi[jrel0 + jl]; aux[jl] = (uint16_t)st.g[jrel0 + jl]; ci[jl] = 0; }
    }
    if (tid == 0) { sel.baseG = 0; sel.baseC = 0; sel.prefix = 0; sel.done = 0; sel.thr = 0; }
    __syncthreads();

    // ---- radix select: the largest set {key > thr} whose total cost fits
    for (int shift = 24; shift >= 0 && width > 0; shift -= 8) {
        for (uint32_t i = tid; i < 256; i += PASS_THREADS) { sel.histG[i] = 0; sel.histC[i] = 0; }
        __syncthreads();
        const uint32_t prefix = sel.prefix;
        for (uint32_t jl = tid; jl < nj; jl += PASS_THREADS) {
            for (uint32_t k = 0; k < width; ++k) {
                const size_t e = (size_t)k * H.stride + jrel0 + jl;
                const uint32_t key = H.key[e];
                if (!key) break;
                const uint32_t hi = shift == 24 ? 0u : key >> (shift + 8);
                if (hi < prefix) break;                        // keys only decrease along a walk
                if (hi == prefix) {
                    const uint32_t bin = (key >> shift) & 255u;
                    const uint32_t dg = H.dg[e];
                    const unsigned long long dc = H.dc[e];
                    if (dg) atomicAdd(&sel.histG[bin], dg);
                    if (dc) atomicAdd(&sel.histC[bin], dc);
                }
            }
        }
        __syncthreads();
        if (tid == 0) {
            unsigned long long cg = sel.baseG, cc = sel.baseC;
            int b = 255;
            while (b >= 0 && cg + sel.histG[b] <= freeG && cc + sel.histC[b] <= freeC) {
                cg += sel.histG[b]; cc += sel.histC[b]; --b;
            }
            sel.baseG = cg; sel.baseC = cc;
            if (b < 0) {                                       // everything under this prefix fits
                const unsigned long long lower = (unsigned long long)prefix << (shift + 8);
                sel.thr = lower ? (unsigned int)(lower - 1) : 0u;
                sel.done = 1;
            } else {
                sel.prefix = (prefix << 8) | (unsigned int)b;
                if (shift == 0) sel.thr = sel.prefix;          // this key's group does not fit as a whole
            }
        }
        __syncthreads();
        if (sel.done) break;
    }
    const uint32_t thr = sel.thr;
    freeG -= sel.baseG;
    freeC -= sel.baseC;

    // position of (job, row, segment) in the segment-layout arrays
    auto at = [&](uint32_t j, uint32_t c, uint32_t mi, uint32_t s) -> uint64_t {
        const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
        return (uint64_t)n_rows * (s0 - seg_base) + (uint64_t)(c * n_mem + mi) * ns + s;
    };
    // best step of local job jl under the current free capacity, from scratch
    auto best_step = [&](uint32_t jl) {
        const uint32_t j = J0 + jl;
        float top = 0.f;
        uint32_t top_t = 0, top_aux = 0;
        if (PASS == 0) {
            const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
            const int32_t cur_i = gi[jl];
            const uint32_t g_cur = cur_i < 0 ? 0u : tb.seg_g[s0 + cur_i];
            const uint64_t row = (uint64_t)n_rows * (s0 - seg_base) + (uint64_t)m_top * ns;   // CPU level 0
            const float cur = cur_i < 0 ? 0.f : vals[row + cur_i];
            const float ref = ref_thr[j];
            const unsigned long long c_cur = cur_i < 0 ? 0ull : cpu_cost(grid, 0, g_cur);
            for (uint32_t s = (uint32_t)(cur_i + 1); s < ns; ++s) {
                const uint32_t dg = tb.seg_g[s0 + s] - g_cur;
                if (dg > freeG) break;
                const float v = vals[row + s];
                if (!(v > cur)) continue;
                if (cpu_cost(grid, 0, g_cur + dg) - c_cur > freeC) continue;
                float sl = (v - cur) / ref;
                sl = sl / (float)dg;
                if (sl > top) { top = sl; top_t = s; top_aux = dg; }
            }
            aux[jl] = (uint16_t)top_aux;
        } else if (gi[jl] >= 0) {
            const uint32_t g = aux[jl], c0 = ci[jl], s_i = (uint32_t)gi[jl];
            const float cur = vals[at(j, c0, m_top, s_i)];
            const float ref = ref_thr[j];
            const unsigned long long have = cpu_cost(grid, c0, g);
            for (uint32_t c = c0 + 1; c < grid.n_cpu; ++c) {
                const unsigned long long dc = cpu_cost(grid, c, g) - have;
                if (dc > freeC) break;
                const float v = vals[at(j, c, m_top, s_i)];
                if (!(v > cur)) continue;
                float sl = (v - cur) / ref;
                sl = sl / (float)dc;
                if (sl > top) { top = sl; top_t = c; }
            }
        }
        slope[jl] = top;
        tgt[jl] = (uint16_t)top_t;
    };
    // CPUs a cached step of job jl costs
    auto step_cpus = [&](uint32_t jl) -> unsigned long long {
        if (PASS == 0)
            return grid.cpu_mode ? (unsigned long long)grid.cpu_levels[0] * aux[jl]
                                 : (gi[jl] < 0 ? (unsigned long long)grid.cpu_levels[0] : 0ull);
        return cpu_cost(grid, tgt[jl], aux[jl]) - cpu_cost(grid, ci[jl], aux[jl]);
    };

    // ---- apply the selected prefix of every walk; the next step of the walk,
    // if it still fits, is the job's best step, otherwise it is searched anew
    for (uint32_t jl = tid; jl < nj; jl += PASS_THREADS) {
        uint32_t k = 0;
        uint32_t key = 0;
        size_t e = 0;
        for (; k < width; ++k) {
            e = (size_t)k * H.stride + jrel0 + jl;
            key = H.key[e];
            if (!key || key <= thr) break;
            if (PASS == 0) gi[jl] = (int16_t)H.tgt[e]; else ci[jl] = H.tgt[e];
        }
        if (k == width) key = 0;
        if (!key) {                                            // the walk is over: nothing left to gain
            slope[jl] = 0.f; tgt[jl] = 0; if (PASS == 0) aux[jl] = 0;
        } else if (H.dg[e] <= freeG && H.dc[e] <= freeC) {
            slope[jl] = H.raw[e]; tgt[jl] = H.tgt[e]; if (PASS == 0) aux[jl] = (uint16_t)H.dg[e];
        } else {
            best_step(jl);
        }
    }
    __syncthreads();

    // ---- step by step on what is left
    for (;;) {
        unsigned long long k = 0;
        for (uint32_t jl = tid; jl < nj; jl += PASS_THREADS) {
            const unsigned long long c = ((unsigned long long)__float_as_uint(slope[jl]) << 32) | (0xFFFFFFFFu - jl);
            k = c > k ? c : k;
        }
        k = block_max_u64(k, sel.red);
        if (!(k >> 32)) break;                                  // no positive slope left
        const uint32_t jw = 0xFFFFFFFFu - (uint32_t)k;
        if (PASS == 0) freeG -= aux[jw];
        freeC -= step_cpus(jw);
        __syncthreads();                                        // everyone has read the winner's state
        if (tid == (jw % PASS_THREADS)) { if (PASS == 0) gi[jw] = (int16_t)tgt[jw]; else ci[jw] = tgt[jw]; }
        // cached steps that no longer fit, and the winner's next step, are recomputed
        for (uint32_t jl = tid; jl < nj; jl += PASS_THREADS) {
            bool redo = jl == jw;
            if (!redo && slope[jl] > 0.f) redo = (PASS == 0 && aux[jl] > freeG) || step_cpus(jl) > freeC;
            if (redo) best_step(jl);
        }
        __syncthreads();
    }

    for (uint32_t jl = tid; jl < nj; jl += PASS_THREADS) {
        if (PASS == 0) {
            const int32_t s_i = gi[jl];
            st.gi[jrel0 + jl] = s_i;
            st.g[jrel0 + jl] = s_i < 0 ? 0u : tb.seg_g[tb.seg_off[J0 + jl] + s_i];
        } else {
            st.ci[jrel0 + jl] = ci[jl];
        }
    }
    if (PASS == 0 && tid == 0) st.free_c[rnd] = freeC;
}

// ------------------------------------------------------------------ memory
// Wish of a job: the smallest tier that reaches its best throughput over all
// tiers.  The wishes are written as the result; k_mem_finish keeps them when
// all of them together stay 1 % below the round's host memory (then every job
// finds its wish still free when its turn comes: the float32 running remainder
// of the in-order rule drifts by far less), and redoes the round in job order
// otherwise.
__global__ __launch_bounds__(WISH_THREADS) void k_mem_wish(const float *__restrict__ ref_thr, TableDev tb,
                                                           GridDev grid, RoundArgs R, uint32_t jb,
                                                           const float *__restrict__ best_thr,
                                                           const uint32_t *__restrict__ best_plan, JobState st,
                                                           rk_assign *__restrict__ assign) {
    __shared__ double red[2][WISH_THREADS / 64];
    const uint32_t rnd = blockIdx.y, tid = threadIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(R, rnd, J0, J1, cl);
    const uint32_t jl = blockIdx.x * WISH_THREADS + tid;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    double cost_d = 0.0, val_d = 0.0;
    if (J0 + jl < J1) {
        const uint32_t j = J0 + jl, jrel = j - jb;
        rk_assign out = {0u, 0u, 0.f, RK_NO_PLAN, 0.f};
        const int32_t gi = st.gi[jrel];
        if (gi >= 0) {
            const uint32_t g = st.g[jrel], c_lvl = st.ci[jrel];
            const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
            const uint64_t base = (uint64_t)n_rows * (s0 - tb.seg_off[jb]) + (uint64_t)(c_lvl * n_mem) * ns + gi;
            float bv = 0.f;
            uint32_t bm = 0;
            for (uint32_t m = 0; m < n_mem; ++m) {
                const float v = best_thr[base + (uint64_t)m * ns];
                if (v > bv) { bv = v; bm = m; }
            }
            if (bv > 0.f) {
                float cost = grid.mem_levels_gb[bm];
                if (grid.mem_mode) cost = cost * (float)g;
                out.g = g;
                out.c = (uint32_t)cpu_cost(grid, c_lvl, g);
                out.mem_gb = cost;
                out.plan = best_plan[base + (uint64_t)bm * ns];
                out.thr = bv;
                cost_d = (double)cost;
                val_d = (double)bv / (double)ref_thr[j];
            }
        }
        assign[jrel] = out;
    }
    cost_d = wave_sum_f64(cost_d);
    val_d = wave_sum_f64(val_d);
    if ((tid & 63u) == 0) { red[0][tid >> 6] = cost_d; red[1][tid >> 6] = val_d; }
    __syncthreads();
    if (tid == 0) {
        double a = 0.0, b = 0.0;
        for (int w = 0; w < WISH_THREADS / 64; ++w) { a += red[0][w]; b += red[1][w]; }
        st.partial[((size_t)rnd * st.blocks_per_round + blockIdx.x) * 2 + 0] = a;
        st.partial[((size_t)rnd * st.blocks_per_round + blockIdx.x) * 2 + 1] = b;
    }
}

// One wavefront per round.
__global__ __launch_bounds__(64) void k_mem_finish(const float *__restrict__ ref_thr, TableDev tb, GridDev grid,
                                                   RoundArgs R, uint32_t jb, const float *__restrict__ best_thr,
                                                   const uint32_t *__restrict__ best_plan, JobState st,
                                                   rk_assign *__restrict__ assign, float *__restrict__ totals) {
    const uint32_t rnd = blockIdx.x, tid = threadIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(R, rnd, J0, J1, cl);
    const uint32_t nj = J1 - J0, jrel0 = J0 - jb;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    const uint32_t used_blocks = (nj + WISH_THREADS - 1) / WISH_THREADS;
    double wish = 0.0, val = 0.0;
    for (uint32_t b = tid; b < used_blocks; b += 64) {
        wish += st.partial[((size_t)rnd * st.blocks_per_round + b) * 2 + 0];
        val += st.partial[((size_t)rnd * st.blocks_per_round + b) * 2 + 1];
    }
    wish = wave_sum_f64(wish);
    val = wave_sum_f64(val);
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
            const uint32_t s0 = tb.seg_off[j];
            ns = tb.seg_off[j + 1] - s0;
            at0 = (uint64_t)n_rows * (s0 - tb.seg_off[jb]) + (uint64_t)(c_lvl * n_mem) * ns + (uint32_t)st.gi[jrel0 + jl];
            float bv = 0.f;
            uint32_t bm = 0;
#pragma unroll
            for (uint32_t m = 0; m < RK_MAX_MEM_LEVELS; ++m) {
                if (m < n_mem) {
                    const float v = best_thr[at0 + (uint64_t)m * ns];
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
                    out.plan = best_plan[at0 + (uint64_t)bm * ns];
                    out.thr = v;
                    sum += (double)v / (double)ref_thr[J0 + jl];
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

template <typename T>
int32_t scratch_typed(rk_ctx *ctx, int slot, size_t count, T **out) {
    return rk_scratch(ctx, slot, count * sizeof(T), reinterpret_cast<void **>(out));
}

}  // namespace

int32_t rk_launch_allocate(rk_ctx *ctx, const float *ref_thr, const TableDev &tb, const rk_alloc_grid *grid,
                           uint32_t n_rounds, const uint32_t *d_round_off, const rk_cluster *d_clusters,
                           const rk_cluster *one_cluster, uint32_t jb, uint32_t n_jobs, uint32_t max_jobs,
                           uint32_t max_segs_per_job, const float *best_thr, const uint32_t *best_plan,
                           const float *curve_thr, rk_assign *assign, float *totals) {
    if (n_rounds == 0) return RK_OK;
    if (max_jobs > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "a round has %u jobs, the allocation kernels take up to %u", max_jobs,
                       RK_MAX_JOBS_PER_ROUND);
    int32_t rc;
    HullBuf H;
    H.stride = n_jobs ? n_jobs : 1;
    H.width = max_segs_per_job > grid->n_cpu ? max_segs_per_job : grid->n_cpu;   // the longest walk of either pass
    if (H.width == 0) H.width = 1;
    const size_t entries = (size_t)H.stride * H.width;
    if ((rc = scratch_typed(ctx, SL_HULL_KEY, entries, &H.key))) return rc;
    if ((rc = scratch_typed(ctx, SL_HULL_RAW, entries, &H.raw))) return rc;
    if ((rc = scratch_typed(ctx, SL_HULL_TGT, entries, &H.tgt))) return rc;
    if ((rc = scratch_typed(ctx, SL_HULL_DG, entries, &H.dg))) return rc;
    if ((rc = scratch_typed(ctx, SL_HULL_DC, entries, &H.dc))) return rc;
    JobState st;
    st.blocks_per_round = (max_jobs + WISH_THREADS - 1) / WISH_THREADS;
    if (st.blocks_per_round == 0) st.blocks_per_round = 1;
    if ((rc = scratch_typed(ctx, SL_ST_GI, (size_t)H.stride, &st.gi))) return rc;
    if ((rc = scratch_typed(ctx, SL_ST_G, (size_t)H.stride, &st.g))) return rc;
    if ((rc = scratch_typed(ctx, SL_ST_CI, (size_t)H.stride, &st.ci))) return rc;
    if ((rc = scratch_typed(ctx, SL_ST_FREEC, (size_t)n_rounds, &st.free_c))) return rc;
    if ((rc = scratch_typed(ctx, SL_ST_PARTIAL, (size_t)n_rounds * st.blocks_per_round * 2, &st.partial))) return rc;

    const GridDev gd = grid_dev(grid);
    RoundArgs R;
    R.round_off = d_round_off; R.clusters = d_clusters; R.n_rounds = n_rounds;
    R.inline_one = one_cluster ? 1u : 0u;
    R.off0 = jb; R.off1 = jb + n_jobs;
    R.cl = one_cluster ? *one_cluster : rk_cluster{0u, 0u, 0.f};

    const uint32_t mj = max_jobs ? ((max_jobs + 1u) & ~1u) : 2u;
    const size_t lds = (size_t)mj * (4 + 2 + 2 + 2 + 2);
    static bool raised[64] = {};
    if (lds > 48 * 1024 && !raised[ctx->device & 63]) {
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_pass<0>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024));
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_pass<1>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024));
        raised[ctx->device & 63] = true;
    }
    const uint32_t hull_blocks = (n_jobs + (HULL_THREADS / 64) - 1) / (HULL_THREADS / 64);
    hipStream_t s = ctx->stream;
    if (n_jobs > 0) {
        k_hull<0><<<hull_blocks, HULL_THREADS, 0, s>>>(ref_thr, tb, gd, R, jb, curve_thr, st, H);
        RK_CHECK_LAUNCH(ctx, "k_hull<gpu>");
    }
    k_pass<0><<<n_rounds, PASS_THREADS, lds, s>>>(ref_thr, tb, gd, R, jb, mj, curve_thr, H, st);
    RK_CHECK_LAUNCH(ctx, "k_pass<gpu>");
    if (n_jobs > 0) {
        k_hull<1><<<hull_blocks, HULL_THREADS, 0, s>>>(ref_thr, tb, gd, R, jb, best_thr, st, H);
        RK_CHECK_LAUNCH(ctx, "k_hull<cpu>");
    }
    k_pass<1><<<n_rounds, PASS_THREADS, lds, s>>>(ref_thr, tb, gd, R, jb, mj, best_thr, H, st);
    RK_CHECK_LAUNCH(ctx, "k_pass<cpu>");
    if (max_jobs > 0) {
        k_mem_wish<<<dim3(st.blocks_per_round, n_rounds), WISH_THREADS, 0, s>>>(ref_thr, tb, gd, R, jb, best_thr,
                                                                                best_plan, st, assign);
        RK_CHECK_LAUNCH(ctx, "k_mem_wish");
    }
    k_mem_finish<<<n_rounds, 64, 0, s>>>(ref_thr, tb, gd, R, jb, best_thr, best_plan, st, assign, totals);
    RK_CHECK_LAUNCH(ctx, "k_mem_finish");
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
    if (!cluster || !total) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (je > jb && (!ref_thr || !best_thr || !best_plan || !curve_thr || !assign))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (!(cluster->host_mem_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "host_mem_gb negative or NaN");
    if (table->max_segs_per_job > 32767u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 32767 segments per job");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    return rk_launch_allocate(ctx, ref_thr, table_dev(table), grid, 1, nullptr, nullptr, cluster, jb, je - jb, je - jb,
                              table->max_segs_per_job, best_thr, best_plan, curve_thr, assign, total);
}
