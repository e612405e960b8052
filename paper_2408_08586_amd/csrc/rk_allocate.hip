// Greedy marginal-gain allocation over the resource sensitivity curves
// (paper Sec. 5.2: prefer the jobs that gain the most per unit of resource,
// GPU slopes before CPU slopes; memory is granted last from the chosen plan's
// estimate).  One workgroup per scheduling round.
//
// The rule is sequential: repeatedly take the (job, larger amount) with the
// highest float32 slope ((v1 - v0) / ref_thr) / delta among the steps that
// still fit; ties go to the smaller amount, then to the lower job index.
// It is evaluated without running every step in sequence:
//
//  1. Each job's steps, were capacity never short, form a fixed walk over the
//     upper hull of its curve.  With each slope replaced by the running
//     minimum of the walk, the sequential order is the descending order of
//     these keys (then job, then position in the walk).
//  2. A radix select over the key bits finds the largest key threshold whose
//     whole set of steps fits the capacity; that set is a prefix of the
//     sequential order and is applied at once.
//  3. From there the plain step-by-step loop runs on the little capacity that
//     is left (a workgroup-wide argmax over cached per-job best steps).
//
// Memory: when the tiers every job would like fit with margin, all are
// granted in parallel; otherwise one wavefront takes the decisions in job
// order.
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int ALLOC_THREADS = 1024;
constexpr int ALLOC_WAVES = ALLOC_THREADS / 64;
constexpr int HULL_THREADS = 256;

struct HullBuf {             // walk steps, entry (k, job) at k*stride + job (job relative to the call's first job)
    uint32_t *key;           // float bits of the running-minimum slope; 0 ends a walk
    uint16_t *dg;            // GPU pass: GPUs the step adds
    uint16_t *tgt;           // target: segment index (GPU pass) or CPU level (CPU pass)
    uint32_t stride, width;
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

struct AllocLds {
    float *slope;        // cached best step of each job (0 = none)
    uint16_t *tgt;       // its target: segment index (GPU pass) or CPU level (CPU pass)
    uint16_t *aux;       // GPU pass: GPUs the step needs; CPU pass: GPUs the job holds
    int16_t *gi;         // granted segment index, -1 = no GPUs
    uint16_t *ci;        // granted CPU level
};

__device__ __forceinline__ unsigned long long cpu_cost(const GridDev &G, uint32_t ci, uint32_t g) {
    return G.cpu_mode ? (unsigned long long)G.cpu_levels[ci] * g : (unsigned long long)G.cpu_levels[ci];
}

// ------------------------------------------------------------------ hull walks of the GPU pass
// One thread per job: the steps the job takes when capacity is never short
// (only amounts beyond the whole cluster are excluded), lowest CPU level,
// highest memory tier.
__global__ __launch_bounds__(HULL_THREADS) void k_hull_gpu(
    const float *__restrict__ ref_thr, TableDev tb, GridDev grid, RoundArgs R, uint32_t jb,
    const float *__restrict__ curve_thr, HullBuf H) {
    const uint32_t jrel = blockIdx.x * HULL_THREADS + threadIdx.x;
    if (jrel >= H.stride) return;
    const uint32_t j = jb + jrel;
    uint32_t lo = 0, hi = R.n_rounds;                     // round of the job: last r with round_off[r] <= j
    while (!R.inline_one && hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (R.round_off[mid] <= j) lo = mid; else hi = mid;
    }
    uint32_t rj0, rj1;
    rk_cluster rcl;
    round_of(R, lo, rj0, rj1, rcl);
    const unsigned long long capG = rcl.G, capC = rcl.C;
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem;
    const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
    const uint64_t row = (uint64_t)n_rows * (s0 - tb.seg_off[jb]) + (uint64_t)(n_mem - 1) * ns;   // ci = 0, top tier
    const float ref = ref_thr[j];
    int32_t cur_i = -1;
    uint32_t g_cur = 0, k = 0;
    float cur = 0.f, prev = __uint_as_float(0x7F800000u);
    while (k < H.width) {
        float top = 0.f;
        uint32_t top_s = 0, top_g = 0;
        for (uint32_t s = (uint32_t)(cur_i + 1); s < ns; ++s) {
            const uint32_t g = tb.seg_g[s0 + s];
            if (g > capG) break;
            const float v = curve_thr[row + s];
            if (!(v > cur)) continue;
            if (cpu_cost(grid, 0, g) > capC) continue;
            float sl = (v - cur) / ref;
            sl = sl / (float)(g - g_cur);
            if (sl > top) { top = sl; top_s = s; top_g = g; }
        }
        if (!(top > 0.f)) break;
        prev = top < prev ? top : prev;
        H.key[(size_t)k * H.stride + jrel] = __float_as_uint(prev);
        H.dg[(size_t)k * H.stride + jrel] = (uint16_t)(top_g - g_cur);
        H.tgt[(size_t)k * H.stride + jrel] = (uint16_t)top_s;
        cur = curve_thr[row + top_s];
        cur_i = (int32_t)top_s;
        g_cur = top_g;
        ++k;
    }
    if (k < H.width) H.key[(size_t)k * H.stride + jrel] = 0u;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// workgroup-wide maximum of a key; every thread gets the result
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long *red) {
    v = wave_max_u64(v);
    if ((threadIdx.x & 63u) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long m = red[0];
#pragma unroll
    for (int w = 1; w < ALLOC_WAVES; ++w) m = red[w] > m ? red[w] : m;
    __syncthreads();
    return m;
}

__device__ __forceinline__ double block_sum_f64(double v, double *red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63u) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < ALLOC_WAVES; ++w) s += red[w];
    __syncthreads();
    return s;
}

struct SelectShared {
    unsigned long long baseG, baseC;
    unsigned int prefix, done, thr;
    unsigned int histG[256];
    unsigned long long histC[256];
};

__global__ __launch_bounds__(ALLOC_THREADS) void k_allocate(
    const float *__restrict__ ref_thr, TableDev tb, GridDev grid, RoundArgs R, uint32_t jb, uint32_t max_jobs,
    const float *__restrict__ best_thr, const uint32_t *__restrict__ best_plan,
    const float *__restrict__ curve_thr, HullBuf H, rk_assign *__restrict__ assign, float *__restrict__ totals) {
    extern __shared__ unsigned long long lds_raw[];
    __shared__ SelectShared sel;
    unsigned long long *red = lds_raw;                                        // [ALLOC_WAVES]
    AllocLds S;
    S.slope = reinterpret_cast<float *>(red + ALLOC_WAVES);
    S.tgt = reinterpret_cast<uint16_t *>(S.slope + max_jobs);
    S.aux = S.tgt + max_jobs;
    S.gi = reinterpret_cast<int16_t *>(S.aux + max_jobs);
    S.ci = reinterpret_cast<uint16_t *>(S.gi + max_jobs);

    const uint32_t tid = threadIdx.x, rnd = blockIdx.x;
    uint32_t J0, J1;
    rk_cluster cl;
    round_of(R, rnd, J0, J1, cl);
    const uint32_t nj = J1 - J0;
    const uint32_t jrel0 = J0 - jb;                       // first job of the round in the hull buffer
    const uint32_t n_mem = grid.n_mem, n_rows = grid.n_cpu * n_mem, m_top = n_mem - 1;
    const uint32_t seg_base = tb.seg_off[jb];
    unsigned long long freeG = cl.G, freeC = cl.C;

    // position of (job, row, segment) in the segment-layout arrays
    auto at = [&](uint32_t j, uint32_t ci, uint32_t mi, uint32_t s) -> uint64_t {
        const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
        return (uint64_t)n_rows * (s0 - seg_base) + (uint64_t)(ci * n_mem + mi) * ns + s;
    };

    // Radix select over the walk keys of the round: finds the largest set
    // {key > thr} whose total cost fits (capG, capC) and leaves the totals in
    // sel.baseG / sel.baseC.  step_cost(jl, k, prev_tgt, tgt, dg&, dc&).
    auto select_threshold = [&](auto step_cost, unsigned long long capG, unsigned long long capC, uint32_t width) {
        if (tid == 0) { sel.baseG = 0; sel.baseC = 0; sel.prefix = 0; sel.done = 0; sel.thr = 0; }
        __syncthreads();
        for (int shift = 24; shift >= 0; shift -= 8) {
            for (uint32_t i = tid; i < 256; i += ALLOC_THREADS) { sel.histG[i] = 0; sel.histC[i] = 0; }
            __syncthreads();
            const uint32_t prefix = sel.prefix;
            for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
                uint32_t prev_tgt = 0;
                for (uint32_t k = 0; k < width; ++k) {
                    const size_t e = (size_t)k * H.stride + jrel0 + jl;
                    const uint32_t key = H.key[e];
                    if (!key) break;
                    const uint32_t tgt = H.tgt[e];
                    const uint32_t hi = shift == 24 ? 0u : key >> (shift + 8);
                    if (hi < prefix) break;                    // keys only decrease along a walk
                    if (hi == prefix) {
                        unsigned long long dg, dc;
                        step_cost(jl, k, prev_tgt, tgt, e, dg, dc);
                        const uint32_t bin = (key >> shift) & 255u;
                        if (dg) atomicAdd(&sel.histG[bin], (unsigned int)dg);
                        if (dc) atomicAdd(&sel.histC[bin], dc);
                    }
                    prev_tgt = tgt;
                }
            }
            __syncthreads();
            if (tid == 0) {
                unsigned long long cg = sel.baseG, cc = sel.baseC;
                int b = 255;
                while (b >= 0 && cg + sel.histG[b] <= capG && cc + sel.histC[b] <= capC) {
                    cg += sel.histG[b]; cc += sel.histC[b]; --b;
                }
                sel.baseG = cg; sel.baseC = cc;
                if (b < 0) {                                   // everything under this prefix fits
                    const unsigned long long lower = (unsigned long long)prefix << (shift + 8);
                    sel.thr = lower ? (unsigned int)(lower - 1) : 0u;
                    sel.done = 1;
                } else {
                    sel.prefix = (prefix << 8) | (unsigned int)b;
                    if (shift == 0) sel.thr = sel.prefix;      // this key's group does not fit as a whole
                }
            }
            __syncthreads();
            if (sel.done) break;
        }
    };

    // ================================================================ GPU pass
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) { S.gi[jl] = -1; S.ci[jl] = 0; }
    {
        auto gpu_cost = [&](uint32_t, uint32_t k, uint32_t, uint32_t, size_t e, unsigned long long &dg,
                            unsigned long long &dc) {
            dg = H.dg[e];
            dc = grid.cpu_mode ? (unsigned long long)grid.cpu_levels[0] * dg
                               : (k == 0 ? (unsigned long long)grid.cpu_levels[0] : 0ull);
        };
        const uint32_t width = H.width;
        select_threshold(gpu_cost, freeG, freeC, width);
        const uint32_t thr = sel.thr;
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            for (uint32_t k = 0; k < width; ++k) {
                const size_t e = (size_t)k * H.stride + jrel0 + jl;
                const uint32_t key = H.key[e];
                if (!key || key <= thr) break;
                S.gi[jl] = (int16_t)H.tgt[e];
            }
        }
        freeG -= sel.baseG;
        freeC -= sel.baseC;
    }

    // best GPU step of local job jl under the current free capacity
    auto gpu_step = [&](uint32_t jl) {
        const uint32_t j = J0 + jl;
        const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
        const int32_t cur_i = S.gi[jl];
        const uint32_t g_cur = cur_i < 0 ? 0u : tb.seg_g[s0 + cur_i];
        const uint64_t row = (uint64_t)n_rows * (s0 - seg_base) + (uint64_t)m_top * ns;   // ci = 0
        const float cur = cur_i < 0 ? 0.f : curve_thr[row + cur_i];
        const float ref = ref_thr[j];
        const unsigned long long c_cur = cur_i < 0 ? 0ull : cpu_cost(grid, 0, g_cur);
        float top = 0.f;
        uint32_t top_s = 0, top_dg = 0;
        for (uint32_t s = (uint32_t)(cur_i + 1); s < ns; ++s) {
            const uint32_t dg = tb.seg_g[s0 + s] - g_cur;
            if (dg > freeG) break;
            const float v = curve_thr[row + s];
            if (!(v > cur)) continue;
            if (cpu_cost(grid, 0, g_cur + dg) - c_cur > freeC) continue;
            float sl = (v - cur) / ref;
            sl = sl / (float)dg;
            if (sl > top) { top = sl; top_s = s; top_dg = dg; }
        }
        S.slope[jl] = top;
        S.tgt[jl] = (uint16_t)top_s;
        S.aux[jl] = (uint16_t)top_dg;
    };
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) gpu_step(jl);
    __syncthreads();
    for (;;) {
        unsigned long long k = 0;
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            const unsigned long long c = ((unsigned long long)__float_as_uint(S.slope[jl]) << 32) | (0xFFFFFFFFu - jl);
            k = c > k ? c : k;
        }
        k = block_max_u64(k, red);
        if (!(k >> 32)) break;                                  // no positive slope left
        const uint32_t jw = 0xFFFFFFFFu - (uint32_t)k;
        const uint32_t dg = S.aux[jw];
        const bool first = S.gi[jw] < 0;
        const unsigned long long dc = grid.cpu_mode ? (unsigned long long)grid.cpu_levels[0] * dg
                                                    : (first ? (unsigned long long)grid.cpu_levels[0] : 0ull);
        freeG -= dg;
        freeC -= dc;
        __syncthreads();                                        // everyone has read the winner's state
        if (tid == (jw % ALLOC_THREADS)) S.gi[jw] = (int16_t)S.tgt[jw];
        // cached steps that no longer fit, and the winner's next step, are recomputed
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            bool redo = jl == jw;
            if (!redo && S.slope[jl] > 0.f) {
                const uint32_t need_g = S.aux[jl];
                const unsigned long long need_c = grid.cpu_mode ? (unsigned long long)grid.cpu_levels[0] * need_g
                                                                : (S.gi[jl] < 0 ? (unsigned long long)grid.cpu_levels[0] : 0ull);
                redo = need_g > freeG || need_c > freeC;
            }
            if (redo) gpu_step(jl);
        }
        __syncthreads();
    }

    // ================================================================ CPU pass
    // S.aux now holds the GPUs each job was granted.
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
        const int32_t cur_i = S.gi[jl];
        S.aux[jl] = cur_i < 0 ? (uint16_t)0 : (uint16_t)tb.seg_g[tb.seg_off[J0 + jl] + cur_i];
    }
    const uint32_t cpu_width = grid.n_cpu - 1 < H.width ? grid.n_cpu - 1 : H.width;
    // walks over the CPU levels at the granted GPU count (each thread writes and later reads its own jobs)
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
        const int32_t cur_i = S.gi[jl];
        uint32_t k = 0;
        if (cur_i >= 0) {
            const uint32_t j = J0 + jl, g = S.aux[jl];
            const float ref = ref_thr[j];
            const unsigned long long base_cost = cpu_cost(grid, 0, g);
            uint32_t c0 = 0;
            float cur = best_thr[at(j, 0, m_top, (uint32_t)cur_i)];
            float prev = __uint_as_float(0x7F800000u);
            while (k < cpu_width) {
                float top = 0.f;
                uint32_t top_c = 0;
                const unsigned long long have = cpu_cost(grid, c0, g);
                for (uint32_t c = c0 + 1; c < grid.n_cpu; ++c) {
                    if (cpu_cost(grid, c, g) - base_cost > freeC) break;
                    const float v = best_thr[at(j, c, m_top, (uint32_t)cur_i)];
                    if (!(v > cur)) continue;
                    float sl = (v - cur) / ref;
                    sl = sl / (float)(cpu_cost(grid, c, g) - have);
                    if (sl > top) { top = sl; top_c = c; }
                }
                if (!(top > 0.f)) break;
                prev = top < prev ? top : prev;
                const size_t e = (size_t)k * H.stride + jrel0 + jl;
                H.key[e] = __float_as_uint(prev);
                H.tgt[e] = (uint16_t)top_c;
                cur = best_thr[at(j, top_c, m_top, (uint32_t)cur_i)];
                c0 = top_c;
                ++k;
            }
        }
        if (k < H.width) H.key[(size_t)k * H.stride + jrel0 + jl] = 0u;
    }
    if (cpu_width > 0) {
        auto cpu_step_cost = [&](uint32_t jl, uint32_t, uint32_t prev_tgt, uint32_t tgt, size_t, unsigned long long &dg,
                                 unsigned long long &dc) {
            dg = 0;
            dc = cpu_cost(grid, tgt, S.aux[jl]) - cpu_cost(grid, prev_tgt, S.aux[jl]);
        };
        select_threshold(cpu_step_cost, 0ull, freeC, cpu_width);
        const uint32_t thr = sel.thr;
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            for (uint32_t k = 0; k < cpu_width; ++k) {
                const size_t e = (size_t)k * H.stride + jrel0 + jl;
                const uint32_t key = H.key[e];
                if (!key || key <= thr) break;
                S.ci[jl] = H.tgt[e];
            }
        }
        freeC -= sel.baseC;
    }
    auto cpu_step = [&](uint32_t jl) {
        const int32_t cur_i = S.gi[jl];
        float top = 0.f;
        uint32_t top_c = 0;
        if (cur_i >= 0) {
            const uint32_t j = J0 + jl, g = S.aux[jl], c0 = S.ci[jl];
            const float cur = best_thr[at(j, c0, m_top, (uint32_t)cur_i)];
            const float ref = ref_thr[j];
            const unsigned long long have = cpu_cost(grid, c0, g);
            for (uint32_t c = c0 + 1; c < grid.n_cpu; ++c) {
                const unsigned long long dc = cpu_cost(grid, c, g) - have;
                if (dc > freeC) break;
                const float v = best_thr[at(j, c, m_top, (uint32_t)cur_i)];
                if (!(v > cur)) continue;
                float sl = (v - cur) / ref;
                sl = sl / (float)dc;
                if (sl > top) { top = sl; top_c = c; }
            }
        }
        S.slope[jl] = top;
        S.tgt[jl] = (uint16_t)top_c;
    };
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) cpu_step(jl);
    __syncthreads();
    for (;;) {
        unsigned long long k = 0;
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            const unsigned long long c = ((unsigned long long)__float_as_uint(S.slope[jl]) << 32) | (0xFFFFFFFFu - jl);
            k = c > k ? c : k;
        }
        k = block_max_u64(k, red);
        if (!(k >> 32)) break;
        const uint32_t jw = 0xFFFFFFFFu - (uint32_t)k;
        freeC -= cpu_cost(grid, S.tgt[jw], S.aux[jw]) - cpu_cost(grid, S.ci[jw], S.aux[jw]);
        __syncthreads();
        if (tid == (jw % ALLOC_THREADS)) S.ci[jw] = S.tgt[jw];
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            bool redo = jl == jw;
            if (!redo && S.slope[jl] > 0.f)
                redo = cpu_cost(grid, S.tgt[jl], S.aux[jl]) - cpu_cost(grid, S.ci[jl], S.aux[jl]) > freeC;
            if (redo) cpu_step(jl);
        }
        __syncthreads();
    }

    // ================================================================ memory
    // Wish of a job: the smallest tier that reaches its best throughput over
    // all tiers.  If all wishes together stay 1 % below the host memory, every
    // job finds its wish still free when its turn comes (the float32 running
    // remainder drifts by far less), so the in-order rule grants exactly the
    // wishes and they are written in parallel.
    double wish_sum = 0.0;
    for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
        if (S.gi[jl] < 0) continue;
        const uint32_t j = J0 + jl, g = S.aux[jl];
        float bv = 0.f;
        uint32_t bm = 0;
        for (uint32_t m = 0; m < n_mem; ++m) {
            const float v = best_thr[at(j, S.ci[jl], m, (uint32_t)S.gi[jl])];
            if (v > bv) { bv = v; bm = m; }
        }
        if (bv > 0.f) {
            float cost = grid.mem_levels_gb[bm];
            if (grid.mem_mode) cost = cost * (float)g;
            wish_sum += (double)cost;
        }
    }
    wish_sum = block_sum_f64(wish_sum, reinterpret_cast<double *>(red));
    if (wish_sum <= 0.99 * (double)cl.host_mem_gb) {
        double sum = 0.0;
        for (uint32_t jl = tid; jl < nj; jl += ALLOC_THREADS) {
            rk_assign out = {0u, 0u, 0.f, RK_NO_PLAN, 0.f};
            if (S.gi[jl] >= 0) {
                const uint32_t j = J0 + jl, g = S.aux[jl], c_lvl = S.ci[jl], s_i = (uint32_t)S.gi[jl];
                float bv = 0.f;
                uint32_t bm = 0;
                for (uint32_t m = 0; m < n_mem; ++m) {
                    const float v = best_thr[at(j, c_lvl, m, s_i)];
                    if (v > bv) { bv = v; bm = m; }
                }
                if (bv > 0.f) {
                    float cost = grid.mem_levels_gb[bm];
                    if (grid.mem_mode) cost = cost * (float)g;
                    out.g = g;
                    out.c = (uint32_t)cpu_cost(grid, c_lvl, g);
                    out.mem_gb = cost;
                    out.plan = best_plan[at(j, c_lvl, bm, s_i)];
                    out.thr = bv;
                    sum += (double)bv / (double)ref_thr[j];
                }
            }
            assign[jrel0 + jl] = out;
        }
        sum = block_sum_f64(sum, reinterpret_cast<double *>(red));
        if (tid == 0) totals[rnd] = (float)sum;
        return;
    }
    // in job order, by the first wavefront: lanes load a batch of 64 jobs,
    // then take their decisions one after the other
    if (tid < 64) {
        float freeM = cl.host_mem_gb;
        double sum = 0.0;
        for (uint32_t base = 0; base < nj; base += 64) {
            const uint32_t jl = base + tid;
            const bool have = jl < nj && S.gi[jl] >= 0;
            uint32_t g = 0, c_lvl = 0, s_i = 0, j = 0;
            unsigned long long choice = 0;      // 4 bits per prefix length: best tier among tiers 0..k
            uint32_t valid = 0;                 // bit k: that best throughput is positive
            float thr_m[RK_MAX_MEM_LEVELS];
#pragma unroll
            for (uint32_t m = 0; m < RK_MAX_MEM_LEVELS; ++m) thr_m[m] = 0.f;
            if (have) {
                j = J0 + jl; g = S.aux[jl]; c_lvl = S.ci[jl]; s_i = (uint32_t)S.gi[jl];
                float bv = 0.f;
                uint32_t bm = 0;
#pragma unroll
                for (uint32_t m = 0; m < RK_MAX_MEM_LEVELS; ++m) {
                    if (m < n_mem) {
                        const float v = best_thr[at(j, c_lvl, m, s_i)];
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
                        out.plan = best_plan[at(j, c_lvl, bm, s_i)];
                        out.thr = v;
                        sum += (double)v / (double)ref_thr[j];
                    }
                }
                spent = __shfl(spent, (int)turn, 64);
                freeM = freeM - spent;
            }
            if (jl < nj) assign[jrel0 + jl] = out;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (tid == 0) totals[rnd] = (float)sum;
    }
}

}  // namespace

int32_t rk_launch_allocate(rk_ctx *ctx, const float *ref_thr, const TableDev &tb, const rk_alloc_grid *grid,
                           uint32_t n_rounds, const uint32_t *d_round_off, const rk_cluster *d_clusters,
                           const rk_cluster *one_cluster, uint32_t jb, uint32_t n_jobs, uint32_t max_jobs,
                           uint32_t max_segs_per_job,
                           const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                           rk_assign *assign, float *totals) {
    if (n_rounds == 0) return RK_OK;
    if (max_jobs > RK_MAX_JOBS_PER_ROUND)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "a round has %u jobs, the allocation kernel takes up to %u", max_jobs,
                       RK_MAX_JOBS_PER_ROUND);
    // walk buffers: width = the longest possible walk of either pass
    HullBuf H;
    H.stride = n_jobs ? n_jobs : 1;
    H.width = max_segs_per_job > grid->n_cpu ? max_segs_per_job : grid->n_cpu;
    if (H.width == 0) H.width = 1;
    const size_t entries = (size_t)H.stride * H.width;
    int32_t rc;
    if ((rc = rk_scratch(ctx, SL_HULL_KEY, entries * 4, (void **)&H.key))) return rc;
    if ((rc = rk_scratch(ctx, SL_HULL_DG, entries * 2, (void **)&H.dg))) return rc;
    if ((rc = rk_scratch(ctx, SL_HULL_TGT, entries * 2, (void **)&H.tgt))) return rc;
    const GridDev gd = grid_dev(grid);
    RoundArgs R;
    R.round_off = d_round_off; R.clusters = d_clusters; R.n_rounds = n_rounds;
    R.inline_one = one_cluster ? 1u : 0u;
    R.off0 = jb; R.off1 = jb + n_jobs;
    R.cl = one_cluster ? *one_cluster : rk_cluster{0u, 0u, 0.f};
    if (n_jobs > 0) {
        k_hull_gpu<<<(n_jobs + HULL_THREADS - 1) / HULL_THREADS, HULL_THREADS, 0, ctx->stream>>>(
            ref_thr, tb, gd, R, jb, curve_thr, H);
        RK_CHECK_LAUNCH(ctx, "k_hull_gpu");
    }
    const uint32_t mj = max_jobs ? ((max_jobs + 1u) & ~1u) : 2u;
    const size_t lds = ALLOC_WAVES * 8 + (size_t)mj * (4 + 2 + 2 + 2 + 2);
    static bool raised[64] = {};
    if (lds > 48 * 1024 && !raised[ctx->device & 63]) {
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_allocate),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 156 * 1024));
        raised[ctx->device & 63] = true;
    }
    k_allocate<<<n_rounds, ALLOC_THREADS, lds, ctx->stream>>>(ref_thr, tb, gd, R, jb, mj, best_thr, best_plan,
                                                             curve_thr, H, assign, totals);
    RK_CHECK_LAUNCH(ctx, "k_allocate");
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
