// Node-level placement of an allocation (paper Sec. 5.2, Algorithm 1,
// ScheduleJob: a job walks the nodes in order, takes what each node has free
// and records {node, resources}).
//
// The rule is sequential: what a job finds depends on what the jobs before it
// took.  One workgroup does it in two stages:
//
//  1. All jobs at once, assuming only GPUs bind.  Then first fit in node order
//     is the jobs laid end to end on the nodes' GPU slots: job j covers slots
//     [S_j, S_j + g_j) with S the prefix sum of the GPU counts, and its parts
//     follow from the node boundaries inside that range.  While the parts are
//     written, every node adds up the CPUs its parts would have needed to be
//     free (ceil(c*k/g) each, an upper bound of what they book) and their
//     memory.  If on every node these sums stay within the node (memory with
//     0.1 % to spare for the rounding of the float32 remainder), no job could
//     have met a node short of CPUs or memory, and the result stands.
//  2. Otherwise the first wavefront redoes the round job by job: lanes take
//     one node each, 64 nodes at a time from the first node that still has a
//     free GPU; a lane finds the most GPUs its node can give, a prefix sum
//     over the lanes cuts the offers at what the job still lacks, and the
//     parts are booked only when the whole amount has been found.
//
// rk_place_plans adds what Algorithm 1 does with a placement: a job that does
// not find its amount falls back to its next smaller valid GPU count (k_place
// with a Retry), and the plan of every placed job is searched again among the
// plans of its GPU count under the bandwidths of the actual node split
// (k_replan).
#include "rk_internal.h"
#include "rk_model.h"

namespace {

constexpr int PLACE_THREADS = 512;
constexpr int PLACE_WAVES = PLACE_THREADS / 64;

// Fall-back of a job that does not find its amount (on != 0): the next smaller GPU count of its list, not below
// its floor, that has a feasible plan at the job's CPU level and memory tier; CPUs and memory follow the grid.
struct Retry {
    uint32_t on;
    const uint32_t *seg_off, *seg_g;
    const float *best_thr;   // segment layout of all jobs
    const int32_t *min_seg;  // per job, may be null; -1 = no floor
    GridDev grid;
};

// An earlier placement of the same jobs: a job whose amounts are what its earlier parts add up to keeps them.
struct Keep {
    const uint32_t *prev_off;            // n_jobs + 1 offsets into prev_entries; null: every node starts empty
    const rk_place_entry *prev_entries;
    uint8_t *flag;                       // scratch, per job: keeps its parts
};

struct PlaceArgs {
    uint32_t n_jobs, n_nodes, gpn, cpn;
    float mpn;
    const rk_assign *assign;
    uint32_t *place_off;
    rk_place_entry *entries;
    uint32_t *status;
    uint32_t *result;        // n_entries, n_placed, n_failed, in_order
    Retry retry;
    Keep keep;
};

// Where a record's amounts sit in the job's lists: segment of the GPU count, CPU level, memory tier (-1: not
// found).  Evaluated by a whole wavefront, the result is uniform.
struct GridPos { int32_t s, ci, mi; };
__device__ __forceinline__ GridPos locate(const GridDev &G, const uint32_t *seg_g, uint32_t s_off, uint32_t ns, uint32_t g,
                                          uint32_t c, float mem, uint32_t lane) {
    GridPos P = {-1, -1, -1};
    for (uint32_t base = 0; base < ns && P.s < 0; base += 64) {
        const uint32_t s = base + lane;
        const unsigned long long hit = __ballot(s < ns && seg_g[s_off + s] == g);
        if (hit) P.s = (int32_t)(base + (uint32_t)__ffsll((long long)hit) - 1u);
    }
    const unsigned long long hc = __ballot(lane < G.n_cpu && cpus_of(G, lane, g) == c);
    if (hc) P.ci = (int32_t)__ffsll((long long)hc) - 1;
    const unsigned long long hm = __ballot(lane < G.n_mem && tier_gib(G, lane, g) == mem);
    if (hm) P.mi = (int32_t)__ffsll((long long)hm) - 1;
    return P;
}

// Whether a record is an allocation on this table and grid: a GPU count of the job, a CPU level and a memory tier of
// the grid at that count, with a feasible plan there.  By one thread (the counts of a job ascend: bisection).
__device__ inline bool on_the_grid(const Retry &R, uint32_t j, uint32_t g, uint32_t c, float mem) {
    const uint32_t s_off = R.seg_off[j], ns = R.seg_off[j + 1] - s_off;
    uint32_t lo = 0, hi = ns;
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if (R.seg_g[s_off + mid] < g) lo = mid + 1; else hi = mid;
    }
    if (lo >= ns || R.seg_g[s_off + lo] != g) return false;
    int32_t ci = -1, mi = -1;
    for (uint32_t k = 0; k < R.grid.n_cpu && ci < 0; ++k) if (cpus_of(R.grid, k, g) == c) ci = (int32_t)k;
    for (uint32_t k = 0; k < R.grid.n_mem && mi < 0; ++k) if (tier_gib(R.grid, k, g) == mem) mi = (int32_t)k;
    if (ci < 0 || mi < 0) return false;
    const uint64_t at = (uint64_t)R.grid.n_cpu * R.grid.n_mem * s_off + ((uint64_t)ci * R.grid.n_mem + (uint32_t)mi) * ns + lo;
    return R.best_thr[at] > 0.f;
}

__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long v, uint32_t lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long o = __shfl_up(v, off, 64);
        if ((int)lane >= off) v += o;
    }
    return v;
}

// Inclusive prefix sum over the wavefront; all 64 lanes must be active.  Inside
// each row of 16 lanes by data-parallel-primitive shifts (lanes shifted in from
// outside the row read 0), then the rows' totals through scalar registers.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, uint32_t lane) {
    v += dpp_or_zero<0x111>(v);                             // row_shr:1
    v += dpp_or_zero<0x112>(v);                             // row_shr:2
    v += dpp_or_zero<0x114>(v);                             // row_shr:4
    v += dpp_or_zero<0x118>(v);                             // row_shr:8
    const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
    const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
    const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
    const uint32_t row = lane >> 4;
    return v + (row >= 1 ? t0 : 0u) + (row >= 2 ? t1 : 0u) + (row >= 3 ? t2 : 0u);
}

// exclusive prefix of one value per thread over the workgroup and the total; red = PLACE_WAVES words
__device__ __forceinline__ unsigned long long block_excl_scan(unsigned long long v, unsigned long long *red,
                                                              unsigned long long &total) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const unsigned long long incl = wave_incl_scan_u64(v, lane);
    if (lane == 63u) red[wave] = incl;
    __syncthreads();
    unsigned long long before = 0, all = 0;
#pragma unroll
    for (uint32_t w = 0; w < PLACE_WAVES; ++w) {
        if (w < wave) before += red[w];
        all += red[w];
    }
    __syncthreads();
    total = all;
    return before + incl - v;
}

// c*k / g and c*k % g; 32-bit arithmetic when the product cannot overflow (k <= g)
struct DivMod { unsigned long long q; uint32_t r; };
__device__ __forceinline__ DivMod cpus_times(uint32_t c, uint32_t k, uint32_t g) {
    DivMod d;
    if (((c | g) >> 16) == 0u) {
        const uint32_t t = c * k;
        d.q = t / g; d.r = t % g;
    } else {
        const unsigned long long t = (unsigned long long)c * k;
        d.q = t / g; d.r = (uint32_t)(t % g);
    }
    return d;
}
// CPUs that must be free for k of the job's g GPUs: ceil(c*k/g); and the memory of that part
__device__ __forceinline__ unsigned long long cpus_needed(uint32_t c, uint32_t k, uint32_t g) {
    const DivMod d = cpus_times(c, k, g);
    return d.q + (d.r ? 1u : 0u);
}
__device__ __forceinline__ float mem_of_part(float mem, uint32_t k, uint32_t g) {
    return (mem * (float)k) / (float)g;
}
// CPUs booked for k GPUs after `done` GPUs on earlier nodes: floor(c*(done+k)/g) - floor(c*done/g)
__device__ __forceinline__ uint32_t cpus_booked(uint32_t c, uint32_t done, uint32_t k, uint32_t g) {
    const DivMod a = cpus_times(c, done, g), b = cpus_times(c, k, g);
    return (uint32_t)(b.q + ((unsigned long long)a.r + b.r >= g ? 1u : 0u));
}

constexpr uint32_t PLACE_PER = 8;                         // jobs per thread in the first stage

__global__ __launch_bounds__(PLACE_THREADS) void k_place(PlaceArgs A) {
    extern __shared__ uint32_t lds[];
    uint32_t *nodeA = lds;                               // stage 1: CPUs needed per node; stage 2: free GPUs
    uint32_t *nodeB = nodeA + A.n_nodes;                 // stage 2: free CPUs
    float *nodeM = reinterpret_cast<float *>(nodeB + A.n_nodes);   // stage 1: memory per node; stage 2: free memory
    uint32_t *take = reinterpret_cast<uint32_t *>(nodeM + A.n_nodes);   // stage 2: GPUs offered by each node
    uint32_t *before = take + A.n_nodes;                 // stage 2: the job's GPUs on earlier nodes
    __shared__ unsigned long long red[PLACE_WAVES];
    __shared__ uint32_t redo;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;

    for (uint32_t n = tid; n < A.n_nodes; n += PLACE_THREADS) { nodeA[n] = 0u; nodeM[n] = 0.f; }
    if (tid == 0) redo = 0u;
    __syncthreads();

    // ---- stage 1: the jobs end to end on the GPU slots; a thread takes eight neighbouring jobs.  Not with an earlier
    // placement to respect: the kept jobs sit where they sat, so the others go job by job into what is left.
    const bool keeping = A.keep.prev_off != nullptr;
    const unsigned long long slots = (unsigned long long)A.n_nodes * A.gpn;
    unsigned long long carry_g = 0, carry_e = 0;          // GPU slots and parts before the tile
    uint32_t n_sched = 0, n_off = 0;                      // jobs with parts; records that are no allocation here
    if (keeping && tid == 0) redo = 1u;
    for (uint32_t base = 0; base < (keeping ? 0u : A.n_jobs); base += PLACE_THREADS * PLACE_PER) {
        const uint32_t j0 = base + tid * PLACE_PER;
        uint32_t g[PLACE_PER], c[PLACE_PER];
        float mem[PLACE_PER];
        unsigned long long sum_g = 0;
        // the thread's eight records are 160 contiguous bytes: ten 16-byte loads where that is possible
        static_assert(sizeof(rk_assign) == 20 && PLACE_PER == 8, "record layout of the vector loads");
        if (j0 + PLACE_PER <= A.n_jobs && (reinterpret_cast<uintptr_t>(A.assign) & 15u) == 0) {
            const uint4 *src = reinterpret_cast<const uint4 *>(A.assign + j0);
            uint32_t raw[40];
#pragma unroll
            for (uint32_t q = 0; q < 10; ++q) {
                const uint4 v = src[q];
                raw[4 * q] = v.x; raw[4 * q + 1] = v.y; raw[4 * q + 2] = v.z; raw[4 * q + 3] = v.w;
            }
#pragma unroll
            for (uint32_t i = 0; i < PLACE_PER; ++i) { g[i] = raw[5 * i]; c[i] = raw[5 * i + 1]; mem[i] = __uint_as_float(raw[5 * i + 2]); }
        } else {
#pragma unroll
            for (uint32_t i = 0; i < PLACE_PER; ++i) {
                g[i] = 0; c[i] = 0; mem[i] = 0.f;
                if (j0 + i < A.n_jobs) { g[i] = A.assign[j0 + i].g; c[i] = A.assign[j0 + i].c; mem[i] = A.assign[j0 + i].mem_gb; }
            }
        }
        uint32_t off_grid = 0;                             // bit i: the record is no allocation here (not placed, status 3)
        if (A.retry.on) {
#pragma unroll
            for (uint32_t i = 0; i < PLACE_PER; ++i)
                if (g[i] > 0 && !on_the_grid(A.retry, j0 + i, g[i], c[i], mem[i])) { off_grid |= 1u << i; g[i] = 0; }
            n_off += (uint32_t)__popc(off_grid);
        }
#pragma unroll
        for (uint32_t i = 0; i < PLACE_PER; ++i) sum_g += g[i];
        unsigned long long tile_g, tile_e;
        unsigned long long start = carry_g + block_excl_scan(sum_g, red, tile_g);
        uint32_t parts[PLACE_PER], k_first[PLACE_PER], node0[PLACE_PER];
        unsigned long long sum_e = 0;
#pragma unroll
        for (uint32_t i = 0; i < PLACE_PER; ++i) {
            const bool inside = g[i] > 0 && start + g[i] <= slots;      // then start fits in 32 bits (slots do)
            if (g[i] > 0 && !inside) redo = 1u;           // more GPUs than slots: job by job decides who fails
            const uint32_t s32 = inside ? (uint32_t)start : 0u;
            node0[i] = s32 / A.gpn;
            const uint32_t room = A.gpn - (s32 - node0[i] * A.gpn);      // free slots of the node the job starts on
            k_first[i] = g[i] < room ? g[i] : room;
            const uint32_t rest = g[i] - k_first[i], whole = rest / A.gpn;
            parts[i] = inside ? 1u + whole + (rest - whole * A.gpn ? 1u : 0u) : 0u;
            sum_e += parts[i];
            start += g[i];
            n_sched += g[i] > 0 ? 1u : 0u;
        }
        unsigned long long at = carry_e + block_excl_scan(sum_e, red, tile_e);
        // one part of a job: its k GPUs after `done` GPUs on earlier nodes go to node n
        auto write_part = [&](uint32_t jg, uint32_t jc, float jm, size_t where, uint32_t n, uint32_t done, uint32_t k) {
            rk_place_entry e;
            e.node = n;
            e.g = k;
            e.c = cpus_booked(jc, done, k, jg);
            e.mem_gb = mem_of_part(jm, k, jg);
            A.entries[where] = e;
            const unsigned long long need = cpus_needed(jc, k, jg);
            if (need > A.cpn) redo = 1u;                  // (and the sum below cannot wrap: at most gpn parts of <= cpn)
            else atomicAdd(&nodeA[n], (uint32_t)need);
            atomicAdd(&nodeM[n], e.mem_gb);
        };
        {   // offsets and status words of the thread's eight jobs: two 16-byte stores per array where that is possible
            uint32_t offs[PLACE_PER], stat[PLACE_PER], run = (uint32_t)at;
#pragma unroll
            for (uint32_t i = 0; i < PLACE_PER; ++i) {
                offs[i] = run;
                stat[i] = g[i] > 0 ? 1u : ((off_grid >> i) & 1u) ? 3u : 0u;
                run += parts[i];
            }
            const bool whole8 = j0 + PLACE_PER <= A.n_jobs &&
                                ((reinterpret_cast<uintptr_t>(A.place_off) | reinterpret_cast<uintptr_t>(A.status)) & 15u) == 0;
            if (whole8) {
                uint4 *po = reinterpret_cast<uint4 *>(A.place_off + j0), *ps = reinterpret_cast<uint4 *>(A.status + j0);
                po[0] = make_uint4(offs[0], offs[1], offs[2], offs[3]); po[1] = make_uint4(offs[4], offs[5], offs[6], offs[7]);
                ps[0] = make_uint4(stat[0], stat[1], stat[2], stat[3]); ps[1] = make_uint4(stat[4], stat[5], stat[6], stat[7]);
            } else {
#pragma unroll
                for (uint32_t i = 0; i < PLACE_PER; ++i)
                    if (j0 + i < A.n_jobs) { A.place_off[j0 + i] = offs[i]; A.status[j0 + i] = stat[i]; }
            }
        }
#pragma unroll
        for (uint32_t i = 0; i < PLACE_PER; ++i) {
            const uint32_t n0 = node0[i];
            if (parts[i] > 0 && parts[i] <= 2) {          // short jobs: by their own thread
                write_part(g[i], c[i], mem[i], at, n0, 0, k_first[i]);
                if (parts[i] == 2) write_part(g[i], c[i], mem[i], at + 1, n0 + 1, k_first[i], g[i] - k_first[i]);
            }
            // jobs over three nodes or more: by the whole wavefront, a lane per part
            unsigned long long todo = __ballot(parts[i] > 2);
            while (todo) {
                const int src = (int)__ffsll((long long)todo) - 1;
                todo &= todo - 1ull;
                const uint32_t jg = (uint32_t)__builtin_amdgcn_readlane((int)g[i], src);
                const uint32_t jc = (uint32_t)__builtin_amdgcn_readlane((int)c[i], src);
                const float jm = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mem[i]), src));
                const uint32_t jparts = (uint32_t)__builtin_amdgcn_readlane((int)parts[i], src);
                const uint32_t jfirst = (uint32_t)__builtin_amdgcn_readlane((int)k_first[i], src);
                const uint32_t jn0 = (uint32_t)__builtin_amdgcn_readlane((int)n0, src);
                const uint32_t jat = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)at, src);   // parts fit in 32 bits
                for (uint32_t p = lane; p < jparts; p += 64) {
                    const uint32_t done = p == 0 ? 0u : jfirst + (p - 1) * A.gpn;
                    const uint32_t rest = jg - done;
                    const uint32_t k = p == 0 ? jfirst : (rest < A.gpn ? rest : A.gpn);
                    write_part(jg, jc, jm, (size_t)jat + p, jn0 + p, done, k);
                }
            }
            at += parts[i];
        }
        carry_g += tile_g;
        carry_e += tile_e;
    }
    __syncthreads();
    for (uint32_t n = tid; n < A.n_nodes; n += PLACE_THREADS)
        if (nodeA[n] > A.cpn || !(nodeM[n] <= 0.999f * A.mpn)) redo = 1u;
    unsigned long long placed_all;
    (void)block_excl_scan(((unsigned long long)n_off << 32) | n_sched, red, placed_all);   // also the barrier after the writes to redo
    if (!redo) {
        if (tid == 0) {
            A.place_off[A.n_jobs] = (uint32_t)carry_e;
            A.result[0] = (uint32_t)carry_e; A.result[1] = (uint32_t)placed_all; A.result[2] = (uint32_t)(placed_all >> 32);
            A.result[3] = 0u;
        }
        return;
    }

    // ---- stage 2: job by job, by the first wavefront
    for (uint32_t n = tid; n < A.n_nodes; n += PLACE_THREADS) { nodeA[n] = A.gpn; nodeB[n] = A.cpn; nodeM[n] = A.mpn; }
    if (keeping) {
        // which jobs stay: the amounts asked are an allocation here and every earlier part is what first fit books
        // for these amounts on that split (all threads, a job each)
        for (uint32_t j = tid; j < A.n_jobs; j += PLACE_THREADS) {
            const uint32_t g = A.assign[j].g, c = A.assign[j].c;
            const float mem = A.assign[j].mem_gb;
            const uint32_t a = A.keep.prev_off[j], b = A.keep.prev_off[j + 1];
            bool same = g > 0 && b > a && (!A.retry.on || on_the_grid(A.retry, j, g, c, mem));
            uint32_t done = 0;
            for (uint32_t i = a; i < b && same; ++i) {
                const rk_place_entry e = A.keep.prev_entries[i];
                if (e.node >= A.n_nodes || e.g == 0 || e.g > g - done) { same = false; break; }
                if (e.c != cpus_booked(c, done, e.g, g) || !(e.mem_gb == mem_of_part(mem, e.g, g))) same = false;
                done += e.g;
            }
            A.keep.flag[j] = (same && done == g) ? 1 : 0;
        }
    }
    __syncthreads();
    if (tid >= 64) return;
    uint32_t cursor = 0, n_placed = 0, n_failed = 0;
    uint32_t first_g = 0, first_gc = 0;                  // first node with a free GPU; with a free GPU and a free CPU
    unsigned long long free_gpus = slots;                 // of the whole cluster
    if (keeping) {
        // the kept jobs are booked first, in job order (a node's free memory is a float32 running remainder, so the
        // order of the subtractions is part of the result); a job's parts sit on different nodes: a lane each
        bool fits = true;
        for (uint32_t base = 0; base < A.n_jobs && fits; base += 64) {
            const uint32_t j = base + lane;
            unsigned long long todo = __ballot(j < A.n_jobs && A.keep.flag[j] != 0);
            while (todo && fits) {
                const uint32_t jj = base + (uint32_t)__ffsll((long long)todo) - 1u;
                todo &= todo - 1ull;
                const uint32_t a = A.keep.prev_off[jj], b = A.keep.prev_off[jj + 1];
                for (uint32_t ib = a; ib < b && fits; ib += 64) {
                    const uint32_t i = ib + lane;
                    bool ok = true;
                    if (i < b) {
                        const rk_place_entry e = A.keep.prev_entries[i];
                        ok = nodeA[e.node] >= e.g && nodeB[e.node] >= e.c && e.mem_gb <= nodeM[e.node];
                        if (ok) {
                            nodeA[e.node] -= e.g;
                            nodeB[e.node] -= e.c;
                            nodeM[e.node] = nodeM[e.node] - e.mem_gb;
                        }
                    }
                    fits = __ballot(!ok) == 0ull;
                }
                free_gpus -= A.assign[jj].g;
            }
        }
        if (!fits) {
            // the earlier placement is no placement on these nodes: it is ignored, everything is placed anew
            for (uint32_t n = lane; n < A.n_nodes; n += 64) { nodeA[n] = A.gpn; nodeB[n] = A.cpn; nodeM[n] = A.mpn; }
            for (uint32_t j = lane; j < A.n_jobs; j += 64) A.keep.flag[j] = 0;
            free_gpus = slots;
        }
    }
    for (uint32_t base = 0; base < A.n_jobs; base += 64) {
        const uint32_t j = base + lane;
        uint32_t g = 0, c = 0;
        float mem = 0.f;
        if (j < A.n_jobs) { g = A.assign[j].g; c = A.assign[j].c; mem = A.assign[j].mem_gb; }
        uint32_t my_off = 0, my_status = 0;
        if (A.retry.on && g > 0 && !on_the_grid(A.retry, j, g, c, mem)) { g = 0; my_status = 3u; }   // no allocation here
        n_failed += (uint32_t)__popcll(__ballot(my_status == 3u));
        bool have_off = false;
        unsigned long long todo = __ballot(g > 0);
        while (todo) {
            const int turn = (int)__ffsll((long long)todo) - 1;
            todo &= todo - 1ull;
            if ((int)lane <= turn && !have_off) { my_off = cursor; have_off = true; }   // jobs up to this one start here
            uint32_t jg = (uint32_t)__builtin_amdgcn_readlane((int)g, turn);
            uint32_t jc = (uint32_t)__builtin_amdgcn_readlane((int)c, turn);
            float jm = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mem), turn));
            if (keeping && A.keep.flag[base + (uint32_t)turn]) {           // stays: its earlier parts, booked above
                const uint32_t jj = base + (uint32_t)turn;
                const uint32_t a = A.keep.prev_off[jj], b = A.keep.prev_off[jj + 1];
                for (uint32_t i = a + lane; i < b; i += 64) A.entries[cursor + (i - a)] = A.keep.prev_entries[i];
                cursor += b - a;
                if ((int)lane == turn) my_status = 1u;
                ++n_placed;
                continue;
            }
            GridPos pos = {-2, -1, -1};                    // -2: not looked up yet
            uint32_t tries = 0, first, left, end;
            for (;;) {                                     // the amount asked for, then smaller ones if allowed
            // the offers of the nodes, cut at what the job still lacks (none are asked when the cluster has too few);
            // a job that needs CPUs gets nothing from a node without a free CPU
            first = jc > 0 ? first_gc : first_g;
            left = jg;
            end = first;
            for (uint32_t nb = first; nb < A.n_nodes && left > 0 && jg <= free_gpus; nb += 64) {
                const uint32_t n = nb + lane;
                uint32_t k = 0;
                if (n < A.n_nodes) {
                    // the most GPUs whose CPUs and memory are free here; both needs grow with k, so a bisection finds it
                    const uint32_t fc = nodeB[n];
                    const float fm = nodeM[n];
                    auto fits = [&](uint32_t x) { return cpus_needed(jc, x, jg) <= fc && mem_of_part(jm, x, jg) <= fm; };
                    uint32_t lo = 0, hi = nodeA[n] < jg ? nodeA[n] : jg;
                    if (hi > 0 && !fits(hi)) {
                        while (hi - lo > 1) {
                            const uint32_t mid = lo + (hi - lo) / 2;
                            if (fits(mid)) lo = mid; else hi = mid;
                        }
                        hi = lo;
                    }
                    k = hi;
                }
                const uint32_t incl = wave_incl_scan_u32(k, lane), excl = incl - k;
                const uint32_t room = left > excl ? left - excl : 0u;
                k = k < room ? k : room;
                if (n < A.n_nodes) { take[n] = k; before[n] = (jg - left) + excl; }
                const uint32_t all = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                left -= all < left ? all : left;
                end = nb + 64;
            }
            if (left == 0 || !A.retry.on) break;
            {                                             // not found: the next smaller count the job may run on
                const Retry &R = A.retry;
                const uint32_t jj = base + (uint32_t)turn;
                const uint32_t s_off = R.seg_off[jj], ns = R.seg_off[jj + 1] - s_off;
                if (pos.s == -2) pos = locate(R.grid, R.seg_g, s_off, ns, jg, jc, jm, lane);
                int32_t next = -1;
                if (pos.s >= 0 && pos.ci >= 0 && pos.mi >= 0) {
                    const int32_t floor_s = R.min_seg && R.min_seg[jj] > 0 ? R.min_seg[jj] : 0;
                    const uint64_t row = (uint64_t)R.grid.n_cpu * R.grid.n_mem * s_off +
                                         ((uint64_t)pos.ci * R.grid.n_mem + pos.mi) * ns;
                    for (int32_t hi = pos.s - 1; hi >= floor_s && next < 0; hi -= 64) {
                        const int32_t s = hi - (int32_t)lane;                 // lane 0 looks at the nearest count
                        const unsigned long long ok = __ballot(s >= floor_s && R.best_thr[row + (uint32_t)(s < 0 ? 0 : s)] > 0.f);
                        if (ok) next = hi - ((int32_t)__ffsll((long long)ok) - 1);
                    }
                }
                if (next < 0) break;
                pos.s = next;
                jg = R.seg_g[s_off + (uint32_t)next];
                jc = cpus_of(R.grid, (uint32_t)pos.ci, jg);
                jm = tier_gib(R.grid, (uint32_t)pos.mi, jg);
                ++tries;
            }
            }
            if (left > 0) {                               // not found: nothing is booked
                if ((int)lane == turn) my_status = A.retry.on ? 3u : 2u;
                ++n_failed;
                continue;
            }
            if ((int)lane == turn) my_status = tries ? 2u : 1u;
            ++n_placed;
            free_gpus -= jg;
            for (uint32_t nb = first; nb < end; nb += 64) {
                const uint32_t n = nb + lane;
                const uint32_t k = n < A.n_nodes ? take[n] : 0u;
                const unsigned long long with = __ballot(k > 0);
                if (k > 0) {
                    rk_place_entry e;
                    e.node = n;
                    e.g = k;
                    e.c = cpus_booked(jc, before[n], k, jg);
                    e.mem_gb = mem_of_part(jm, k, jg);
                    nodeA[n] -= k;
                    nodeB[n] -= e.c;
                    nodeM[n] = nodeM[n] - e.mem_gb;
                    A.entries[cursor + (uint32_t)__popcll(with & ((1ull << lane) - 1ull))] = e;
                }
                cursor += (uint32_t)__popcll(with);
            }
            // the first nodes that are still of use
            while (first_g < A.n_nodes) {
                const uint32_t n = first_g + lane;
                const unsigned long long open = __ballot(n < A.n_nodes && nodeA[n] > 0);
                if (open) { first_g += (uint32_t)__ffsll((long long)open) - 1u; break; }
                first_g += 64;
            }
            if (first_g > A.n_nodes) first_g = A.n_nodes;
            if (first_gc < first_g) first_gc = first_g;
            while (first_gc < A.n_nodes) {
                const uint32_t n = first_gc + lane;
                const unsigned long long open = __ballot(n < A.n_nodes && nodeA[n] > 0 && nodeB[n] > 0);
                if (open) { first_gc += (uint32_t)__ffsll((long long)open) - 1u; break; }
                first_gc += 64;
            }
            if (first_gc > A.n_nodes) first_gc = A.n_nodes;
        }
        if (!have_off) my_off = cursor;
        if (j < A.n_jobs) { A.place_off[j] = my_off; A.status[j] = my_status; }
    }
    if (lane == 0) {
        A.place_off[A.n_jobs] = cursor;
        A.result[0] = cursor; A.result[1] = n_placed; A.result[2] = n_failed; A.result[3] = 1u;
    }
}

// ------------------------------------------------------------ the plan of a placed job
// GetBestPlan(j, placement): a wavefront per job.  The job's parts give its GPU count and the greatest common
// divisor of the counts at which its slots cross a node boundary, which decides the bandwidth of every kind of
// communication group (placed_links); its lanes then take the triples of that GPU count, all sixteen options each,
// with the arithmetic of the candidate evaluation, and the best (throughput, lowest plan index) wins.
constexpr int REPLAN_THREADS = 256;

struct ReplanArgs {
    JobDev jobs;
    TableDev tb;
    GridDev grid;
    rk_env env;
    uint32_t n_jobs, option_mask;
    const rk_assign *assign;         // what was asked for: fixes the CPU level and the memory tier
    const uint32_t *place_off;
    const rk_place_entry *entries;
    const uint32_t *status;          // null: a job is placed when it has parts
    rk_assign *placed;
};

__device__ __forceinline__ uint32_t gcd_u32(uint32_t a, uint32_t b) {
    while (b) { const uint32_t r = a % b; a = b; b = r; }
    return a;
}

__global__ __launch_bounds__(REPLAN_THREADS) void k_replan(ReplanArgs A) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t j = blockIdx.x * (REPLAN_THREADS / 64) + (threadIdx.x >> 6);
    if (j >= A.n_jobs) return;
    rk_assign out = {0u, 0u, 0.f, RK_NO_PLAN, 0.f};
    const uint32_t st = A.status ? A.status[j] : (A.place_off[j + 1] > A.place_off[j] ? 1u : 0u);
    if (st == 1u || st == 2u) {
        const uint32_t e0 = A.place_off[j], e1 = A.place_off[j + 1];
        uint32_t run = 0, ge = 0;                          // GPUs so far; gcd of the boundaries this lane has seen
        for (uint32_t base = e0; base < e1; base += 64) {
            const uint32_t i = base + lane;
            const uint32_t k = i < e1 ? A.entries[i].g : 0u;
            uint32_t incl = k;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t o = __shfl_up(incl, off, 64);
                if ((int)lane >= off) incl += o;
            }
            incl += run;
            if (i + 1 < e1) ge = gcd_u32(ge, incl);       // the end of the last part is not a boundary inside the job
            run = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ge = gcd_u32(ge, __shfl_xor(ge, off, 64));
        const uint32_t g = run;
        const uint32_t s_off = A.tb.seg_off[j], ns = A.tb.seg_off[j + 1] - s_off;
        const rk_assign asked = A.assign[j];
        const GridPos lv = locate(A.grid, A.tb.seg_g, s_off, ns, asked.g, asked.c, asked.mem_gb, lane);
        const GridPos at = locate(A.grid, A.tb.seg_g, s_off, ns, g, 0u, 0.f, lane);
        if (lv.ci >= 0 && lv.mi >= 0 && at.s >= 0) {
            const uint32_t ci = (uint32_t)lv.ci, mi = (uint32_t)lv.mi, s = (uint32_t)at.s;
            const uint32_t c = cpus_of(A.grid, ci, g);
            const float tier = tier_bytes(A.grid, mi, g);
            const uint32_t t0 = A.tb.triple_off[j], nt = A.tb.triple_off[j + 1] - t0;
            const uint32_t first = A.tb.seg_first[s_off + s];
            const uint32_t last = s + 1 < ns ? A.tb.seg_first[s_off + s + 1] : nt;
            const Job J = load_job(A.jobs, j);
            unsigned long long key = 0;
            for (uint32_t tl = first + lane; tl < last; tl += 64) {
                const Triple T = triple_terms_on<true>(J, A.env, A.tb.triples[t0 + tl], ge);
                bool any_off = false;
#pragma unroll
                for (uint32_t z = 0; z < 4; ++z)
#pragma unroll
                    for (uint32_t gc = 0; gc < 2; ++gc) {
                        const uint32_t o = z * 4 + gc * 2;
                        if (((A.option_mask >> o) & 1u) && gpu_mem_fits(J, A.env, T, z, gc, 0)) {
                            const unsigned long long k2 = make_key(thr_plain(J, T, z, gc), tl * 16 + o);
                            key = k2 > key ? k2 : key;
                        }
                        if (z >= 2 && ((A.option_mask >> (o + 1)) & 1u)) any_off = true;
                    }
                if (any_off && host_bytes_needed(J, T) <= tier) {
                    const Offload O = offload_terms(J, A.env, T);
                    const float sw = swap_term(J, O, c);
#pragma unroll
                    for (uint32_t z = 2; z < 4; ++z)
#pragma unroll
                        for (uint32_t gc = 0; gc < 2; ++gc) {
                            const uint32_t o = z * 4 + gc * 2 + 1;
                            if (((A.option_mask >> o) & 1u) && gpu_mem_fits(J, A.env, T, z, gc, 1)) {
                                const unsigned long long k2 = make_key(thr_offload(T, O, gc, sw), tl * 16 + o);
                                key = k2 > key ? k2 : key;
                            }
                        }
                }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const unsigned long long o = __shfl_xor(key, off, 64);
                key = o > key ? o : key;
            }
            out.g = g; out.c = c; out.mem_gb = tier_gib(A.grid, mi, g);
            out.plan = key_plan(key); out.thr = key_thr(key);
        }
    }
    if (lane == 0) A.placed[j] = out;
}

// total = sum of thr / ref_thr over the records, in float64, in a fixed order (thread t takes the jobs t, t + 1024, ...)
__global__ __launch_bounds__(1024) void k_place_total(uint32_t n_jobs, const rk_assign *placed, const float *ref_thr,
                                                      float *total) {
    __shared__ double part[1024];
    double sum = 0.0;
    for (uint32_t j = threadIdx.x; j < n_jobs; j += 1024)
        if (placed[j].g > 0) sum += (double)placed[j].thr / (double)ref_thr[j];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (uint32_t w = 512; w >= 1; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *total = (float)part[0];
}

int32_t launch_place(rk_ctx *ctx, const rk_nodes *nodes, uint32_t n_jobs, const rk_assign *assign, uint32_t *place_off,
                     rk_place_entry *entries, uint64_t cap_entries, uint32_t *status, const Retry &retry,
                     const uint32_t *prev_off, const rk_place_entry *prev_entries, rk_place_result *result) {
    if (!nodes || !place_off) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (n_jobs > 0 && (!assign || !status)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "assign or status is null");
    if (nodes->n_nodes < 1 || nodes->n_nodes > RK_MAX_NODES)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "n_nodes must be in 1..%u", RK_MAX_NODES);
    if (nodes->gpus_per_node < 1 || nodes->gpus_per_node > 65535)
        return rk_fail(ctx, RK_ERR_UNSUPPORTED, "gpus_per_node must be in 1..65535");
    if (nodes->cpus_per_node > 65535) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "cpus_per_node must be at most 65535");
    if (!(nodes->mem_per_node_gb >= 0.f)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "mem_per_node_gb is negative or not a number");
    const uint64_t need = (uint64_t)nodes->n_nodes * nodes->gpus_per_node;
    if (cap_entries < need)
        return rk_fail(ctx, RK_ERR_CAPACITY, "entries holds %llu parts, %llu needed (n_nodes * gpus_per_node)",
                       (unsigned long long)cap_entries, (unsigned long long)need);
    if (!entries) return rk_fail(ctx, RK_ERR_INVALID_ARG, "entries is null");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    PlaceArgs A;
    A.n_jobs = n_jobs; A.n_nodes = nodes->n_nodes; A.gpn = nodes->gpus_per_node; A.cpn = nodes->cpus_per_node;
    A.mpn = nodes->mem_per_node_gb;
    A.assign = assign; A.place_off = place_off; A.entries = entries; A.status = status;
    A.retry = retry;
    A.keep = Keep{nullptr, nullptr, nullptr};
    int32_t rc;
    if (prev_off && n_jobs > 0) {
        if (!prev_entries) return rk_fail(ctx, RK_ERR_INVALID_ARG, "prev_off without prev_entries");
        if (prev_entries == entries || prev_off == place_off)
            return rk_fail(ctx, RK_ERR_INVALID_ARG, "the earlier placement must not be the output buffers");
        A.keep.prev_off = prev_off; A.keep.prev_entries = prev_entries;
        if ((rc = rk_scratch(ctx, SL_PLACE_KEEP, (size_t)n_jobs, (void **)&A.keep.flag))) return rc;
    }
    if ((rc = rk_scratch(ctx, SL_PLACE_RESULT, 4 * sizeof(uint32_t), (void **)&A.result))) return rc;
    const size_t lds = (size_t)A.n_nodes * 5 * sizeof(uint32_t);
    if (lds > 48 * 1024 && !ctx->place_lds_raised) {
        RK_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(k_place),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, RK_MAX_NODES * 5 * sizeof(uint32_t)));
        ctx->place_lds_raised = true;
    }
    k_place<<<1, PLACE_THREADS, lds, ctx->stream>>>(A);
    RK_CHECK_LAUNCH(ctx, "k_place");
    (void)result;
    return RK_OK;
}

int32_t fetch_place_result(rk_ctx *ctx, rk_place_result *result) {
    uint32_t *d_result = static_cast<uint32_t *>(ctx->scratch[SL_PLACE_RESULT]);
    uint32_t *h = ctx->h_pinned;
    RK_HIP(ctx, hipMemcpyAsync(h, d_result, 4 * sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
    RK_HIP(ctx, hipStreamSynchronize(ctx->stream));
    result->n_entries = h[0]; result->n_placed = h[1]; result->n_failed = h[2]; result->in_order = h[3];
    return RK_OK;
}

}  // namespace

extern "C" int32_t rk_place(rk_ctx *ctx, const rk_nodes *nodes, uint32_t n_jobs, const rk_assign *assign,
                            uint32_t *place_off, rk_place_entry *entries, uint64_t cap_entries, uint32_t *status,
                            rk_place_result *result) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    Retry none = {};
    int32_t rc;
    if ((rc = launch_place(ctx, nodes, n_jobs, assign, place_off, entries, cap_entries, status, none, nullptr, nullptr,
                           result))) return rc;
    return result ? fetch_place_result(ctx, result) : RK_OK;
}

int32_t rk_launch_place_plans(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                              const rk_env *env, const rk_nodes *nodes, const float *best_thr, const rk_assign *assign,
                              const int32_t *min_seg, const uint32_t *prev_off, const rk_place_entry *prev_entries,
                              rk_assign *placed, uint32_t *place_off, rk_place_entry *entries,
                              uint64_t cap_entries, uint32_t *status, float *total, rk_place_result *result) {
    const uint32_t n_jobs = table->n_jobs;
    Retry retry = {};
    retry.on = 1u;
    retry.seg_off = table->seg_off; retry.seg_g = table->seg_g;
    retry.best_thr = best_thr; retry.min_seg = min_seg;
    retry.grid = grid_dev(grid);
    int32_t rc;
    if ((rc = launch_place(ctx, nodes, n_jobs, assign, place_off, entries, cap_entries, status, retry, prev_off, prev_entries,
                           result))) return rc;
    if (n_jobs > 0) {
        ReplanArgs R;
        R.jobs = job_dev(jobs); R.tb = table_dev(table); R.grid = retry.grid; R.env = *env;
        R.n_jobs = n_jobs; R.option_mask = table->option_mask;
        R.assign = assign; R.place_off = place_off; R.entries = entries; R.status = status; R.placed = placed;
        const uint32_t per = REPLAN_THREADS / 64;
        k_replan<<<(n_jobs + per - 1) / per, REPLAN_THREADS, 0, ctx->stream>>>(R);
        RK_CHECK_LAUNCH(ctx, "k_replan");
    }
    k_place_total<<<1, 1024, 0, ctx->stream>>>(n_jobs, placed, jobs->ref_thr, total);
    RK_CHECK_LAUNCH(ctx, "k_place_total");
    return result ? fetch_place_result(ctx, result) : RK_OK;
}

extern "C" int32_t rk_place_plans(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                                  const rk_env *env, const rk_nodes *nodes, const float *best_thr, const rk_assign *assign,
                                  const int32_t *min_seg, const uint32_t *prev_off, const rk_place_entry *prev_entries,
                                  rk_assign *placed, uint32_t *place_off, rk_place_entry *entries,
                                  uint64_t cap_entries, uint32_t *status, float *total, rk_place_result *result) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!jobs || !total) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if ((rc = rk_check_table(ctx, table, 0, table ? table->n_jobs : 0))) return rc;
    if (jobs->n_jobs != table->n_jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs and table disagree on n_jobs");
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if ((rc = rk_check_env(ctx, env))) return rc;
    if (table->n_jobs > 0 && (!placed || !jobs->ref_thr || (table->n_segs > 0 && !best_thr)))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    return rk_launch_place_plans(ctx, jobs, table, grid, env, nodes, best_thr, assign, min_seg, prev_off, prev_entries, placed,
                                 place_off, entries, cap_entries, status, total, result);
}

extern "C" int32_t rk_best_plan_placed(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                                       const rk_alloc_grid *grid, const rk_env *env, const rk_assign *assign,
                                       const uint32_t *place_off, const rk_place_entry *entries, rk_assign *placed,
                                       float *total) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!jobs || !total || !place_off) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if ((rc = rk_check_table(ctx, table, 0, table ? table->n_jobs : 0))) return rc;
    if (jobs->n_jobs != table->n_jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs and table disagree on n_jobs");
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if ((rc = rk_check_env(ctx, env))) return rc;
    const uint32_t n_jobs = table->n_jobs;
    if (n_jobs > 0 && (!placed || !assign || !entries || !jobs->ref_thr)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (placed == assign) return rk_fail(ctx, RK_ERR_INVALID_ARG, "placed must not be the records it is chosen from");
    RK_HIP(ctx, hipSetDevice(ctx->device));
    return rk_launch_best_plan_placed(ctx, jobs, table, grid, env, assign, place_off, entries, placed, total);
}

int32_t rk_launch_best_plan_placed(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                                   const rk_env *env, const rk_assign *assign, const uint32_t *place_off,
                                   const rk_place_entry *entries, rk_assign *placed, float *total) {
    const uint32_t n_jobs = table->n_jobs;
    if (n_jobs > 0) {
        ReplanArgs R;
        R.jobs = job_dev(jobs); R.tb = table_dev(table); R.grid = grid_dev(grid); R.env = *env;
        R.n_jobs = n_jobs; R.option_mask = table->option_mask;
        R.assign = assign; R.place_off = place_off; R.entries = entries; R.status = nullptr; R.placed = placed;
        const uint32_t per = REPLAN_THREADS / 64;
        k_replan<<<(n_jobs + per - 1) / per, REPLAN_THREADS, 0, ctx->stream>>>(R);
        RK_CHECK_LAUNCH(ctx, "k_replan");
    }
    k_place_total<<<1, 1024, 0, ctx->stream>>>(n_jobs, placed, jobs->ref_thr, total);
    RK_CHECK_LAUNCH(ctx, "k_place_total");
    return RK_OK;
}
