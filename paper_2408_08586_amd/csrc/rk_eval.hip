// Materialising path: candidate evaluation (paper Sec. 4, Eq. 1) with
// feasibility masking, the segmented best-plan reduction (GetBestPlan,
// Sec. 5.2) and the curve prefix maximum (Sec. 5.2, Fig. 6).
#include "rk_internal.h"
#include "rk_model.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));   // 16-byte vector the streaming builtins accept

constexpr int EVAL_THREADS = 256;
constexpr int TRIPLES_PER_BLOCK = EVAL_THREADS / 4;

// ---------------------------------------------------------------- evaluation
// A thread owns (triple, ZeRO stage z): the four options gc x off of that
// stage, i.e. 16 contiguous bytes of every row.  A wavefront therefore writes
// 1 KiB contiguous per row.  Everything that does not depend on the row is
// computed once per thread; the CPU-dependent swap term once per CPU level.
template <bool WITH_FEAS>
__global__ __launch_bounds__(EVAL_THREADS) void k_eval(JobDev jobs, TableDev tb, GridDev grid, rk_env env,
                                                       uint32_t jb, uint32_t option_mask, uint32_t c_per_block,
                                                       float *__restrict__ thr, uint8_t *__restrict__ feas) {
    const uint32_t j = jb + blockIdx.y;
    const uint32_t t0 = tb.triple_off[j];
    const uint32_t nt = tb.triple_off[j + 1] - t0;
    const uint32_t tl = blockIdx.x * TRIPLES_PER_BLOCK + (threadIdx.x >> 2);
    if (tl >= nt) return;
    const uint32_t z = threadIdx.x & 3u;
    const uint32_t n_rows = grid.n_cpu * grid.n_mem;
    const uint64_t cbase = 16ull * n_rows * (uint64_t)(t0 - tb.triple_off[jb]);

    const Job J = load_job(jobs, j);
    const Triple T = triple_terms(J, env, tb.triples[t0 + tl]);

    // options without offload: o = z*4 + gc*2
    float plain[2];
    uint32_t why_plain[2];
#pragma unroll
    for (uint32_t gc = 0; gc < 2; ++gc) {
        const bool allowed = (option_mask >> (z * 4 + gc * 2)) & 1u;
        const bool fits = gpu_mem_fits(J, env, T, z, gc, 0);
        why_plain[gc] = allowed ? (fits ? 0u : RK_INFEASIBLE_GPU_MEM) : RK_INFEASIBLE_STRUCT;
        plain[gc] = why_plain[gc] ? 0.f : thr_plain(J, T, z, gc);
    }
    // options with offload: o = z*4 + gc*2 + 1, need z >= 2
    uint32_t why_off[2];
#pragma unroll
    for (uint32_t gc = 0; gc < 2; ++gc) {
        const bool allowed = z >= 2 && ((option_mask >> (z * 4 + gc * 2 + 1)) & 1u);
        why_off[gc] = allowed ? (gpu_mem_fits(J, env, T, z, gc, 1) ? 0u : RK_INFEASIBLE_GPU_MEM)
                              : RK_INFEASIBLE_STRUCT;
    }
    const bool any_off = z >= 2 && (!(why_off[0] & RK_INFEASIBLE_STRUCT) || !(why_off[1] & RK_INFEASIBLE_STRUCT));
    Offload O = {};
    float need_host = 0.f;
    if (any_off) {
        O = offload_terms(J, env, T);
        need_host = host_bytes_needed(J, T);
    }

    const uint32_t c_lo = blockIdx.z * c_per_block;
    const uint32_t c_hi = c_lo + c_per_block < grid.n_cpu ? c_lo + c_per_block : grid.n_cpu;
    for (uint32_t ci = c_lo; ci < c_hi; ++ci) {
        float off_thr[2] = {0.f, 0.f};
        if (any_off) {
            const float sw = swap_term(J, O, cpus_of(grid, ci, T.g));
            off_thr[0] = thr_offload(T, O, 0, sw);
            off_thr[1] = thr_offload(T, O, 1, sw);
        }
        for (uint32_t mi = 0; mi < grid.n_mem; ++mi) {
            uint32_t w0 = why_off[0], w1 = why_off[1];
            if (any_off && !(need_host <= tier_bytes(grid, mi, T.g))) {
                if (!(w0 & RK_INFEASIBLE_STRUCT)) w0 |= RK_INFEASIBLE_HOST_MEM;
                if (!(w1 & RK_INFEASIBLE_STRUCT)) w1 |= RK_INFEASIBLE_HOST_MEM;
            }
            v4f v;
            v.x = plain[0];
            v.y = w0 ? 0.f : off_thr[0];
            v.z = plain[1];
            v.w = w1 ? 0.f : off_thr[1];
            const uint64_t idx = cbase + ((uint64_t)(ci * grid.n_mem + mi) * nt + tl) * 16 + z * 4;
            *reinterpret_cast<v4f *>(thr + idx) = v;
            if (WITH_FEAS) {
                const uint32_t packed = why_plain[0] | (w0 << 8) | (why_plain[1] << 16) | (w1 << 24);
                *reinterpret_cast<uint32_t *>(feas + idx) = packed;
            }
        }
    }
}

// ---------------------------------------------------------- best plan per segment
// A workgroup of `wpb` wavefronts takes wpb rows of one job, one wavefront per
// row.  The triple -> segment map of the job is built once per workgroup in
// LDS.  Lanes stream the row as 16-byte streaming loads (four options of one
// triple), the next chunk being requested before the current one is reduced;
// four lanes reduce a triple with DPP and the quad leader pushes the triple's
// packed key (throughput bits, inverted plan index: larger throughput, then
// lower index) into the wavefront's per-segment keys with an LDS atomic max.
constexpr int BEST_MAX_WAVES = 16;
constexpr int BEST_UNROLL = 4;

__device__ __forceinline__ unsigned long long max_u64(unsigned long long a, unsigned long long b) {
    return a > b ? a : b;
}

template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_u64(unsigned long long v) {
    const uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    const uint32_t l2 = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, 0xF, 0xF, false);
    const uint32_t h2 = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, 0xF, 0xF, false);
    return ((unsigned long long)h2 << 32) | l2;
}

__global__ __launch_bounds__(BEST_MAX_WAVES * 64) void k_best_plan(TableDev tb, uint32_t n_rows, uint32_t jb,
                                                                   uint32_t wpb, uint32_t grp_per_job, uint32_t max_nt,
                                                                   uint32_t max_ns,
                                                                   const float *__restrict__ thr,
                                                                   float *__restrict__ best_thr,
                                                                   uint32_t *__restrict__ best_plan) {
    extern __shared__ unsigned long long lds64[];
    unsigned long long *seg_key = lds64;                                          // [wpb][max_ns]
    uint16_t *seg_of = reinterpret_cast<uint16_t *>(seg_key + (size_t)wpb * max_ns);   // [max_nt]
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u, tid = threadIdx.x, nthr = wpb * 64;
    const uint32_t j = jb + blockIdx.x / grp_per_job;
    const uint32_t r = (blockIdx.x % grp_per_job) * wpb + wave;
    const uint32_t t0 = tb.triple_off[j], nt = tb.triple_off[j + 1] - t0;
    const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
    for (uint32_t s = tid; s < ns; s += nthr) {
        const uint32_t first = tb.seg_first[s0 + s];
        const uint32_t last = s + 1 < ns ? tb.seg_first[s0 + s + 1] : nt;
        for (uint32_t t = first; t < last; ++t) seg_of[t] = (uint16_t)s;
    }
    for (uint32_t i = tid; i < wpb * max_ns; i += nthr) seg_key[i] = 0ull;
    __syncthreads();
    if (r >= n_rows || nt == 0) return;
    unsigned long long *my = seg_key + (size_t)wave * max_ns;
    const v4f *row = reinterpret_cast<const v4f *>(thr + 16ull * n_rows * (uint64_t)(t0 - tb.triple_off[jb]) +
                                                   (uint64_t)r * nt * 16);
    const uint32_t n_vec = nt * 4, last_vec = n_vec - 1;      // 16-byte elements of the row
    // loads past the end are clamped to the last element (and ignored), which keeps them branch-free
    v4f cur[BEST_UNROLL], nxt[BEST_UNROLL];
#pragma unroll
    for (uint32_t u = 0; u < BEST_UNROLL; ++u) {
        const uint32_t i = u * 64 + lane;
        cur[u] = __builtin_nontemporal_load(row + (i < n_vec ? i : last_vec));
    }
    for (uint32_t base = 0; base < n_vec; base += BEST_UNROLL * 64) {
#pragma unroll
        for (uint32_t u = 0; u < BEST_UNROLL; ++u) {
            const uint32_t i = base + (BEST_UNROLL + u) * 64 + lane;
            nxt[u] = __builtin_nontemporal_load(row + (i < n_vec ? i : last_vec));
        }
#pragma unroll
        for (uint32_t u = 0; u < BEST_UNROLL; ++u) {
            const uint32_t i = base + u * 64 + lane;
            const uint32_t plan0 = i * 4;
            unsigned long long k = make_key(cur[u].x, plan0);
            k = max_u64(k, make_key(cur[u].y, plan0 + 1));
            k = max_u64(k, make_key(cur[u].z, plan0 + 2));
            k = max_u64(k, make_key(cur[u].w, plan0 + 3));
            k = max_u64(k, dpp_u64<0xB1>(k));               // quad_perm [1,0,3,2]
            k = max_u64(k, dpp_u64<0x4E>(k));               // quad_perm [2,3,0,1]
            if ((lane & 3u) == 0 && i < n_vec && (k >> 32)) atomicMax(&my[seg_of[i >> 2]], k);
        }
#pragma unroll
        for (uint32_t u = 0; u < BEST_UNROLL; ++u) cur[u] = nxt[u];
    }
    const uint64_t sbase = (uint64_t)n_rows * (s0 - tb.seg_off[jb]) + (uint64_t)r * ns;
    for (uint32_t s = lane; s < ns; s += 64) {
        const unsigned long long k = my[s];
        best_thr[sbase + s] = key_thr(k);
        best_plan[sbase + s] = key_plan(k);
    }
}

// ------------------------------------------- evaluation and best plan in one pass
// The evaluation kernel's grid, thread mapping and stores (a workgroup takes 64 triples of a job, a thread owns
// (triple, ZeRO stage), a wavefront writes 1 KiB contiguous per row); in addition the workgroup keeps, per row and
// per segment that its tile touches, the packed key of the best plan in LDS: the candidate tensor is written once
// and never read back.  The options without offload are the same in every row and the offload options depend on the
// CPU level only (the memory tier masks them), so the four lanes of a triple reduce their keys once per tile and
// once per CPU level (two DPP steps each); a row then costs the quad leader a select and one LDS atomic maximum.
// The triples of a job are ordered by segment, so only the first and the last segment of a tile can continue in a
// neighbouring tile: the segments that lie inside the tile are written out as results, the (at most two) others as
// partial keys, which k_merge_spanning combines.  The keys are those of k_best_plan on the values stored, so the
// results are the same bits.
#ifndef EB_TILE
#define EB_TILE 64                               // triples per workgroup of the one-pass kernel
#endif
constexpr int EB_THREADS = 4 * EB_TILE;

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// A workgroup barrier that orders LDS traffic only: every wavefront waits for its own LDS operations (lgkmcnt 0), not
// for its global loads and stores, which __syncthreads() would also drain.  Enough where the data exchanged is in LDS.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("" ::: "memory");               // the compiler keeps memory accesses on their side of the barrier
    __builtin_amdgcn_s_waitcnt(0xC07F);          // vmcnt 63, expcnt 7, lgkmcnt 0
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// index of a (job, tile) among the tiles of a call: tiles of different jobs never share an index (a job adds at
// least its own number of tiles: floor(a + b) >= floor(a) + floor(b), and the job's own 1 covers a last partial tile)
__device__ __forceinline__ uint32_t tile_index(const TableDev &tb, uint32_t jb, uint32_t j, uint32_t tile) {
    return (tb.triple_off[j] - tb.triple_off[jb]) / EB_TILE + (j - jb) + tile;
}

template <bool WITH_FEAS>
__global__ __launch_bounds__(EB_THREADS) void k_eval_best(JobDev jobs, TableDev tb, GridDev grid, rk_env env, uint32_t jb,
                                                            uint32_t option_mask, uint32_t c_per_block, uint32_t key_stride,
                                                            float *__restrict__ thr, uint8_t *__restrict__ feas,
                                                            float *__restrict__ best_thr, uint32_t *__restrict__ best_plan,
                                                            unsigned long long *__restrict__ partial) {
    // [rows of this workgroup][key_stride local segments]; key_stride = min(64, longest segment list of the table)
    extern __shared__ unsigned long long seg_key[];
    __shared__ uint16_t seg_of[EB_TILE];                   // segment of each triple of the tile
    __shared__ uint32_t seg_lo_sh;                                   // segment of the tile's first triple
    const uint32_t tid = threadIdx.x;
    const uint32_t j = jb + blockIdx.y;
    const uint32_t t0 = tb.triple_off[j], nt = tb.triple_off[j + 1] - t0;
    const uint32_t tile_lo = blockIdx.x * EB_TILE;
    if (tile_lo >= nt) return;
    const uint32_t tile_hi = tile_lo + EB_TILE < nt ? tile_lo + EB_TILE : nt;
    const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
    const uint32_t tl = tile_lo + (tid >> 2);                        // the four lanes of a quad share tl
    const bool active = tl < tile_hi;
    const uint32_t packed_triple = active ? tb.triples[t0 + tl] : 0u;
    const uint32_t z = tid & 3u;
    const uint32_t n_rows = grid.n_cpu * grid.n_mem;
    const uint64_t cbase = 16ull * n_rows * (uint64_t)(t0 - tb.triple_off[jb]);
    const uint32_t c_lo = blockIdx.z * c_per_block;
    const uint32_t c_hi = c_lo + c_per_block < grid.n_cpu ? c_lo + c_per_block : grid.n_cpu;
    const uint32_t rows_here = (c_hi - c_lo) * grid.n_mem;
    // Where the results go.  Read here and not where they are used: a load after the candidate stores would make the
    // wavefront wait for all of them (the counter it waits on counts loads and stores alike, in order).
    const uint64_t sbase = (uint64_t)n_rows * (s0 - tb.seg_off[jb]);
    const uint64_t pbase = (uint64_t)tile_index(tb, jb, j, blockIdx.x) * 2 * n_rows;
    const Job J = load_job(jobs, j);

    // Which segments the tile touches; whether its first and its last segment go on in a neighbouring tile.  The loads
    // of this part are issued before the arithmetic below and used after it.
    __shared__ uint32_t first_open_sh, last_open_sh;
    uint32_t my_first[2] = {0u, 0u}, my_end[2] = {0u, 0u};           // a thread looks at segments tid and tid + 256 here,
    for (uint32_t k = 0; k < 2; ++k) {                               // at the others (jobs with more than 512) below
        const uint32_t s = tid + k * EB_THREADS;
        if (s < ns) {
            my_first[k] = tb.seg_first[s0 + s];
            my_end[k] = s + 1 < ns ? tb.seg_first[s0 + s + 1] : nt;
        }
    }

    // everything that does not depend on the row (as in k_eval)
    Triple T = {};
    float plain[2] = {0.f, 0.f};
    uint32_t why_plain[2] = {0u, 0u}, why_off[2] = {0u, 0u};
    bool any_off = false;
    Offload O = {};
    float need_host = 0.f, quad_host = 0.f;
    unsigned long long k_plain = 0ull;
    const uint32_t plan0 = tl * 16 + z * 4;
    if (active) {
        T = triple_terms(J, env, packed_triple);
#pragma unroll
        for (uint32_t gc = 0; gc < 2; ++gc) {
            const bool allowed = (option_mask >> (z * 4 + gc * 2)) & 1u;
            const bool fits = gpu_mem_fits(J, env, T, z, gc, 0);
            why_plain[gc] = allowed ? (fits ? 0u : RK_INFEASIBLE_GPU_MEM) : RK_INFEASIBLE_STRUCT;
            plain[gc] = why_plain[gc] ? 0.f : thr_plain(J, T, z, gc);
        }
#pragma unroll
        for (uint32_t gc = 0; gc < 2; ++gc) {
            const bool allowed = z >= 2 && ((option_mask >> (z * 4 + gc * 2 + 1)) & 1u);
            why_off[gc] = allowed ? (gpu_mem_fits(J, env, T, z, gc, 1) ? 0u : RK_INFEASIBLE_GPU_MEM)
                                  : RK_INFEASIBLE_STRUCT;
        }
        any_off = z >= 2 && (!(why_off[0] & RK_INFEASIBLE_STRUCT) || !(why_off[1] & RK_INFEASIBLE_STRUCT));
        if (any_off) {
            O = offload_terms(J, env, T);
            need_host = host_bytes_needed(J, T);
        }
        // what the quad knows together: the best option without offload, and the host bytes of the triple (the same
        // in every lane that offloads, 0 in the others; not negative, so the float maximum picks it)
        k_plain = max_u64(make_key(plain[0], plan0), make_key(plain[1], plan0 + 2));
        k_plain = max_u64(k_plain, dpp_u64<0xB1>(k_plain));                            // quad_perm [1,0,3,2]
        k_plain = max_u64(k_plain, dpp_u64<0x4E>(k_plain));                            // quad_perm [2,3,0,1]
        quad_host = fmaxf(need_host, dpp_f32<0xB1>(need_host));
        quad_host = fmaxf(quad_host, dpp_f32<0x4E>(quad_host));
    }

    // the triple -> segment map of the tile, and empty keys
    auto note_segment = [&](uint32_t s, uint32_t first, uint32_t end) {
        if (first < tile_hi && end > tile_lo) {
            if (first <= tile_lo) {                                  // it holds the tile's first triple
                seg_lo_sh = s;
                first_open_sh = (first < tile_lo || end > tile_hi) ? 1u : 0u;
            }
            if (end >= tile_hi) last_open_sh = end > tile_hi ? 1u : 0u;   // it holds the tile's last triple
            const uint32_t a = first > tile_lo ? first : tile_lo, b = end < tile_hi ? end : tile_hi;
            for (uint32_t t = a; t < b; ++t) seg_of[t - tile_lo] = (uint16_t)s;
        }
    };
    for (uint32_t k = 0; k < 2; ++k)
        if (tid + k * EB_THREADS < ns) note_segment(tid + k * EB_THREADS, my_first[k], my_end[k]);
    for (uint32_t s = tid + 2 * EB_THREADS; s < ns; s += EB_THREADS)
        note_segment(s, tb.seg_first[s0 + s], s + 1 < ns ? tb.seg_first[s0 + s + 1] : nt);
    for (uint32_t i = tid; i < rows_here * key_stride; i += EB_THREADS) seg_key[i] = 0ull;
    lds_barrier();
    const uint32_t seg_lo = seg_lo_sh;
    const uint32_t n_seg_here = seg_of[tile_hi - 1 - tile_lo] - seg_lo + 1;

    if (active) {
        unsigned long long *keys = seg_key + (seg_of[tl - tile_lo] - seg_lo);
        for (uint32_t ci = c_lo; ci < c_hi; ++ci) {
            float off_thr[2] = {0.f, 0.f};
            if (any_off) {
                const float sw = swap_term(J, O, cpus_of(grid, ci, T.g));
                off_thr[0] = thr_offload(T, O, 0, sw);
                off_thr[1] = thr_offload(T, O, 1, sw);
            }
            // the best of all options when the tier holds the offloaded state
            unsigned long long k_all = max_u64(make_key(why_off[0] ? 0.f : off_thr[0], plan0 + 1),
                                               make_key(why_off[1] ? 0.f : off_thr[1], plan0 + 3));
            k_all = max_u64(k_all, dpp_u64<0xB1>(k_all));
            k_all = max_u64(k_all, dpp_u64<0x4E>(k_all));
            k_all = max_u64(k_all, k_plain);
            for (uint32_t mi = 0; mi < grid.n_mem; ++mi) {
                const float tier = tier_bytes(grid, mi, T.g);
                uint32_t w0 = why_off[0], w1 = why_off[1];
                if (any_off && !(need_host <= tier)) {
                    if (!(w0 & RK_INFEASIBLE_STRUCT)) w0 |= RK_INFEASIBLE_HOST_MEM;
                    if (!(w1 & RK_INFEASIBLE_STRUCT)) w1 |= RK_INFEASIBLE_HOST_MEM;
                }
                v4f v;
                v.x = plain[0];
                v.y = w0 ? 0.f : off_thr[0];
                v.z = plain[1];
                v.w = w1 ? 0.f : off_thr[1];
                const uint64_t idx = cbase + ((uint64_t)(ci * grid.n_mem + mi) * nt + tl) * 16 + z * 4;
                *reinterpret_cast<v4f *>(thr + idx) = v;
                if (WITH_FEAS) {
                    const uint32_t packed = why_plain[0] | (w0 << 8) | (why_plain[1] << 16) | (w1 << 24);
                    *reinterpret_cast<uint32_t *>(feas + idx) = packed;
                }
                const unsigned long long k = quad_host <= tier ? k_all : k_plain;
                if (z == 0 && (k >> 32)) atomicMax(keys + ((ci - c_lo) * grid.n_mem + mi) * key_stride, k);
            }
        }
    }
    lds_barrier();                                                                     // the stores above need not have landed

    // a segment that lies inside the tile is finished; one that goes on in a neighbouring tile leaves its key: in
    // slot 0 if it holds the tile's first triple, else (it then holds the last one) in slot 1
    const bool first_open = first_open_sh != 0u, last_open = last_open_sh != 0u;
    for (uint32_t i = tid; i < rows_here * n_seg_here; i += EB_THREADS) {
        const uint32_t r_l = i / n_seg_here, q = i - r_l * n_seg_here, s = seg_lo + q;
        const uint32_t r = c_lo * grid.n_mem + r_l;
        const unsigned long long k = seg_key[r_l * key_stride + q];
        const bool open = q == 0 ? first_open : (q + 1 == n_seg_here && last_open);
        if (!open) {
            best_thr[sbase + (uint64_t)r * ns + s] = key_thr(k);
            best_plan[sbase + (uint64_t)r * ns + s] = key_plan(k);
        } else {
            partial[pbase + (q == 0 ? 0u : 1u) * n_rows + r] = k;
        }
    }
}

// The segments of a job that span tiles: the maximum of the keys their tiles left.  Half a wavefront per job: its
// 32 lanes look at 32 segments at a time, and for every one of them that spans tiles the lanes take a row each.
constexpr int MERGE_THREADS = 256;
constexpr int MERGE_LANES = 32;
__global__ __launch_bounds__(MERGE_THREADS) void k_merge_spanning(TableDev tb, uint32_t n_rows, uint32_t jb, uint32_t n_jobs,
                                                                  const unsigned long long *__restrict__ partial,
                                                                  float *__restrict__ best_thr,
                                                                  uint32_t *__restrict__ best_plan) {
    const uint32_t lane = threadIdx.x % MERGE_LANES;
    const uint32_t slot_in_block = threadIdx.x / MERGE_LANES;
    const uint32_t jl = blockIdx.x * (MERGE_THREADS / MERGE_LANES) + slot_in_block;
    if (jl >= n_jobs) return;
    const uint32_t j = jb + jl;
    const uint32_t t0 = tb.triple_off[j], nt = tb.triple_off[j + 1] - t0;
    if (nt <= (uint32_t)EB_TILE) return;                             // one tile: nothing spans
    const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
    const uint64_t sbase = (uint64_t)n_rows * (s0 - tb.seg_off[jb]);
    const uint64_t tile0 = tile_index(tb, jb, j, 0);
    // the half of the wavefront this job has: shuffles and ballots stay inside it
    const uint32_t half = (threadIdx.x & 63u) / MERGE_LANES;
    for (uint32_t sb = 0; sb < ns; sb += MERGE_LANES) {
        const uint32_t s = sb + lane;
        uint32_t first = 0, end = 0;
        if (s < ns) {
            first = tb.seg_first[s0 + s];
            end = s + 1 < ns ? tb.seg_first[s0 + s + 1] : nt;
        }
        const bool spans = s < ns && first / EB_TILE != (end - 1) / EB_TILE;
        uint32_t todo = (uint32_t)(__ballot(spans) >> (half * MERGE_LANES));
        while (todo) {
            const uint32_t src = (uint32_t)__ffs((int)todo) - 1u;
            todo &= todo - 1u;
            const uint32_t f = (uint32_t)__shfl((int)first, (int)(half * MERGE_LANES + src), 64);
            const uint32_t e = (uint32_t)__shfl((int)end, (int)(half * MERGE_LANES + src), 64);
            const uint32_t ta = f / EB_TILE, tz = (e - 1) / EB_TILE;
            for (uint32_t r = lane; r < n_rows; r += MERGE_LANES) {
                unsigned long long k = 0;
                for (uint32_t t = ta; t <= tz; ++t) {
                    const uint32_t slot = f <= t * EB_TILE ? 0u : 1u;                  // it holds that tile's first triple
                    k = max_u64(k, partial[((tile0 + t) * 2 + slot) * n_rows + r]);
                }
                best_thr[sbase + (uint64_t)r * ns + sb + src] = key_thr(k);
                best_plan[sbase + (uint64_t)r * ns + sb + src] = key_plan(k);
            }
        }
    }
}

// ------------------------------------------------------------------- curves
// One workgroup per job; its wavefronts split the job's rows.  A wavefront
// walks its rows, which are contiguous in memory, 64 entries at a time: each
// lane packs its entry into a key (throughput bits, inverted segment index,
// GPUs of the segment), the running maximum along the row is a segmented scan
// by shuffles (lower segment index wins among equal throughputs, as in the
// step-by-step definition), and a row that continues from the previous 64
// entries takes their last key along.  The plan of an entry is loaded with its
// throughput and moves through the scan with the key.
constexpr int CURVE_THREADS = 256;

__global__ __launch_bounds__(CURVE_THREADS) void k_curves(TableDev tb, uint32_t n_rows, uint32_t jb,
                                                          const float *__restrict__ best_thr,
                                                          const uint32_t *__restrict__ best_plan,
                                                          float *__restrict__ curve_thr, uint32_t *__restrict__ curve_plan,
                                                          uint32_t *__restrict__ curve_g) {
    constexpr uint32_t WAVES = CURVE_THREADS / 64;
    const uint32_t j = jb + blockIdx.x, lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t s0 = tb.seg_off[j], ns = tb.seg_off[j + 1] - s0;
    if (ns == 0) return;
    const uint32_t per = (n_rows + WAVES - 1) / WAVES;
    const uint32_t r_lo = wave * per < n_rows ? wave * per : n_rows;
    const uint32_t r_hi = r_lo + per < n_rows ? r_lo + per : n_rows;
    const uint32_t n = (r_hi - r_lo) * ns;                          // this wavefront's entries; they start a row
    const uint64_t off = (uint64_t)n_rows * (s0 - tb.seg_off[jb]) + (uint64_t)r_lo * ns;
    unsigned long long carry = 0;                                   // key at the end of the previous 64 entries
    uint32_t carry_plan = RK_NO_PLAN;                               // and the plan that goes with it
    for (uint32_t base = 0; base < n; base += 64) {
        const uint32_t i = base + lane;
        const bool in = i < n;
        const uint32_t s = i % ns;                                  // place in its row
        // the three loads do not depend on each other; the plan travels with the key through the scan
        float v = 0.f;
        uint32_t plan = RK_NO_PLAN, g = 0;
        if (in) {
            v = best_thr[off + i];
            plan = best_plan[off + i];
            g = tb.seg_g[s0 + s];
        }
        unsigned long long key = 0;                                 // 0 = nothing feasible so far
        if (v > 0.f) key = ((unsigned long long)__float_as_uint(v) << 32) | ((0xFFFFu - s) << 16) | g;
#pragma unroll
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const unsigned long long o = __shfl_up(key, d, 64);
            const uint32_t op = __shfl_up(plan, d, 64);
            if (lane >= d && s >= d && o > key) {                   // the lane d below is in the same row
                key = o;
                plan = op;
            }
        }
        if (s > lane && carry > key) {                              // the row began before these 64 entries
            key = carry;
            plan = carry_plan;
        }
        carry = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(key >> 32), 63) << 32) |
                (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)key, 63);
        carry_plan = (uint32_t)__builtin_amdgcn_readlane((int)plan, 63);
        if (in) {
            curve_thr[off + i] = __uint_as_float((uint32_t)(key >> 32));
            curve_plan[off + i] = key ? plan : RK_NO_PLAN;
            curve_g[off + i] = (uint32_t)key & 0xFFFFu;
        }
    }
}

}  // namespace

extern "C" {

int32_t rk_eval_candidates(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table,
                           const rk_alloc_grid *grid, const rk_env *env, uint32_t jb, uint32_t je,
                           float *thr, uint8_t *feas, uint64_t cap, uint64_t *n_needed) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs is null");
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if (jobs->n_jobs != table->n_jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs and table disagree on n_jobs");
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if ((rc = rk_check_env(ctx, env))) return rc;
    RK_HIP(ctx, hipSetDevice(ctx->device));
    uint64_t nt, ns;
    if ((rc = rk_range_offsets(ctx, table, jb, je, &nt, &ns))) return rc;
    const uint64_t n_rows = (uint64_t)grid->n_cpu * grid->n_mem;
    const uint64_t need = 16ull * n_rows * nt;
    if (n_needed) *n_needed = need;
    if (need == 0) return RK_OK;
    if (!thr) return rk_fail(ctx, RK_ERR_INVALID_ARG, "thr is null");
    if (cap < need) return rk_fail(ctx, RK_ERR_CAPACITY, "thr holds %llu candidates, %llu needed",
                                   (unsigned long long)cap, (unsigned long long)need);
    if (((uintptr_t)thr & 15u) || ((uintptr_t)feas & 15u)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "output not 16-byte aligned");

    const uint32_t bx = (table->max_triples_per_job + TRIPLES_PER_BLOCK - 1) / TRIPLES_PER_BLOCK;
    const uint32_t nj = je - jb;
    // split the CPU levels over blockIdx.z when there are few jobs, so the chip is filled
    uint32_t split = 1;
    const uint64_t blocks = (uint64_t)bx * nj;
    if (blocks < 2048) {
        split = (uint32_t)((2048 + blocks - 1) / blocks);
        if (split > grid->n_cpu) split = grid->n_cpu;
    }
    const uint32_t c_per_block = (grid->n_cpu + split - 1) / split;
    split = (grid->n_cpu + c_per_block - 1) / c_per_block;
    if (nj > 65535u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 65535 jobs in one call; use job ranges");
    const dim3 g3(bx, nj, split);
    const JobDev jd = job_dev(jobs);
    const TableDev td = table_dev(table);
    const GridDev gd = grid_dev(grid);
    if (feas)
        k_eval<true><<<g3, EVAL_THREADS, 0, ctx->stream>>>(jd, td, gd, *env, jb, table->option_mask, c_per_block, thr, feas);
    else
        k_eval<false><<<g3, EVAL_THREADS, 0, ctx->stream>>>(jd, td, gd, *env, jb, table->option_mask, c_per_block, thr, nullptr);
    RK_CHECK_LAUNCH(ctx, "k_eval");
    return RK_OK;
}

int32_t rk_best_plan(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid, uint32_t jb,
                     uint32_t je, const float *thr, float *best_thr, uint32_t *best_plan, uint64_t cap_segs,
                     uint64_t *n_needed) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    RK_HIP(ctx, hipSetDevice(ctx->device));
    uint64_t nt, ns;
    if ((rc = rk_range_offsets(ctx, table, jb, je, &nt, &ns))) return rc;
    const uint64_t n_rows = (uint64_t)grid->n_cpu * grid->n_mem;
    const uint64_t need = n_rows * ns;
    if (n_needed) *n_needed = need;
    if (need == 0) return RK_OK;
    if (!thr || !best_thr || !best_plan) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null buffer");
    if (cap_segs < need) return rk_fail(ctx, RK_ERR_CAPACITY, "outputs hold %llu entries, %llu needed",
                                        (unsigned long long)cap_segs, (unsigned long long)need);
    if ((uintptr_t)thr & 15u) return rk_fail(ctx, RK_ERR_INVALID_ARG, "thr not 16-byte aligned");
    // wavefronts (rows) per workgroup: split the job's rows evenly over as few workgroups as possible
    const uint32_t max_nt = table->max_triples_per_job ? table->max_triples_per_job : 1;
    const uint32_t max_ns = table->max_segs_per_job ? table->max_segs_per_job : 1;
    uint32_t cap_waves = (uint32_t)((56 * 1024 - ((size_t)max_nt * 2 + 8)) / ((size_t)max_ns * 8));
    if (cap_waves < 1) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "too many segments per job for the best-plan kernel");
    if (cap_waves > BEST_MAX_WAVES) cap_waves = BEST_MAX_WAVES;
    const uint32_t groups = (uint32_t)((n_rows + cap_waves - 1) / cap_waves);
    const uint32_t wpb = (uint32_t)((n_rows + groups - 1) / groups);
    const uint64_t blocks = (uint64_t)(je - jb) * groups;
    if (blocks > 0x7FFFFFFFull) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "too many rows in one call; use job ranges");
    const size_t lds = (size_t)wpb * max_ns * 8 + (((size_t)max_nt * 2 + 7) & ~(size_t)7);
    k_best_plan<<<(uint32_t)blocks, wpb * 64, lds, ctx->stream>>>(table_dev(table), (uint32_t)n_rows, jb, wpb, groups,
                                                                 max_nt, max_ns, thr, best_thr, best_plan);
    RK_CHECK_LAUNCH(ctx, "k_best_plan");
    return RK_OK;
}

int32_t rk_eval_best_plan(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_table *table, const rk_alloc_grid *grid,
                          const rk_env *env, uint32_t jb, uint32_t je, float *thr, uint8_t *feas, uint64_t cap,
                          float *best_thr, uint32_t *best_plan, uint64_t cap_segs) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if (!jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs is null");
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if (jobs->n_jobs != table->n_jobs) return rk_fail(ctx, RK_ERR_INVALID_ARG, "jobs and table disagree on n_jobs");
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    if ((rc = rk_check_env(ctx, env))) return rc;
    RK_HIP(ctx, hipSetDevice(ctx->device));
    uint64_t nt, ns;
    if ((rc = rk_range_offsets(ctx, table, jb, je, &nt, &ns))) return rc;
    const uint64_t n_rows = (uint64_t)grid->n_cpu * grid->n_mem;
    const uint64_t need = 16ull * n_rows * nt, need_segs = n_rows * ns;
    if (need == 0) return RK_OK;
    if (!thr || !best_thr || !best_plan) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null buffer");
    if (cap < need) return rk_fail(ctx, RK_ERR_CAPACITY, "thr holds %llu candidates, %llu needed",
                                   (unsigned long long)cap, (unsigned long long)need);
    if (cap_segs < need_segs) return rk_fail(ctx, RK_ERR_CAPACITY, "outputs hold %llu entries, %llu needed",
                                             (unsigned long long)cap_segs, (unsigned long long)need_segs);
    if (((uintptr_t)thr & 15u) || ((uintptr_t)feas & 15u)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "output not 16-byte aligned");

    const uint32_t nj = je - jb;
    if (nj > 65535u) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 65535 jobs in one call; use job ranges");
    const uint32_t bx = (table->max_triples_per_job + EB_TILE - 1) / EB_TILE;
    // a tile of 64 triples touches at most 64 segments, and no more than the longest segment list of the table; the
    // keys of a workgroup's rows stay within 8 KiB of LDS, so that LDS never limits how many workgroups a compute
    // unit holds: as many CPU levels per workgroup as that allows, the others over blockIdx.z; with few jobs the
    // levels are split further so that the chip is filled
    const uint32_t max_ns = table->max_segs_per_job ? table->max_segs_per_job : 1;
    const uint32_t key_stride = max_ns < (uint32_t)EB_TILE ? max_ns : (uint32_t)EB_TILE;
    const size_t level_bytes = (size_t)grid->n_mem * key_stride * 8;             // at most 16 * 64 * 8 = 8 KiB
    uint32_t c_per_block = (uint32_t)((8 * 1024) / level_bytes);
    if (c_per_block < 1) c_per_block = 1;
    if (c_per_block > grid->n_cpu) c_per_block = grid->n_cpu;
    const uint64_t blocks = (uint64_t)bx * nj;
    if (blocks < 2048) {
        uint32_t split = (uint32_t)((2048 + blocks - 1) / blocks);
        if (split > grid->n_cpu) split = grid->n_cpu;
        const uint32_t c2 = (grid->n_cpu + split - 1) / split;
        if (c2 < c_per_block) c_per_block = c2;
    }
    const uint32_t split = (grid->n_cpu + c_per_block - 1) / c_per_block;
    const size_t lds = (size_t)c_per_block * level_bytes;
    // partial keys of the segments that span tiles: two per (tile, row)
    const uint64_t n_tiles = nt / EB_TILE + nj + bx;
    unsigned long long *partial = nullptr;
    if ((rc = rk_scratch(ctx, SL_EVAL_PARTIAL, (size_t)(n_tiles * 2 * n_rows * 8), (void **)&partial))) return rc;
    const dim3 g3(bx, nj, split);
    const JobDev jd = job_dev(jobs);
    const TableDev td = table_dev(table);
    const GridDev gd = grid_dev(grid);
    if (feas)
        k_eval_best<true><<<g3, EB_THREADS, lds, ctx->stream>>>(jd, td, gd, *env, jb, table->option_mask, c_per_block,
                                                                 key_stride, thr, feas, best_thr, best_plan, partial);
    else
        k_eval_best<false><<<g3, EB_THREADS, lds, ctx->stream>>>(jd, td, gd, *env, jb, table->option_mask, c_per_block,
                                                                  key_stride, thr, nullptr, best_thr, best_plan, partial);
    RK_CHECK_LAUNCH(ctx, "k_eval_best");
    if (bx > 1) {
        const uint32_t per_block = MERGE_THREADS / MERGE_LANES;
        k_merge_spanning<<<(nj + per_block - 1) / per_block, MERGE_THREADS, 0, ctx->stream>>>(td, (uint32_t)n_rows, jb, nj, partial,
                                                                                           best_thr, best_plan);
        RK_CHECK_LAUNCH(ctx, "k_merge_spanning");
    }
    return RK_OK;
}

int32_t rk_curves(rk_ctx *ctx, const rk_plan_table *table, const rk_alloc_grid *grid, uint32_t jb, uint32_t je,
                  const float *best_thr, const uint32_t *best_plan, float *curve_thr, uint32_t *curve_plan,
                  uint32_t *curve_g, uint64_t cap_segs) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    int32_t rc;
    if ((rc = rk_check_table(ctx, table, jb, je))) return rc;
    if ((rc = rk_check_grid(ctx, grid))) return rc;
    RK_HIP(ctx, hipSetDevice(ctx->device));
    uint64_t nt, ns;
    if ((rc = rk_range_offsets(ctx, table, jb, je, &nt, &ns))) return rc;
    const uint64_t n_rows = (uint64_t)grid->n_cpu * grid->n_mem;
    const uint64_t need = n_rows * ns;
    if (need == 0) return RK_OK;
    if (!best_thr || !best_plan || !curve_thr || !curve_plan || !curve_g) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null buffer");
    if (cap_segs < need) return rk_fail(ctx, RK_ERR_CAPACITY, "outputs hold %llu entries, %llu needed",
                                        (unsigned long long)cap_segs, (unsigned long long)need);
    k_curves<<<je - jb, CURVE_THREADS, 0, ctx->stream>>>(table_dev(table), (uint32_t)n_rows, jb, best_thr, best_plan,
                                                        curve_thr, curve_plan, curve_g);
    RK_CHECK_LAUNCH(ctx, "k_curves");
    return RK_OK;
}

}  // extern "C"
