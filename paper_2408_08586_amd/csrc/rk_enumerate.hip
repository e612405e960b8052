// Plan enumeration on the device (paper Sec. 3: 3D-parallel plans with
// d*t*p = g, Table 1; Fig. 6: only some GPU counts are valid).
//
// One workgroup per job.  Instead of testing every g it builds the divisor
// lists of b/mu (data-parallel sizes) and of the layer count (pipeline sizes),
// forms the products d*t*p <= g_max with t in {1,2,4,8} for every allowed
// micro-batch shift v (d must divide b/(mu*2^v)), and orders them by the key
// (g, t, p, v) in LDS: a bitmap of the GPU counts that occur gives every key
// its segment (rank of its g among the distinct counts = a population count),
// the keys are gathered by segment, and only the few keys of one segment are
// compared with each other.  The counting pass also parks the
// sorted keys in a scratch buffer; after the exclusive scan of the counts the
// fill pass only decodes them into place (it repeats the search only when the
// scratch buffer was too small).  Jobs whose searches would be identical (same
// layer count, same number of micro-batches per step) share one: a hash table
// names a leader for each such group, only leaders search, the others take
// the leader's counts and decode the leader's parked keys.  The fill pass is launched while the counts
// are still on their way to the host: it checks on the device that the table
// is large enough and leaves it alone otherwise.
#include <cstring>

#include "rk_internal.h"

namespace {

constexpr int ENUM_THREADS = 256;
constexpr uint32_t MAX_T = RK_MAX_TRIPLES_PER_JOB;
constexpr uint32_t MAX_DIV = 1024;

enum { TOT_NT_LO = 0, TOT_NT_HI, TOT_NS_LO, TOT_NS_HI, TOT_MAX_T, TOT_MAX_S, TOT_ERR, TOT_CURSOR, TOT_WORDS };
enum { ERR_TOO_MANY_TRIPLES = 1, ERR_TOO_MANY_DIVISORS = 2, ERR_PARK_FULL = 4 };
enum { MODE_COUNT = 0, MODE_FILL_SEARCH = 1, MODE_FILL_PARKED = 2 };

// exclusive prefix sum of one value per thread over the workgroup (all threads call it): inside the
// wavefronts by shuffles, then the wavefronts' totals through LDS (lds: one word per wavefront)
__device__ uint32_t block_excl_scan(uint32_t v, uint32_t *lds, uint32_t *total) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, off, 64);
        if ((int)lane >= off) incl += o;
    }
    if (lane == 63u) lds[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (uint32_t w = 0; w < ENUM_THREADS / 64; ++w) {
        if (w < wave) before += lds[w];
        all += lds[w];
    }
    *total = all;
    __syncthreads();
    return before + incl - v;
}

// What the search of a job depends on (besides the bounds of the call): its layer count and b/mu; (0, 0) for a
// job that has no plan at all.
__device__ __forceinline__ void search_key(uint32_t l, uint32_t b, uint32_t mu, uint32_t &kl, uint32_t &kn) {
    const bool any = l > 0 && b > 0 && mu > 0 && (b % mu) == 0;
    kl = any ? l : 0u;
    kn = any ? b / mu : 0u;
}

__device__ __forceinline__ uint32_t search_hash(uint32_t kl, uint32_t kn) {
    uint32_t h = (kl * 0x9E3779B1u) ^ (kn * 0x85EBCA77u);
    h ^= h >> 15;
    h *= 0x2C1B3C6Du;
    h ^= h >> 12;
    return h;
}

// leader[j] = the job whose search job j shares (itself for the leaders).  Open addressing with linear probing,
// an entry is a job index + 1 and never changes once set; the table has at least twice as many slots as there are
// jobs, so every probe sequence ends at an empty slot or at the job's own kind, and nobody waits for anybody.
// Equal jobs of a workgroup first elect one of them through a table in LDS; only that one goes to the global table.
constexpr int LEAD_THREADS = 256;
constexpr uint32_t SHARE_MIN_JOBS = 2048;                  // calls with fewer jobs do not look for equal ones

__global__ __launch_bounds__(LEAD_THREADS) void k_enum_leaders(const uint32_t *__restrict__ layers,
                                                               const uint32_t *__restrict__ gbatch,
                                                               const uint32_t *__restrict__ mbatch, uint32_t n_jobs,
                                                               uint32_t *__restrict__ tab, uint32_t tab_mask,
                                                               uint32_t *__restrict__ leader) {
    __shared__ uint32_t ltab[2 * LEAD_THREADS], s_kl[LEAD_THREADS], s_kn[LEAD_THREADS], s_lead[LEAD_THREADS];
    const uint32_t tid = threadIdx.x, j = blockIdx.x * LEAD_THREADS + tid;
    const bool valid = j < n_jobs;
    uint32_t kl = 0, kn = 0;
    if (valid) search_key(layers[j], gbatch[j], mbatch[j], kl, kn);
    s_kl[tid] = kl;
    s_kn[tid] = kn;
    ltab[tid] = 0u;
    ltab[tid + LEAD_THREADS] = 0u;
    __syncthreads();
    const uint32_t h = search_hash(kl, kn);
    uint32_t rep = tid;                                     // the thread that speaks for this job's kind
    if (valid) {
        uint32_t slot = h & (2u * LEAD_THREADS - 1u);
        for (;;) {
            const uint32_t old = atomicCAS(&ltab[slot], 0u, tid + 1u);
            if (old == 0u) break;
            if (s_kl[old - 1u] == kl && s_kn[old - 1u] == kn) { rep = old - 1u; break; }
            slot = (slot + 1u) & (2u * LEAD_THREADS - 1u);
        }
    }
    if (valid && rep == tid) {
        uint32_t slot = h & tab_mask, lead = j;
        for (;;) {
            const uint32_t old = atomicCAS(&tab[slot], 0u, j + 1u);
            if (old == 0u) break;
            const uint32_t o = old - 1u;
            uint32_t ol, on;
            search_key(layers[o], gbatch[o], mbatch[o], ol, on);
            if (ol == kl && on == kn) { lead = o; break; }
            slot = (slot + 1u) & tab_mask;
        }
        s_lead[tid] = lead;
    }
    __syncthreads();
    if (valid) leader[j] = s_lead[rep];
}

// the counts of a job that did not search are its leader's
__global__ __launch_bounds__(LEAD_THREADS) void k_spread_counts(const uint32_t *__restrict__ leader, uint32_t n_jobs,
                                                                uint32_t *__restrict__ cnt_t, uint32_t *__restrict__ cnt_s) {
    const uint32_t j = blockIdx.x * LEAD_THREADS + threadIdx.x;
    if (j >= n_jobs) return;
    const uint32_t l = leader[j];
    if (l != j) {
        cnt_t[j] = cnt_t[l];
        cnt_s[j] = cnt_s[l];
    }
}

template <int MODE>
__global__ __launch_bounds__(ENUM_THREADS) void k_enumerate(
    const uint32_t *__restrict__ layers, const uint32_t *__restrict__ gbatch,
    const uint32_t *__restrict__ mbatch, rk_plan_bounds bounds, const uint32_t *__restrict__ leader,
    uint32_t *__restrict__ cnt_t, uint32_t *__restrict__ cnt_s,
    uint32_t *__restrict__ park, uint32_t park_stride,
    const uint32_t *__restrict__ triple_off, const uint32_t *__restrict__ seg_off,
    uint32_t *__restrict__ triples, uint32_t *__restrict__ seg_g, uint32_t *__restrict__ seg_first,
    uint32_t *__restrict__ totals, uint64_t cap_triples, uint64_t cap_segs) {
    extern __shared__ uint32_t gmap[];                      // counting and search modes: bitmap of the GPU counts, word prefixes
    // Two arrays serve everything (a third would cost occupancy): `lists` holds the two divisor lists and later
    // the keys gathered by segment; `keys` holds the keys as they are found, then (once every thread has its keys
    // in registers) the segments' sizes and starts, and at the end the keys in order.
    __shared__ uint32_t lists[2 * MAX_DIV];
    uint32_t *dlist = lists, *plist = lists + MAX_DIV;
    __shared__ __align__(16) uint32_t keys[MAX_T + 4];
    static_assert(TOT_WORDS <= 16, "the totals share a block with the leaders' table");
    static_assert(2 * MAX_DIV >= MAX_T, "the gathered keys reuse the divisor lists");
    __shared__ uint32_t scan_tmp[ENUM_THREADS];
    __shared__ uint32_t nd, np, nk;

    const uint32_t j = blockIdx.x, tid = threadIdx.x;
    if (MODE == MODE_COUNT && leader && leader[j] != j) return;   // (whole workgroup) the leader searches for this job
    uint32_t cnt, err = 0;
    if (MODE == MODE_FILL_PARKED) {
        // launched before the host has seen the totals: nothing is written unless the
        // counting pass raised no flag and the table takes everything (same in all threads)
        const uint64_t nt = ((uint64_t)totals[TOT_NT_HI] << 32) | totals[TOT_NT_LO];
        const uint64_t ns = ((uint64_t)totals[TOT_NS_HI] << 32) | totals[TOT_NS_LO];
        if (totals[TOT_ERR] != 0u || nt > 0xFFFFFFFFull || nt > cap_triples || ns > cap_segs) return;
        cnt = cnt_t[j];
        const size_t at = (size_t)(leader ? leader[j] : j) * park_stride;   // the keys were parked by the job that searched
        for (uint32_t i = tid; i < cnt; i += ENUM_THREADS) keys[i] = park[at + i];
        __syncthreads();
    } else {
        const uint32_t l = layers[j], b = gbatch[j], mu = mbatch[j];
        if (tid == 0) { nd = 0; np = 0; nk = 0; }
        __syncthreads();

        const bool any = l > 0 && b > 0 && mu > 0 && (b % mu) == 0;
        const uint32_t n = any ? b / mu : 0;
        // divisors of n (data-parallel sizes) and of l (pipeline sizes), unordered
        // (every divisor d with d*d <= n brings n/d along, so the search stops at the square root)
        const uint32_t dmax = n < bounds.g_max ? n : bounds.g_max;
        for (uint32_t d = tid + 1; (uint64_t)d * d <= n; d += ENUM_THREADS) {
            const uint32_t e = n / d;
            if (e * d == n) {
                if (d <= dmax) { uint32_t i = atomicAdd(&nd, 1u); if (i < MAX_DIV) dlist[i] = d; }
                if (e != d && e <= dmax) { uint32_t i = atomicAdd(&nd, 1u); if (i < MAX_DIV) dlist[i] = e; }
            }
        }
        uint32_t pmax = l < bounds.pp_max ? l : bounds.pp_max;
        pmax = pmax < bounds.g_max ? pmax : bounds.g_max;
        if (!any) pmax = 0;
        for (uint32_t p = tid + 1; p <= pmax; p += ENUM_THREADS)
            if (l % p == 0) { uint32_t i = atomicAdd(&np, 1u); if (i < MAX_DIV) plist[i] = p; }
        __syncthreads();
        if (nd > MAX_DIV || np > MAX_DIV) err |= ERR_TOO_MANY_DIVISORS;
        const uint32_t cd = nd < MAX_DIV ? nd : MAX_DIV, cp = np < MAX_DIV ? np : MAX_DIV;

        // products d * 2^lt * p <= g_max (at most 1024 * 1024 * 4 combinations: 32-bit arithmetic)
        uint32_t nlt = 0;                               // tensor-parallel sizes allowed: 2^0..2^(nlt-1)
        for (uint32_t t = 1; t <= 8 && t <= bounds.tp_max; t <<= 1) ++nlt;
        const uint32_t pairs = cd * cp;
        for (uint32_t c = tid; c < pairs; c += ENUM_THREADS) {
            const uint32_t p = plist[c % cp], d = dlist[c / cp];
            const uint64_t dp = (uint64_t)d * p;
            // micro-batch shifts this d works with: mu*2^v divides b and d divides b/(mu*2^v)
            uint32_t vmask = 0;
            for (uint32_t v = 0; v < 4; ++v)
                if (((bounds.mu_mask >> v) & 1u) && (n & ((1u << v) - 1u)) == 0 && ((n >> v) % d) == 0) vmask |= 1u << v;
            for (uint32_t lt = 0; lt < nlt; ++lt) {
                const uint64_t g = dp << lt;
                if (g <= bounds.g_max) {
                    for (uint32_t v = 0; v < 4; ++v) {
                        if (!((vmask >> v) & 1u)) continue;
                        const uint32_t i = atomicAdd(&nk, 1u);
                        if (i < MAX_T) keys[i] = ((uint32_t)g << 16) | (lt << 14) | (p << 2) | v;
                    }
                }
            }
        }
        __syncthreads();
        if (nk > MAX_T) err |= ERR_TOO_MANY_TRIPLES;
        cnt = nk < MAX_T ? nk : MAX_T;

        // Sort.  Keys are distinct.  (1) bitmap of the GPU counts that occur; (2) population counts in front of
        // every bitmap word: a key's segment is the rank of its g among the distinct counts; (3) sizes of the
        // segments, every key takes a slot in its own; (4) starts of the segments; (5) keys gathered by segment;
        // (6) a key's final place = start of its segment + number of smaller keys inside it.
        constexpr uint32_t PER = MAX_T / ENUM_THREADS;          // keys per thread, at most
        const uint32_t n_words = (bounds.g_max >> 5) + 1u;
        uint32_t *bitmap = gmap, *before = gmap + n_words, *seg = keys, *gathered = lists;
        uint32_t mine[PER], slot[PER], place[PER];
#pragma unroll
        for (uint32_t r = 0; r < PER; ++r) {
            const uint32_t i = tid + r * ENUM_THREADS;
            mine[r] = i < cnt ? keys[i] : 0u;
        }
        for (uint32_t w = tid; w < n_words; w += ENUM_THREADS) bitmap[w] = 0u;
        __syncthreads();                                        // every key is in a register: `keys` becomes the segment table
        for (uint32_t i = tid; i <= cnt; i += ENUM_THREADS) seg[i] = 0u;     // there are at most cnt segments
#pragma unroll
        for (uint32_t r = 0; r < PER; ++r)
            if (tid + r * ENUM_THREADS < cnt) atomicOr(&bitmap[mine[r] >> 21], 1u << ((mine[r] >> 16) & 31u));
        __syncthreads();
        const uint32_t wpt = (n_words + ENUM_THREADS - 1) / ENUM_THREADS;
        const uint32_t w_lo = tid * wpt < n_words ? tid * wpt : n_words;
        const uint32_t w_hi = w_lo + wpt < n_words ? w_lo + wpt : n_words;
        uint32_t bits = 0;
        for (uint32_t w = w_lo; w < w_hi; ++w) bits += (uint32_t)__popc(bitmap[w]);
        uint32_t n_seg;
        uint32_t run = block_excl_scan(bits, scan_tmp, &n_seg);
        for (uint32_t w = w_lo; w < w_hi; ++w) { before[w] = run; run += (uint32_t)__popc(bitmap[w]); }
        __syncthreads();
        auto segment_of = [&](uint32_t key) -> uint32_t {
            const uint32_t g = key >> 16;
            return before[g >> 5] + (uint32_t)__popc(bitmap[g >> 5] & ((1u << (g & 31u)) - 1u));
        };
#pragma unroll
        for (uint32_t r = 0; r < PER; ++r)
            if (tid + r * ENUM_THREADS < cnt) slot[r] = atomicAdd(&seg[segment_of(mine[r])], 1u);
        __syncthreads();
        const uint32_t spt = (n_seg + ENUM_THREADS - 1) / ENUM_THREADS;
        const uint32_t s_lo = tid * spt < n_seg ? tid * spt : n_seg;
        const uint32_t s_hi = s_lo + spt < n_seg ? s_lo + spt : n_seg;
        uint32_t sizes = 0, all;
        for (uint32_t q = s_lo; q < s_hi; ++q) sizes += seg[q];
        run = block_excl_scan(sizes, scan_tmp, &all);
        for (uint32_t q = s_lo; q < s_hi; ++q) { const uint32_t n = seg[q]; seg[q] = run; run += n; }
        if (tid == 0) seg[n_seg] = cnt;
        __syncthreads();
#pragma unroll
        for (uint32_t r = 0; r < PER; ++r)
            if (tid + r * ENUM_THREADS < cnt) gathered[seg[segment_of(mine[r])] + slot[r]] = mine[r];
        __syncthreads();
#pragma unroll
        for (uint32_t r = 0; r < PER; ++r) {
            place[r] = 0;
            if (tid + r * ENUM_THREADS < cnt) {
                const uint32_t q = segment_of(mine[r]), a = seg[q], b = seg[q + 1];
                uint32_t rank = a;
                for (uint32_t x = a; x < b; ++x) rank += gathered[x] < mine[r] ? 1u : 0u;
                place[r] = rank;
            }
        }
        __syncthreads();                                        // the segment table has been read: `keys` takes the result
#pragma unroll
        for (uint32_t r = 0; r < PER; ++r)
            if (tid + r * ENUM_THREADS < cnt) keys[place[r]] = mine[r];
        __syncthreads();
    }
    const uint32_t *fin = keys;                                 // the keys in order

    // segments: runs of equal g.  Each thread owns a contiguous chunk.
    const uint32_t chunk = (cnt + ENUM_THREADS - 1) / ENUM_THREADS;
    const uint32_t lo = tid * chunk < cnt ? tid * chunk : cnt;
    const uint32_t hi = lo + chunk < cnt ? lo + chunk : cnt;
    uint32_t starts = 0;
    for (uint32_t i = lo; i < hi; ++i)
        starts += (i == 0 || (fin[i] >> 16) != (fin[i - 1] >> 16)) ? 1u : 0u;
    uint32_t nseg;
    uint32_t sidx = block_excl_scan(starts, scan_tmp, &nseg);

    if (MODE == MODE_COUNT) {
        if (tid == 0) {
            cnt_t[j] = cnt;
            cnt_s[j] = nseg;
            if (cnt > park_stride) err |= ERR_PARK_FULL;
            if (err) atomicOr(&totals[TOT_ERR], err);
        }
        // park the sorted keys in the job's slot for the fill pass, if they fit
        if (cnt <= park_stride) {
            const size_t at = (size_t)j * park_stride;
            for (uint32_t i = tid; i < cnt; i += ENUM_THREADS) park[at + i] = fin[i];
        }
        return;
    }
    const uint32_t t0 = triple_off[j], s0 = seg_off[j];
    for (uint32_t i = lo; i < hi; ++i) {
        const uint32_t k = fin[i];
        const uint32_t g = k >> 16, lt = (k >> 14) & 3u, p = (k >> 2) & 0xFFFu, v = k & 3u;
        const uint32_t d = g / (p << lt);
        triples[t0 + i] = d | (lt << 16) | (p << 18) | (v << 30);
        if (i == 0 || g != (fin[i - 1] >> 16)) {
            seg_g[s0 + sidx] = g;
            seg_first[s0 + sidx] = i;
            ++sidx;
        }
    }
}

// exclusive scan of the per-job counts, totals and maxima: one workgroup walks
// the jobs in tiles of 8192, every thread taking eight neighbouring jobs with
// two 16-byte loads per array (the next tile is requested before the current
// one is scanned); a thread sums its eight, the sums are scanned inside the
// wavefronts by shuffles and across them through LDS, and the offsets leave
// through LDS so that the stores are coalesced too.
// back: [16 words of totals | n_jobs + 1 triple offsets | n_jobs + 1 segment offsets], one piece for the host
// (the offsets only when the host keeps mirrors of them: back_offsets)
constexpr uint32_t SCAN_PER = 8, SCAN_TILE = 1024 * SCAN_PER;

struct Eight { uint32_t v[SCAN_PER]; };

// counts of jobs j0 .. j0+7 (0 beyond the end); cnt + j0 is 32-byte aligned
__device__ __forceinline__ Eight load_eight(const uint32_t *__restrict__ cnt, uint32_t j0, uint32_t n_jobs) {
    Eight e;
    if (j0 + SCAN_PER <= n_jobs) {
        const uint4 a = *reinterpret_cast<const uint4 *>(cnt + j0), b = *reinterpret_cast<const uint4 *>(cnt + j0 + 4);
        e.v[0] = a.x; e.v[1] = a.y; e.v[2] = a.z; e.v[3] = a.w;
        e.v[4] = b.x; e.v[5] = b.y; e.v[6] = b.z; e.v[7] = b.w;
    } else {
#pragma unroll
        for (uint32_t i = 0; i < SCAN_PER; ++i) e.v[i] = j0 + i < n_jobs ? cnt[j0 + i] : 0u;
    }
    return e;
}

__global__ __launch_bounds__(1024) void k_scan_counts(const uint32_t *__restrict__ cnt_t,
                                                      const uint32_t *__restrict__ cnt_s, uint32_t n_jobs,
                                                      uint32_t *__restrict__ off_t, uint32_t *__restrict__ off_s,
                                                      uint32_t *__restrict__ totals, uint32_t *__restrict__ back,
                                                      bool back_offsets) {
    __shared__ __align__(16) uint32_t buf_t[SCAN_TILE], buf_s[SCAN_TILE];
    __shared__ unsigned long long wave_t[16], wave_s[16];
    __shared__ uint32_t wave_mt[16], wave_ms[16];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    unsigned long long carry_t = 0, carry_s = 0;            // everything before the tile (same in every thread)
    uint32_t mt = 0, ms = 0;                                // running maxima of this thread's elements
    Eight nt_next = load_eight(cnt_t, tid * SCAN_PER, n_jobs), ns_next = load_eight(cnt_s, tid * SCAN_PER, n_jobs);
    for (uint32_t base = 0; base < n_jobs; base += SCAN_TILE) {
        const Eight ct = nt_next, cs = ns_next;
        if (base + SCAN_TILE < n_jobs) {
            nt_next = load_eight(cnt_t, base + SCAN_TILE + tid * SCAN_PER, n_jobs);
            ns_next = load_eight(cnt_s, base + SCAN_TILE + tid * SCAN_PER, n_jobs);
        }
        unsigned long long sum_t = 0, sum_s = 0;
#pragma unroll
        for (uint32_t i = 0; i < SCAN_PER; ++i) {
            sum_t += ct.v[i]; sum_s += cs.v[i];
            mt = ct.v[i] > mt ? ct.v[i] : mt;
            ms = cs.v[i] > ms ? cs.v[i] : ms;
        }
        unsigned long long it = sum_t, is = sum_s;          // inclusive scan of the threads' sums inside the wavefront
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned long long at = __shfl_up(it, off, 64), as = __shfl_up(is, off, 64);
            if ((int)lane >= off) { it += at; is += as; }
        }
        if (lane == 63u) { wave_t[wave] = it; wave_s[wave] = is; }
        __syncthreads();
        unsigned long long before_t = 0, before_s = 0, all_t = 0, all_s = 0;
#pragma unroll
        for (uint32_t w = 0; w < 16; ++w) {
            if (w < wave) { before_t += wave_t[w]; before_s += wave_s[w]; }
            all_t += wave_t[w]; all_s += wave_s[w];
        }
        uint32_t run_t = (uint32_t)(carry_t + before_t + it - sum_t), run_s = (uint32_t)(carry_s + before_s + is - sum_s);
        uint32_t ot[SCAN_PER], os[SCAN_PER];
#pragma unroll
        for (uint32_t i = 0; i < SCAN_PER; ++i) {
            ot[i] = run_t; os[i] = run_s;
            run_t += ct.v[i]; run_s += cs.v[i];
        }
        uint4 *dt = reinterpret_cast<uint4 *>(buf_t + tid * SCAN_PER), *ds = reinterpret_cast<uint4 *>(buf_s + tid * SCAN_PER);
        dt[0] = make_uint4(ot[0], ot[1], ot[2], ot[3]); dt[1] = make_uint4(ot[4], ot[5], ot[6], ot[7]);
        ds[0] = make_uint4(os[0], os[1], os[2], os[3]); ds[1] = make_uint4(os[4], os[5], os[6], os[7]);
        __syncthreads();
#pragma unroll
        for (uint32_t i = 0; i < SCAN_PER; ++i) {
            const uint32_t at = i * 1024 + tid, j = base + at;
            if (j < n_jobs) {
                const uint32_t a = buf_t[at], b = buf_s[at];
                off_t[j] = a;
                off_s[j] = b;
                if (back_offsets) {
                    back[16 + j] = a;
                    back[16 + n_jobs + 1 + j] = b;
                }
            }
        }
        carry_t += all_t; carry_s += all_s;
        __syncthreads();                                    // LDS is read before the next tile overwrites it
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t a = __shfl_xor(mt, off, 64), b = __shfl_xor(ms, off, 64);
        mt = a > mt ? a : mt; ms = b > ms ? b : ms;
    }
    if (lane == 0) { wave_mt[wave] = mt; wave_ms[wave] = ms; }
    __syncthreads();
    if (tid == 0) {
        for (uint32_t w = 0; w < 16; ++w) { mt = wave_mt[w] > mt ? wave_mt[w] : mt; ms = wave_ms[w] > ms ? wave_ms[w] : ms; }
        off_t[n_jobs] = (uint32_t)carry_t; off_s[n_jobs] = (uint32_t)carry_s;
        totals[TOT_NT_LO] = (uint32_t)carry_t; totals[TOT_NT_HI] = (uint32_t)(carry_t >> 32);
        totals[TOT_NS_LO] = (uint32_t)carry_s; totals[TOT_NS_HI] = (uint32_t)(carry_s >> 32);
        totals[TOT_MAX_T] = mt; totals[TOT_MAX_S] = ms;
        back[16 + n_jobs] = (uint32_t)carry_t; back[16 + 2 * n_jobs + 1] = (uint32_t)carry_s;
        back[TOT_NT_LO] = (uint32_t)carry_t; back[TOT_NT_HI] = (uint32_t)(carry_t >> 32);
        back[TOT_NS_LO] = (uint32_t)carry_s; back[TOT_NS_HI] = (uint32_t)(carry_s >> 32);
        back[TOT_MAX_T] = mt; back[TOT_MAX_S] = ms;
        back[TOT_ERR] = totals[TOT_ERR];                    // flags of the counting pass
    }
}

__global__ void k_zero_words(uint32_t *p, uint32_t n) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

}  // namespace

extern "C" int32_t rk_enumerate_plans(rk_ctx *ctx, const rk_jobs *jobs, const rk_plan_bounds *bounds,
                                      rk_plan_table *table) {
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!jobs || !bounds || !table) return rk_fail(ctx, RK_ERR_INVALID_ARG, "null argument");
    if (jobs->n_jobs > 0 && (!jobs->layers || !jobs->gbatch || !jobs->mbatch)) return rk_fail(ctx, RK_ERR_INVALID_ARG, "job arrays are null");
    if (bounds->g_max < 1 || bounds->g_max > RK_MAX_G) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "g_max must be in 1..%u", RK_MAX_G);
    if (bounds->pp_max < 1 || bounds->pp_max > RK_MAX_PP) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "pp_max must be in 1..%u", RK_MAX_PP);
    if (bounds->tp_max < 1) return rk_fail(ctx, RK_ERR_INVALID_ARG, "tp_max below 1");
    if (bounds->zero_mask > 0xF || bounds->gc_mask > 3 || bounds->off_mask > 3 || bounds->mu_mask > 0xF)
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "option mask has unknown bits");
    if (bounds->mu_mask == 0) return rk_fail(ctx, RK_ERR_INVALID_ARG, "mu_mask allows no micro-batch size");
    RK_HIP(ctx, hipSetDevice(ctx->device));

    const uint32_t J = jobs->n_jobs;
    uint32_t opt = 0;
    for (uint32_t o = 0; o < 16; ++o) {
        const uint32_t z = o >> 2, gc = (o >> 1) & 1u, off = o & 1u;
        if (((bounds->zero_mask >> z) & 1u) && ((bounds->gc_mask >> gc) & 1u) && ((bounds->off_mask >> off) & 1u))
            opt |= 1u << o;
    }
    table->option_mask = opt;
    table->n_jobs = J;
    table->n_triples = table->n_segs = 0;
    table->max_triples_per_job = table->max_segs_per_job = 0;

    uint32_t *cnt_t, *cnt_s, *totals, *off_t, *off_s, *park, *back;
    int32_t rc;
    if ((rc = rk_scratch(ctx, SL_CNT_T, (size_t)(2 * (size_t)J + 2) * 4, (void **)&cnt_t))) return rc;
    if ((rc = rk_scratch(ctx, SL_CNT_S, (size_t)(2 * (size_t)J + 2) * 4, (void **)&cnt_s))) return rc;
    // totals (16 words) and the leaders' hash table (a power of two, at least twice the jobs) are cleared together
    uint64_t tab_slots = 64;
    while (tab_slots < 2 * (uint64_t)J) tab_slots <<= 1;
    // (a call with few jobs searches for each of them: two more launches would cost more than they save)
    const bool share = J >= SHARE_MIN_JOBS;
    if (!share) tab_slots = 0;
    uint32_t *tab, *leader = nullptr;
    if ((rc = rk_scratch(ctx, SL_TOTALS, (size_t)(16 + tab_slots) * 4, (void **)&totals))) return rc;
    tab = totals + 16;
    if (share && (rc = rk_scratch(ctx, SL_ENUM_LEADER, ((size_t)J + 1) * 4, (void **)&leader))) return rc;
    // one slot per job for the parked keys: as wide as the widest job seen so far, or a first guess
    if (ctx->park_stride == 0) ctx->park_stride = 512;
    const uint32_t park_stride = ctx->park_stride;
    if ((rc = rk_scratch(ctx, SL_PARK, ((size_t)J * park_stride + 1) * 4, (void **)&park))) return rc;
    const bool fill = table->triples != nullptr;              // otherwise a sizing call
    if (fill && (!table->triple_off || !table->seg_off || !table->seg_g || !table->seg_first))
        return rk_fail(ctx, RK_ERR_INVALID_ARG, "table buffer is null");
    off_t = fill ? table->triple_off : cnt_t + J;             // offsets go straight into the table
    off_s = fill ? table->seg_off : cnt_s + J;
    // what comes back in one piece: totals, then the two offset arrays (pinned staging on the host)
    const size_t words_back = 16 + 2 * ((size_t)J + 1);
    if ((rc = rk_scratch(ctx, SL_ENUM_BACK, words_back * 4, (void **)&back))) return rc;
    if (ctx->h_stage_words < words_back) {
        if (ctx->h_stage) RK_HIP(ctx, hipHostFree(ctx->h_stage));
        ctx->h_stage = nullptr; ctx->h_stage_words = 0;
        RK_HIP(ctx, hipHostMalloc((void **)&ctx->h_stage, (words_back + words_back / 4) * 4, hipHostMallocDefault));
        ctx->h_stage_words = words_back + words_back / 4;
    }
    uint32_t *h = ctx->h_stage;
    if (!ctx->counts_ev) RK_HIP(ctx, hipEventCreateWithFlags(&ctx->counts_ev, hipEventDisableTiming));

    const size_t gmap_bytes = (size_t)((bounds->g_max >> 5) + 1u) * 2 * sizeof(uint32_t);   // bitmap + word prefixes
    k_zero_words<<<(uint32_t)((16 + tab_slots + 255) / 256), 256, 0, ctx->stream>>>(totals, (uint32_t)(16 + tab_slots));
    if (J > 0) {
        const uint32_t job_blocks = (J + LEAD_THREADS - 1) / LEAD_THREADS;
        if (share) {
            k_enum_leaders<<<job_blocks, LEAD_THREADS, 0, ctx->stream>>>(jobs->layers, jobs->gbatch, jobs->mbatch, J, tab,
                                                                        (uint32_t)(tab_slots - 1), leader);
            RK_CHECK_LAUNCH(ctx, "k_enum_leaders");
        }
        k_enumerate<MODE_COUNT><<<J, ENUM_THREADS, gmap_bytes, ctx->stream>>>(
            jobs->layers, jobs->gbatch, jobs->mbatch, *bounds, leader, cnt_t, cnt_s, park, park_stride,
            nullptr, nullptr, nullptr, nullptr, nullptr, totals, 0, 0);
        RK_CHECK_LAUNCH(ctx, "k_enumerate<count>");
        if (share) {
            k_spread_counts<<<job_blocks, LEAD_THREADS, 0, ctx->stream>>>(leader, J, cnt_t, cnt_s);
            RK_CHECK_LAUNCH(ctx, "k_spread_counts");
        }
    }
    const bool mirrors = fill && table->h_triple_off && table->h_seg_off;
    k_scan_counts<<<1, 1024, 0, ctx->stream>>>(cnt_t, cnt_s, J, off_t, off_s, totals, back, mirrors);
    RK_CHECK_LAUNCH(ctx, "k_scan_counts");
    RK_HIP(ctx, hipMemcpyAsync(h, back, (mirrors ? words_back : 16) * 4, hipMemcpyDeviceToHost, ctx->stream));
    RK_HIP(ctx, hipEventRecord(ctx->counts_ev, ctx->stream));
    // The fill pass goes out before the host knows the totals, so that the device does not wait for the
    // round trip: the kernel itself checks the flags and the table's capacity.
    if (fill && J > 0) {
        k_enumerate<MODE_FILL_PARKED><<<J, ENUM_THREADS, 0, ctx->stream>>>(
            jobs->layers, jobs->gbatch, jobs->mbatch, *bounds, leader, cnt_t, cnt_s, park, park_stride,
            off_t, off_s, table->triples, table->seg_g, table->seg_first, totals, table->cap_triples, table->cap_segs);
        RK_CHECK_LAUNCH(ctx, "k_enumerate<fill>");
    }
    RK_HIP(ctx, hipEventSynchronize(ctx->counts_ev));

    if (h[TOT_ERR] & ERR_TOO_MANY_TRIPLES) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "a job has more than %u triples", MAX_T);
    if (h[TOT_ERR] & ERR_TOO_MANY_DIVISORS) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "a job has more than %u candidate d or p sizes", MAX_DIV);
    const uint64_t nt = ((uint64_t)h[TOT_NT_HI] << 32) | h[TOT_NT_LO];
    const uint64_t ns = ((uint64_t)h[TOT_NS_HI] << 32) | h[TOT_NS_LO];
    if (nt > 0xFFFFFFFFull) return rk_fail(ctx, RK_ERR_UNSUPPORTED, "more than 2^32-1 triples");
    table->n_triples = nt;
    table->n_segs = ns;
    table->max_triples_per_job = h[TOT_MAX_T];
    table->max_segs_per_job = h[TOT_MAX_S];
    const bool parked = !(h[TOT_ERR] & ERR_PARK_FULL);
    if (!parked) {                                            // next time the slots will be wide enough
        uint32_t want = h[TOT_MAX_T] + h[TOT_MAX_T] / 4;
        want = (want + 63u) & ~63u;
        ctx->park_stride = want > MAX_T ? MAX_T : want;
    }

    if (!fill) return RK_OK;
    if (table->cap_triples < nt || table->cap_segs < ns)
        return rk_fail(ctx, RK_ERR_CAPACITY, "table too small: need %llu triples and %llu segments",
                       (unsigned long long)nt, (unsigned long long)ns);
    if (mirrors) {
        memcpy(table->h_triple_off, h + 16, ((size_t)J + 1) * 4);
        memcpy(table->h_seg_off, h + 16 + J + 1, ((size_t)J + 1) * 4);
    }
    if (J > 0 && !parked) {                                   // the parked keys were incomplete: search again
        k_enumerate<MODE_FILL_SEARCH><<<J, ENUM_THREADS, gmap_bytes, ctx->stream>>>(
            jobs->layers, jobs->gbatch, jobs->mbatch, *bounds, leader, cnt_t, cnt_s, park, park_stride,
            off_t, off_s, table->triples, table->seg_g, table->seg_first, totals, 0, 0);
        RK_CHECK_LAUNCH(ctx, "k_enumerate<fill>");
    }
    return RK_OK;
}
