// What Algorithm 1's Schedule loop asks of a job's curves (paper Sec. 5.2, the paragraphs on slopes and on shrinking):
// a job's next step up in GPUs and in CPU levels, and what it gives when it steps down.  Shared by the loop over
// the cluster's totals and the loop over its nodes; `Args` is the kernel's argument struct with
//   X.tb, X.grid, X.ref_thr, X.best_thr, X.curve_thr   plan table, grid and the curves (segment layout, all jobs)
//   st.gi, st.ci                                       what every job holds: index of its GPU count (-1: nothing), CPU level
//   G                                                  GPUs of the cluster (no step goes beyond)
//   state, floor_seg, floor_c                          per job, each may be null
//   ds_g, ds_c, ug, udg, udc_g, uc, udc_c              per job, for the cached values (rs_refresh*)
#pragma once
#include "rk_internal.h"
#include "rk_model.h"

__device__ __forceinline__ unsigned long long cpu_cost(const GridDev &G, uint32_t ci, uint32_t g) {
    return G.cpu_mode ? (unsigned long long)G.cpu_levels[ci] * g : (unsigned long long)G.cpu_levels[ci];
}

struct RsStep { uint32_t any; int32_t tgt; uint32_t lvl; float slope, gain; unsigned long long dg, dc; };
struct RsGive { uint32_t any; int32_t tgt; float loss, slope; unsigned long long dg, dc; };

template <class Args>
__device__ __forceinline__ uint32_t rs_ns(const Args &A, uint32_t j) { return A.X.tb.seg_off[j + 1] - A.X.tb.seg_off[j]; }
template <class Args>
__device__ __forceinline__ unsigned long long rs_g(const Args &A, uint32_t j, int32_t s) {
    return s < 0 ? 0ull : A.X.tb.seg_g[A.X.tb.seg_off[j] + (uint32_t)s];
}
template <class Args>
__device__ __forceinline__ unsigned long long rs_c(const Args &A, uint32_t j, uint32_t c, int32_t s) {
    return s < 0 ? 0ull : cpu_cost(A.X.grid, c, (uint32_t)rs_g(A, j, s));
}
// value of job j at CPU level c, top memory tier, segment s (0 below the first segment)
template <class Args>
__device__ __forceinline__ float rs_at(const Args &A, const float *arr, uint32_t j, uint32_t c, int32_t s) {
    if (s < 0) return 0.f;
    const uint32_t n_mem = A.X.grid.n_mem, ns = rs_ns(A, j);
    return arr[(uint64_t)A.X.grid.n_cpu * n_mem * A.X.tb.seg_off[j] + ((uint64_t)c * n_mem + (n_mem - 1)) * ns + (uint32_t)s];
}
template <class Args>
__device__ __forceinline__ bool rs_part(const Args &A, uint32_t j) { return !A.state || A.state[j] == 0; }
// state 2: the job keeps exactly what it holds (it takes no step and gives nothing); any other non-zero state: it takes
// no part and holds nothing
template <class Args>
__device__ __forceinline__ bool rs_holds(const Args &A, uint32_t j) { return !A.state || A.state[j] == 0 || A.state[j] == 2; }
// the job's floor: segment (-1: none; a segment the job does not have counts as none) and CPU level (clamped)
template <class Args>
__device__ __forceinline__ int32_t rs_fl_s(const Args &A, uint32_t j) {
    if (!A.floor_seg) return -1;
    const int32_t f = A.floor_seg[j];
    return (f >= 0 && (uint32_t)f < rs_ns(A, j)) ? f : -1;
}
template <class Args>
__device__ __forceinline__ uint32_t rs_fl_c(const Args &A, uint32_t j) {
    if (rs_fl_s(A, j) < 0 || !A.floor_c) return 0u;
    const uint32_t c = A.floor_c[j];
    return c < A.X.grid.n_cpu ? c : A.X.grid.n_cpu - 1u;
}

// Next GPU step of job j.  `lanes` threads share the candidates (1: the calling thread alone; 64: a wavefront, all
// lanes get the result).  Highest slope, the smaller amount among equal slopes.
template <class Args>
__device__ RsStep rs_up_gpu(const Args &A, uint32_t j, uint32_t lane, uint32_t lanes) {
    RsStep st = {0u, -1, A.st.ci[j], 0.f, 0.f, 0ull, 0ull};
    const int32_t gi = A.st.gi[j];
    const uint32_t ci = A.st.ci[j];
    const float ref = A.X.ref_thr[j];
    const float cur = rs_at(A, A.X.curve_thr, j, ci, gi);
    const int32_t fl = rs_fl_s(A, j);
    if (fl >= 0 && gi < fl) {
        const uint32_t lvl = ci > rs_fl_c(A, j) ? ci : rs_fl_c(A, j);
        const float v = rs_at(A, A.X.curve_thr, j, lvl, fl);
        st.any = 1u; st.tgt = fl; st.lvl = lvl;
        st.dg = rs_g(A, j, fl) - rs_g(A, j, gi);
        st.dc = rs_c(A, j, lvl, fl) - rs_c(A, j, ci, gi);
        st.gain = (v - cur) / ref;
        st.slope = st.gain / (float)st.dg;
        return st;
    }
    const int32_t ns = (int32_t)rs_ns(A, j);
    unsigned long long key = 0;                            // slope bits, then the inverted segment index
    for (int32_t s = gi + 1 + (int32_t)lane; s < ns; s += (int32_t)lanes) {
        if (rs_g(A, j, s) > A.G) break;
        const float v = rs_at(A, A.X.curve_thr, j, ci, s);
        if (!(v > cur)) continue;
        const unsigned long long dg = rs_g(A, j, s) - rs_g(A, j, gi);
        const float gain = (v - cur) / ref;
        const float sl = gain / (float)dg;
        if (!(sl > 0.f)) continue;
        const unsigned long long k = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - (uint32_t)s);
        key = k > key ? k : key;
    }
    if (lanes > 1) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const unsigned long long o = __shfl_xor(key, off, 64);
            key = o > key ? o : key;
        }
    }
    if (key) {
        const int32_t s = (int32_t)(0xFFFFFFFFu - (uint32_t)key);
        const float v = rs_at(A, A.X.curve_thr, j, ci, s);
        st.any = 1u; st.tgt = s;
        st.dg = rs_g(A, j, s) - rs_g(A, j, gi);
        st.dc = rs_c(A, j, ci, s) - rs_c(A, j, ci, gi);
        st.gain = (v - cur) / ref;
        st.slope = st.gain / (float)st.dg;
    }
    return st;
}

template <class Args>
__device__ RsStep rs_up_cpu(const Args &A, uint32_t j, uint32_t lane, uint32_t lanes) {
    const int32_t gi = A.st.gi[j];
    const uint32_t ci = A.st.ci[j];
    RsStep st = {0u, gi, ci, 0.f, 0.f, 0ull, 0ull};
    if (gi < 0) return st;
    const float ref = A.X.ref_thr[j];
    const float cur = rs_at(A, A.X.best_thr, j, ci, gi);
    unsigned long long key = 0;
    for (uint32_t c = ci + 1 + lane; c < A.X.grid.n_cpu; c += lanes) {
        const float v = rs_at(A, A.X.best_thr, j, c, gi);
        if (!(v > cur)) continue;
        const unsigned long long dc = rs_c(A, j, c, gi) - rs_c(A, j, ci, gi);
        const float gain = (v - cur) / ref;
        const float sl = gain / (float)dc;
        if (!(sl > 0.f)) continue;
        const unsigned long long k = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - c);
        key = k > key ? k : key;
    }
    if (lanes > 1) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const unsigned long long o = __shfl_xor(key, off, 64);
            key = o > key ? o : key;
        }
    }
    if (key) {
        const uint32_t c = 0xFFFFFFFFu - (uint32_t)key;
        const float v = rs_at(A, A.X.best_thr, j, c, gi);
        st.any = 1u; st.lvl = c;
        st.dc = rs_c(A, j, c, gi) - rs_c(A, j, ci, gi);
        st.gain = (v - cur) / ref;
        st.slope = st.gain / (float)st.dc;
    }
    return st;
}

// What job v gives when it steps down in GPUs: to where the curve's value just below its amount begins (the largest
// amount with a lower throughput, or the smallest with the same one when it holds more than it uses), not below
// its floor.  The curve does not fall along a row, so that place is found by bisection.
template <class Args>
__device__ RsGive rs_down_gpu(const Args &A, uint32_t v) {
    RsGive gv = {0u, -1, 0.f, 0.f, 0ull, 0ull};
    const int32_t gi = A.st.gi[v];
    const int32_t fl = rs_fl_s(A, v);
    if (!rs_part(A, v) || gi < 0 || (fl >= 0 && gi <= fl)) return gv;
    const uint32_t ci = A.st.ci[v];
    const float V = rs_at(A, A.X.curve_thr, v, ci, gi);
    const float want = rs_at(A, A.X.curve_thr, v, ci, gi - 1);
    int32_t t = -1;
    if (want > 0.f) {
        int32_t lo = 0, hi = gi - 1;                       // first segment whose value reaches `want`
        while (lo < hi) {
            const int32_t mid = (lo + hi) >> 1;
            if (rs_at(A, A.X.curve_thr, v, ci, mid) >= want) hi = mid; else lo = mid + 1;
        }
        t = lo;
    }
    if (fl >= 0 && t < fl) t = fl;
    gv.any = 1u; gv.tgt = t;
    gv.loss = (V - rs_at(A, A.X.curve_thr, v, ci, t)) / A.X.ref_thr[v];
    gv.dg = rs_g(A, v, gi) - rs_g(A, v, t);
    gv.dc = rs_c(A, v, ci, gi) - rs_c(A, v, ci, t);
    gv.slope = gv.loss / (float)gv.dg;
    return gv;
}

template <class Args>
__device__ RsGive rs_down_cpu(const Args &A, uint32_t v) {
    const int32_t gi = A.st.gi[v];
    RsGive gv = {0u, gi, 0.f, 0.f, 0ull, 0ull};
    const uint32_t ci = A.st.ci[v];
    const uint32_t lowest = rs_fl_s(A, v) >= 0 ? rs_fl_c(A, v) : 0u;
    if (!rs_part(A, v) || gi < 0 || ci == 0 || ci <= lowest) return gv;
    gv.any = 1u;
    gv.loss = (rs_at(A, A.X.best_thr, v, ci, gi) - rs_at(A, A.X.best_thr, v, ci - 1, gi)) / A.X.ref_thr[v];
    gv.dc = rs_c(A, v, ci, gi) - rs_c(A, v, ci - 1, gi);
    gv.slope = gv.loss / (float)gv.dc;
    return gv;
}

// the cached slopes of job v after its state changed: what it loses per unit it gives ...
template <class Args>
__device__ __forceinline__ void rs_refresh_give(const Args &A, uint32_t v) {
    const RsGive a = rs_down_gpu(A, v), b = rs_down_cpu(A, v);
    A.ds_g[v] = a.any ? a.slope : __int_as_float(0x7F800000);
    A.ds_c[v] = b.any ? b.slope : __int_as_float(0x7F800000);
}
// ... and its own next steps as well; `lanes` threads share the search for them (1, or the 64 of a wavefront)
template <class Args>
__device__ __forceinline__ void rs_refresh_lanes(const Args &A, uint32_t v, uint32_t lane, uint32_t lanes) {
    const RsGive a = rs_down_gpu(A, v), b = rs_down_cpu(A, v);
    const RsStep ug = rs_up_gpu(A, v, lane, lanes), uc = rs_up_cpu(A, v, lane, lanes);
    if (lane != 0) return;
    A.ds_g[v] = a.any ? a.slope : __int_as_float(0x7F800000);
    A.ds_c[v] = b.any ? b.slope : __int_as_float(0x7F800000);
    A.ug[v] = ug.any ? ug.slope : 0.f; A.udg[v] = (uint32_t)ug.dg; A.udc_g[v] = ug.dc;
    A.uc[v] = uc.any ? uc.slope : 0.f; A.udc_c[v] = uc.dc;
}
template <class Args>
__device__ __forceinline__ void rs_refresh(const Args &A, uint32_t v) { rs_refresh_lanes(A, v, 0, 1); }

// the two lowest values of ds over all jobs and the job of the lowest (lower index among equal values)
struct RsMin { float m1, m2; uint32_t i1; };
__device__ __forceinline__ RsMin rs_min_merge(const RsMin &a, const RsMin &b) {
    RsMin r;
    const bool a_first = a.m1 < b.m1 || (a.m1 == b.m1 && a.i1 <= b.i1);
    const RsMin &lo = a_first ? a : b, &hi = a_first ? b : a;
    r.m1 = lo.m1; r.i1 = lo.i1;
    r.m2 = lo.m2 < hi.m1 ? lo.m2 : hi.m1;
    return r;
}
