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

template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_u64(unsigned long long v) {
    const uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    const uint32_t l2 = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, 0xF, 0xF, false);
    const uint32_t h2 = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, 0xF, 0xF, false);
    return ((unsigned long long)h2 << 32) | l2;
}

// Maximum over the wavefront, in every lane; all 64 lanes must be active.
// Within each row of 16 lanes by data-parallel-primitive moves (neighbour,
// neighbour pair, mirrored halves of 8, mirrored halves of 16), then the four
// rows through scalar registers.
__device__ __forceinline__ unsigned long long wave_max_u64_rows(unsigned long long v) {
    unsigned long long o;
    o = dpp_u64<0xB1>(v);  v = o > v ? o : v;                   // quad_perm [1,0,3,2]
    o = dpp_u64<0x4E>(v);  v = o > v ? o : v;                   // quad_perm [2,3,0,1]
    o = dpp_u64<0x141>(v); v = o > v ? o : v;                   // row_half_mirror
    o = dpp_u64<0x140>(v); v = o > v ? o : v;                   // row_mirror
    unsigned long long m = 0;
#pragma unroll
    for (int r = 0; r < 64; r += 16) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, r);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), r);
        const unsigned long long row = ((unsigned long long)hi << 32) | lo;
        m = row > m ? row : m;
    }
    return m;
}

// The minimum likewise.
__device__ __forceinline__ unsigned long long wave_min_u64_rows(unsigned long long v) { return ~wave_max_u64_rows(~v); }

// Lane s of a value whose index is the same in all lanes (through a scalar register).
__device__ __forceinline__ uint32_t wave_lane_u32(uint32_t x, uint32_t s) {
    return (uint32_t)__builtin_amdgcn_readlane((int)x, __builtin_amdgcn_readfirstlane((int)s));
}

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
    if (lanes > 1) key = wave_max_u64_rows(key);
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
    if (lanes > 1) key = wave_max_u64_rows(key);
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

// What job v gives when it steps down in GPUs from (gi, ci): to where the curve's value just below its amount begins
// (the largest amount with a lower throughput, or the smallest with the same one when it holds more than it uses), not
// below its floor.  The curve does not fall along a row, so that place, the first amount whose value reaches the one
// just below, is found by bisection (lanes == 1) or by the 64 lanes of a wavefront looking at 64 amounts at a time
// (all lanes get the result).
template <class Args>
__device__ RsGive rs_down_gpu_at(const Args &A, uint32_t v, int32_t gi, uint32_t ci, uint32_t lane, uint32_t lanes) {
    RsGive gv = {0u, -1, 0.f, 0.f, 0ull, 0ull};
    const int32_t fl = rs_fl_s(A, v);
    if (!rs_part(A, v) || gi < 0 || (fl >= 0 && gi <= fl)) return gv;
    const float V = rs_at(A, A.X.curve_thr, v, ci, gi);
    const float want = rs_at(A, A.X.curve_thr, v, ci, gi - 1);
    int32_t t = -1;
    if (want > 0.f) {
        if (lanes > 1) {
            t = gi - 1;                                    // the amount just below reaches its own value
            for (int32_t base = 0; base < gi - 1; base += 64) {
                const int32_t s = base + (int32_t)lane;
                const bool reaches = s < gi - 1 && rs_at(A, A.X.curve_thr, v, ci, s) >= want;
                const unsigned long long m = __ballot(reaches);
                if (m) { t = base + (int32_t)__ffsll((long long)m) - 1; break; }
            }
        } else {
            int32_t lo = 0, hi = gi - 1;
            while (lo < hi) {
                const int32_t mid = (lo + hi) >> 1;
                if (rs_at(A, A.X.curve_thr, v, ci, mid) >= want) hi = mid; else lo = mid + 1;
            }
            t = lo;
        }
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
__device__ __forceinline__ RsGive rs_down_gpu(const Args &A, uint32_t v, uint32_t lane = 0, uint32_t lanes = 1) {
    return rs_down_gpu_at(A, v, A.st.gi[v], A.st.ci[v], lane, lanes);
}

// ... and when it steps down one CPU level from (gi, ci), not below its floor's level
template <class Args>
__device__ RsGive rs_down_cpu_at(const Args &A, uint32_t v, int32_t gi, uint32_t ci) {
    RsGive gv = {0u, gi, 0.f, 0.f, 0ull, 0ull};
    const uint32_t lowest = rs_fl_s(A, v) >= 0 ? rs_fl_c(A, v) : 0u;
    if (!rs_part(A, v) || gi < 0 || ci == 0 || ci <= lowest) return gv;
    gv.any = 1u;
    gv.loss = (rs_at(A, A.X.best_thr, v, ci, gi) - rs_at(A, A.X.best_thr, v, ci - 1, gi)) / A.X.ref_thr[v];
    gv.dc = rs_c(A, v, ci, gi) - rs_c(A, v, ci - 1, gi);
    gv.slope = gv.loss / (float)gv.dc;
    return gv;
}
template <class Args>
__device__ __forceinline__ RsGive rs_down_cpu(const Args &A, uint32_t v) { return rs_down_cpu_at(A, v, A.st.gi[v], A.st.ci[v]); }

// the cached slopes of job v after its state changed to (gi, ci): what it loses per unit it gives ...
template <class Args>
__device__ __forceinline__ void rs_refresh_give_at(const Args &A, uint32_t v, int32_t gi, uint32_t ci, uint32_t lane, uint32_t lanes) {
    const RsGive a = rs_down_gpu_at(A, v, gi, ci, lane, lanes), b = rs_down_cpu_at(A, v, gi, ci);
    if (lane != 0) return;
    A.ds_g[v] = a.any ? a.slope : __int_as_float(0x7F800000);
    A.ds_c[v] = b.any ? b.slope : __int_as_float(0x7F800000);
}
template <class Args>
__device__ __forceinline__ void rs_refresh_give(const Args &A, uint32_t v) { rs_refresh_give_at(A, v, A.st.gi[v], A.st.ci[v], 0, 1); }
// ... and its own next steps as well; `lanes` threads share the search for them (1, or the 64 of a wavefront).  The
// steps themselves go to next[0] (GPUs) and next[1] (CPUs) when the caller wants them.
template <class Args>
__device__ __forceinline__ void rs_refresh_lanes(const Args &A, uint32_t v, uint32_t lane, uint32_t lanes, RsStep *next = nullptr) {
    const RsGive a = rs_down_gpu(A, v, lane, lanes), b = rs_down_cpu(A, v);
    const RsStep ug = rs_up_gpu(A, v, lane, lanes), uc = rs_up_cpu(A, v, lane, lanes);
    if (lane != 0) return;
    A.ds_g[v] = a.any ? a.slope : __int_as_float(0x7F800000);
    A.ds_c[v] = b.any ? b.slope : __int_as_float(0x7F800000);
    A.ug[v] = ug.any ? ug.slope : 0.f; A.udg[v] = (uint32_t)ug.dg; A.udc_g[v] = ug.dc;
    A.uc[v] = uc.any ? uc.slope : 0.f; A.udc_c[v] = uc.dc;
    if (next) { next[0] = ug; next[1] = uc; }
}
template <class Args>
__device__ __forceinline__ void rs_refresh(const Args &A, uint32_t v) { rs_refresh_lanes(A, v, 0, 1); }

// ---- the same steps for a wavefront that holds the job's rows in its registers
// The searches above follow one load with the next.  A job of at most 64 amounts fits a wavefront, an amount per lane:
// the rows its steps from (gi, ci) read are loaded at once (the curve and the best plans at CPU level ci and at the
// level below, the GPUs of every amount, and, a CPU level per lane, the best plans of amount gi), and every step is
// found from the registers, with the arithmetic of the functions above.
struct RsRows {
    uint32_t ns; float ref; int32_t fl; uint32_t fl_c; bool part;         // the same in all lanes
    float curve, curve_lo, best, best_lo;   // lane s: curve_thr and best_thr of amount s at level ci, and at level ci - 1 (0 without)
    uint32_t g;                             // lane s: GPUs of amount s
    float col;                              // lane c: best_thr of amount gi at level c (0 without)
};
__device__ __forceinline__ float rs_lane_f(float x, int32_t s) { return s < 0 ? 0.f : __uint_as_float(wave_lane_u32(__float_as_uint(x), (uint32_t)s)); }
__device__ __forceinline__ uint32_t rs_lane_u(uint32_t x, int32_t s) { return s < 0 ? 0u : wave_lane_u32(x, (uint32_t)s); }

// (so, ns: where the job's amounts begin in the plan table and how many they are, rs_ns)
template <class Args>
__device__ __forceinline__ RsRows rs_rows(const Args &A, uint32_t v, uint32_t so, uint32_t ns, int32_t gi, uint32_t ci, uint32_t lane) {
    RsRows R = {};
    const uint32_t n_mem = A.X.grid.n_mem, n_cpu = A.X.grid.n_cpu;
    R.ns = ns;
    R.ref = A.X.ref_thr[v];
    R.fl = rs_fl_s(A, v); R.fl_c = rs_fl_c(A, v); R.part = rs_part(A, v);
    const uint64_t job = (uint64_t)n_cpu * n_mem * so + (uint64_t)(n_mem - 1) * R.ns;    // level 0, top tier, amount 0
    const uint64_t level = (uint64_t)n_mem * R.ns;
    if (lane < R.ns) {
        R.curve = A.X.curve_thr[job + ci * level + lane];
        R.best = A.X.best_thr[job + ci * level + lane];
        if (ci > 0) {
            R.curve_lo = A.X.curve_thr[job + (ci - 1) * level + lane];
            R.best_lo = A.X.best_thr[job + (ci - 1) * level + lane];
        }
        R.g = A.X.tb.seg_g[so + lane];
    }
    if (gi >= 0 && lane < n_cpu) R.col = A.X.best_thr[job + lane * level + (uint32_t)gi];
    return R;
}

// rs_down_gpu_at on the row `curve` (lane s: the curve of amount s at level ci)
template <class Args>
__device__ __forceinline__ RsGive rs_down_gpu_rows(const Args &A, const RsRows &R, float curve, int32_t gi, uint32_t ci, uint32_t lane) {
    RsGive gv = {0u, -1, 0.f, 0.f, 0ull, 0ull};
    if (!R.part || gi < 0 || (R.fl >= 0 && gi <= R.fl)) return gv;
    const float V = rs_lane_f(curve, gi), want = rs_lane_f(curve, gi - 1);
    int32_t t = -1;
    if (want > 0.f) {
        const unsigned long long m = __ballot((int32_t)lane < gi - 1 && curve >= want);
        t = m ? (int32_t)__ffsll((long long)m) - 1 : gi - 1;
    }
    if (R.fl >= 0 && t < R.fl) t = R.fl;
    const uint32_t g_gi = rs_lane_u(R.g, gi), g_t = rs_lane_u(R.g, t);
    gv.any = 1u; gv.tgt = t;
    gv.loss = (V - rs_lane_f(curve, t)) / R.ref;
    gv.dg = (unsigned long long)g_gi - g_t;
    gv.dc = cpu_cost(A.X.grid, ci, g_gi) - (t < 0 ? 0ull : cpu_cost(A.X.grid, ci, g_t));
    gv.slope = gv.loss / (float)gv.dg;
    return gv;
}
// rs_down_cpu_at; hi and lo are the best plans' values of amount gi at levels ci and ci - 1
template <class Args>
__device__ __forceinline__ RsGive rs_down_cpu_rows(const Args &A, const RsRows &R, int32_t gi, uint32_t ci, float hi, float lo) {
    RsGive gv = {0u, gi, 0.f, 0.f, 0ull, 0ull};
    const uint32_t lowest = R.fl >= 0 ? R.fl_c : 0u;
    if (!R.part || gi < 0 || ci == 0 || ci <= lowest) return gv;
    const uint32_t g = rs_lane_u(R.g, gi);
    gv.any = 1u;
    gv.loss = (hi - lo) / R.ref;
    gv.dc = cpu_cost(A.X.grid, ci, g) - cpu_cost(A.X.grid, ci - 1, g);
    gv.slope = gv.loss / (float)gv.dc;
    return gv;
}
// rs_up_gpu for a job that is not below its floor
template <class Args>
__device__ __forceinline__ RsStep rs_up_gpu_rows(const Args &A, const RsRows &R, int32_t gi, uint32_t ci, uint32_t lane) {
    RsStep st = {0u, -1, ci, 0.f, 0.f, 0ull, 0ull};
    const float cur = rs_lane_f(R.curve, gi);
    const uint32_t g_cur = rs_lane_u(R.g, gi);
    unsigned long long key = 0;
    if ((int32_t)lane > gi && lane < R.ns && (unsigned long long)R.g <= A.G && R.curve > cur) {   // amounts ascend in GPUs
        const float sl = ((R.curve - cur) / R.ref) / (float)((unsigned long long)R.g - g_cur);
        if (sl > 0.f) key = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - lane);
    }
    key = wave_max_u64_rows(key);
    if (key) {
        const int32_t s = (int32_t)(0xFFFFFFFFu - (uint32_t)key);
        const uint32_t g_s = rs_lane_u(R.g, s);
        st.any = 1u; st.tgt = s;
        st.dg = (unsigned long long)g_s - g_cur;
        st.dc = cpu_cost(A.X.grid, ci, g_s) - (gi < 0 ? 0ull : cpu_cost(A.X.grid, ci, g_cur));
        st.gain = (rs_lane_f(R.curve, s) - cur) / R.ref;
        st.slope = st.gain / (float)st.dg;
    }
    return st;
}
// rs_up_cpu
template <class Args>
__device__ __forceinline__ RsStep rs_up_cpu_rows(const Args &A, const RsRows &R, int32_t gi, uint32_t ci, uint32_t lane) {
    RsStep st = {0u, gi, ci, 0.f, 0.f, 0ull, 0ull};
    if (gi < 0) return st;
    const float cur = rs_lane_f(R.best, gi);
    const uint32_t g = rs_lane_u(R.g, gi);
    const unsigned long long here = cpu_cost(A.X.grid, ci, g);
    unsigned long long key = 0;
    if (lane > ci && lane < A.X.grid.n_cpu && R.col > cur) {
        const float sl = ((R.col - cur) / R.ref) / (float)(cpu_cost(A.X.grid, lane, g) - here);
        if (sl > 0.f) key = ((unsigned long long)__float_as_uint(sl) << 32) | (0xFFFFFFFFu - lane);
    }
    key = wave_max_u64_rows(key);
    if (key) {
        const uint32_t c = 0xFFFFFFFFu - (uint32_t)key;
        st.any = 1u; st.lvl = c;
        st.dc = cpu_cost(A.X.grid, c, g) - here;
        st.gain = (rs_lane_f(R.col, (int32_t)c) - cur) / R.ref;
        st.slope = st.gain / (float)st.dc;
    }
    return st;
}

// Job v, which holds (gi, ci), steps down in GPUs (res 0) or one CPU level (res 1): what it gives, what it holds then,
// and what it would lose per GPU / CPU given after that (infinite: nothing to give).  A whole wavefront calls; every
// lane gets the result.
struct RsShrunk { RsGive gv; int32_t gi; uint32_t ci; float ds_g, ds_c; };
template <class Args>
__device__ __forceinline__ RsShrunk rs_shrink_wave(const Args &A, uint32_t v, uint32_t so, uint32_t ns, uint32_t res, int32_t gi, uint32_t ci,
                                                   uint32_t lane) {
    RsShrunk out;
    RsGive a, b;
    if (ns > 64u) {
        out.gv = res == 0 ? rs_down_gpu_at(A, v, gi, ci, lane, 64) : rs_down_cpu_at(A, v, gi, ci);
        out.gi = res == 0 ? out.gv.tgt : gi;
        out.ci = res == 0 ? (out.gv.tgt < 0 ? 0u : ci) : ci - 1u;
        a = rs_down_gpu_at(A, v, out.gi, out.ci, lane, 64);
        b = rs_down_cpu_at(A, v, out.gi, out.ci);
    } else {
        const RsRows R = rs_rows(A, v, so, ns, gi, ci, lane);
        if (res == 0) {
            out.gv = rs_down_gpu_rows(A, R, R.curve, gi, ci, lane);
            out.gi = out.gv.tgt;
            out.ci = out.gv.tgt < 0 ? 0u : ci;                      // (with nothing left, every step down is none)
            a = rs_down_gpu_rows(A, R, R.curve, out.gi, ci, lane);
            b = rs_down_cpu_rows(A, R, out.gi, out.ci, rs_lane_f(R.best, out.gi), rs_lane_f(R.best_lo, out.gi));
        } else {
            out.gv = rs_down_cpu_rows(A, R, gi, ci, rs_lane_f(R.best, gi), rs_lane_f(R.best_lo, gi));
            out.gi = gi;
            out.ci = ci - 1u;
            a = rs_down_gpu_rows(A, R, R.curve_lo, gi, out.ci, lane);
            b = rs_down_cpu_rows(A, R, gi, out.ci, rs_lane_f(R.col, (int32_t)out.ci), rs_lane_f(R.col, (int32_t)out.ci - 1));
        }
    }
    out.ds_g = a.any ? a.slope : __int_as_float(0x7F800000);
    out.ds_c = b.any ? b.slope : __int_as_float(0x7F800000);
    return out;
}

// rs_refresh_lanes for a whole wavefront; with keep_next the next steps also go to next[0] (GPUs) and next[1] (CPUs),
// and whether the job is below its floor to *next_below
template <class Args>
__device__ __forceinline__ void rs_refresh_wave(const Args &A, uint32_t v, uint32_t lane, RsStep *next, uint32_t *next_below, bool keep_next) {
    const int32_t gi = A.st.gi[v];
    const uint32_t ci = A.st.ci[v];
    const int32_t fl = rs_fl_s(A, v);
    const uint32_t so = A.X.tb.seg_off[v], ns = A.X.tb.seg_off[v + 1] - so;
    if (ns > 64u || (fl >= 0 && gi < fl)) {
        RsStep up[2];
        rs_refresh_lanes(A, v, lane, 64, up);
        if (lane == 0 && keep_next) { next[0] = up[0]; next[1] = up[1]; *next_below = (fl >= 0 && gi < fl) ? 1u : 0u; }
        return;
    }
    const RsRows R = rs_rows(A, v, so, ns, gi, ci, lane);
    const RsGive a = rs_down_gpu_rows(A, R, R.curve, gi, ci, lane);
    const RsGive b = rs_down_cpu_rows(A, R, gi, ci, rs_lane_f(R.best, gi), rs_lane_f(R.best_lo, gi));
    const RsStep ug = rs_up_gpu_rows(A, R, gi, ci, lane), uc = rs_up_cpu_rows(A, R, gi, ci, lane);
    if (lane != 0) return;
    A.ds_g[v] = a.any ? a.slope : __int_as_float(0x7F800000);
    A.ds_c[v] = b.any ? b.slope : __int_as_float(0x7F800000);
    A.ug[v] = ug.any ? ug.slope : 0.f; A.udg[v] = (uint32_t)ug.dg; A.udc_g[v] = ug.dc;
    A.uc[v] = uc.any ? uc.slope : 0.f; A.udc_c[v] = uc.dc;
    if (keep_next) { next[0] = ug; next[1] = uc; *next_below = 0u; }
}

// A workgroup barrier that orders LDS traffic only: every wavefront waits for its own LDS operations, not for its
// global loads and stores, which __syncthreads() would also drain.  Enough where what is exchanged is in LDS.
__device__ __forceinline__ void rs_lds_barrier() {
    asm volatile("" ::: "memory");               // the compiler keeps memory accesses on their side of the barrier
    __builtin_amdgcn_s_waitcnt(0xC07F);          // vmcnt 63, expcnt 7, lgkmcnt 0
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// A float as an unsigned word that orders the same way (-0 as +0), and back.
__device__ __forceinline__ uint32_t rs_ordered(float x) {
    const uint32_t b = __float_as_uint(x + 0.f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float rs_unordered(uint32_t u) { return __uint_as_float((u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u); }

// Minimum of a word over the wavefront, in every lane; all 64 lanes must be active (as wave_max_u64_rows).
template <int CTRL>
__device__ __forceinline__ uint32_t rs_dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_min_u32_rows(uint32_t v) {
    uint32_t o;
    o = rs_dpp_u32<0xB1>(v);  v = o < v ? o : v;                // quad_perm [1,0,3,2]
    o = rs_dpp_u32<0x4E>(v);  v = o < v ? o : v;                // quad_perm [2,3,0,1]
    o = rs_dpp_u32<0x141>(v); v = o < v ? o : v;                // row_half_mirror
    o = rs_dpp_u32<0x140>(v); v = o < v ? o : v;                // row_mirror
    uint32_t m = 0xFFFFFFFFu;
#pragma unroll
    for (int r = 0; r < 64; r += 16) {
        const uint32_t row = (uint32_t)__builtin_amdgcn_readlane((int)v, r);
        m = row < m ? row : m;
    }
    return m;
}

// The job that comes first in the loops' order (GPU slope, then CPU slope, both descending, then the lower index)
// among the candidates of a workgroup's threads (j == 0xFFFFFFFF: a thread without one; slopes are not negative).
// All threads call and all get the result.  The slopes travel as one key of two words that order like them, the
// wavefronts reduce by DPP, the first one reduces their results; sh_key and sh_j hold WAVES + 1 entries.
struct RsPick { float g, c; uint32_t j; };
template <int WAVES>
__device__ __forceinline__ RsPick rs_pick_first(float g, float c, uint32_t j, uint32_t lane, uint32_t wave,
                                                unsigned long long *sh_key, uint32_t *sh_j) {
    const uint32_t NONE = 0xFFFFFFFFu;
    const unsigned long long key = j == NONE ? 0ull : ((unsigned long long)rs_ordered(g) << 32) | rs_ordered(c);
    const unsigned long long top = wave_max_u64_rows(key);
    const uint32_t first = wave_min_u32_rows(j != NONE && key == top ? j : NONE);
    if (lane == 0) { sh_key[wave] = top; sh_j[wave] = first; }
    rs_lds_barrier();
    if (wave == 0) {
        const unsigned long long k2 = lane < WAVES ? sh_key[lane] : 0ull;
        const uint32_t j2 = lane < WAVES ? sh_j[lane] : NONE;
        const unsigned long long t2 = wave_max_u64_rows(k2);
        const uint32_t f2 = wave_min_u32_rows(j2 != NONE && k2 == t2 ? j2 : NONE);
        if (lane == 0) { sh_key[WAVES] = t2; sh_j[WAVES] = f2; }
    }
    rs_lds_barrier();
    RsPick out;
    const unsigned long long t = sh_key[WAVES];
    out.j = sh_j[WAVES];
    out.g = rs_unordered((uint32_t)(t >> 32));
    out.c = rs_unordered((uint32_t)t);
    return out;
}

// The two lowest give-slopes over all jobs, per resource, and the job of the lowest (the lower index among equal
// values; none: 0xFFFFFFFF with both values infinite).  ds holds the slopes [2][n_jobs] (LDS).  All THREADS threads of
// the workgroup call and all get the result in out[0] (GPUs) and out[1] (CPUs).  Every thread keeps the two lowest
// of its own jobs; the lowest goes through a DPP minimum of packed keys (slope as a word that orders like it, job),
// the second lowest is the minimum of what the threads hold once the lowest's owner puts its own second in.
// sh_k and sh_s hold 2 * (WAVES + 1) entries each.
struct RsMin { float m1, m2; uint32_t i1; };
template <int WAVES, int THREADS>
__device__ __forceinline__ void rs_two_lowest(const float *ds, uint32_t n_jobs, uint32_t tid, uint32_t lane, uint32_t wave,
                                              unsigned long long *sh_k, uint32_t *sh_s, RsMin (&out)[2]) {
    const float INF = __int_as_float(0x7F800000);
    const uint32_t NONE = 0xFFFFFFFFu;
    float a[2] = {INF, INF}, b[2] = {INF, INF};
    uint32_t ia[2] = {NONE, NONE};
    for (uint32_t v0 = tid; v0 < n_jobs; v0 += 4 * THREADS) {            // four loads per resource in flight
        float x[2][4];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t v = v0 + k * THREADS;
            x[0][k] = v < n_jobs ? ds[v] : INF;
            x[1][k] = v < n_jobs ? ds[n_jobs + v] : INF;
        }
#pragma unroll
        for (uint32_t r = 0; r < 2; ++r)
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {                           // ascending jobs: the lower one stays among equals
                const float y = x[r][k];
                if (y < a[r]) { b[r] = a[r]; a[r] = y; ia[r] = v0 + k * THREADS; }
                else if (y < b[r]) b[r] = y;
            }
    }
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r) {
        const unsigned long long key = ia[r] == NONE ? ~0ull : ((unsigned long long)rs_ordered(a[r]) << 32) | ia[r];
        const unsigned long long w = wave_min_u64_rows(key);
        if (lane == 0) sh_k[r * (WAVES + 1) + wave] = w;
    }
    rs_lds_barrier();
    if (wave == 0) {
#pragma unroll
        for (uint32_t r = 0; r < 2; ++r) {
            const unsigned long long w = wave_min_u64_rows(lane < WAVES ? sh_k[r * (WAVES + 1) + lane] : ~0ull);
            if (lane == 0) sh_k[r * (WAVES + 1) + WAVES] = w;
        }
    }
    rs_lds_barrier();
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r) {
        const unsigned long long low = sh_k[r * (WAVES + 1) + WAVES];
        out[r].i1 = low == ~0ull ? NONE : (uint32_t)low;
        out[r].m1 = low == ~0ull ? INF : rs_unordered((uint32_t)(low >> 32));
        // what this thread holds beside the lowest: its own lowest, or its second when the lowest is its own
        const float mine = (ia[r] != NONE && ia[r] == out[r].i1) ? b[r] : a[r];
        const uint32_t w = wave_min_u32_rows(rs_ordered(mine));
        if (lane == 0) sh_s[r * (WAVES + 1) + wave] = w;
    }
    rs_lds_barrier();
    if (wave == 0) {
#pragma unroll
        for (uint32_t r = 0; r < 2; ++r) {
            const uint32_t w = wave_min_u32_rows(lane < WAVES ? sh_s[r * (WAVES + 1) + lane] : rs_ordered(INF));
            if (lane == 0) sh_s[r * (WAVES + 1) + WAVES] = w;
        }
    }
    rs_lds_barrier();
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r) out[r].m2 = rs_unordered(sh_s[r * (WAVES + 1) + WAVES]);
}
