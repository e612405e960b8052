/*
 * CPU oracle (test infrastructure, see rk_oracle.h).  Written from the
 * paper's Sec. 4 (performance model) and Sec. 5.2 (resource sensitivity
 * curves, best-plan search, slope-ordered greedy).  Every function states the
 * passage it follows and how it is pinned by the CPU test-suite.
 *
 * Build: g++ -O2 -std=c++17 -ffp-contract=off -fPIC -shared -pthread
 */
#include "rk_oracle.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <map>
#include <set>
#include <vector>

namespace {

enum { P_BYTES, SEQ, HIDDEN, ELEM_BYTES, T_FWD_SAMPLE, K_BWD, K_SYNC, K_OPT, K_OPT_OFF,
       K_OFF, K_SWAP, K_CONST, MEM_STATE, MEM_ACT, MEM_ACT_GC, MEM_CONST, REF_THR, N_COEF };
enum { LAYERS, GBATCH, MBATCH, N_INT };

/* order of the terms[] array returned by ork_eval_one */
enum { X_N, X_M, X_A, X_TF_MB, X_T_FWD, X_T_BWD, X_V_DP, X_V_TP, X_V_PP, X_T_DP, X_T_TP,
       X_T_PP, X_T_CC, X_PSI, X_T_OPT, X_T_OFF, X_T_OO, X_T_ITER, X_THR, X_M_GPU, X_H_HOST,
       X_B_DP, X_B_TP, X_B_PP };

const float GIB = 1073741824.0f;

/* Structural validity of a plan on top of the (d,t,p) partitioning rules:
 * the option must be allowed by the bounds, and offloading needs partitioned
 * gradients (Sec. 4.2 "Modeling T_off": ZeRO-Offload moves *partitioned*
 * gradients), i.e. ZeRO stage >= 2. */
bool option_valid(const ork_bounds *b, uint32_t z, uint32_t gc, uint32_t off) {
    if (!((b->zero_mask >> z) & 1u)) return false;
    if (!((b->gc_mask >> gc) & 1u)) return false;
    if (!((b->off_mask >> off) & 1u)) return false;
    if (off && z < 2) return false;
    return true;
}

/* Bottleneck-bandwidth rule of Sec. 4.1 "Modeling T_comm" under a packed
 * placement with tensor-parallel ranks adjacent, then data-parallel, then
 * pipeline stages.  A job inside one node uses the intra-node links for
 * everything.  A job over several nodes keeps a communication group on the
 * intra-node links only when whole groups tile a node. */
void bandwidths(const ork_env *env, uint32_t d, uint32_t t, uint32_t p,
                double *B_dp, double *B_tp, double *B_pp) {
    const uint32_t N = env->gpus_per_node;
    const uint64_t g = (uint64_t)d * t * p;
    const double bi = env->B_intra, bx = env->B_inter;
    if (g <= N) { *B_dp = bi; *B_tp = bi; *B_pp = bi; return; }
    *B_tp = (N % t == 0) ? bi : bx;
    *B_dp = (N % ((uint64_t)t * d) == 0) ? bi : bx;
    *B_pp = bx;
}

/* The same rule for a job whose GPUs are known: parts[i] GPUs on the i-th node
 * of its placement, in placement order.  Ranks are laid over these GPU slots
 * with tensor-parallel ranks adjacent, then data-parallel, then pipeline
 * stages.  A communication group uses the intra-node links only if all its
 * ranks landed on one node (Sec. 4.1: the bottleneck bandwidth decides), which
 * for groups of w adjacent-block ranks means that every node boundary inside
 * the job falls on a multiple of w: w = t for tensor parallelism, w = t*d for
 * data parallelism (its groups interleave over a whole pipeline stage);
 * pipeline neighbours share a node only when the whole job does. */
void bandwidths_placed(const ork_env *env, uint32_t d, uint32_t t, uint32_t p, uint32_t n_parts,
                       const uint32_t *parts, double *B_dp, double *B_tp, double *B_pp) {
    const double bi = env->B_intra, bx = env->B_inter;
    bool tp_in = true, dp_in = true;
    uint64_t edge = 0;
    for (uint32_t i = 0; i + 1 < n_parts; ++i) {          /* the boundaries between consecutive parts */
        edge += parts[i];
        if (edge % t != 0) tp_in = false;
        if (edge % ((uint64_t)t * d) != 0) dp_in = false;
    }
    *B_tp = tp_in ? bi : bx;
    *B_dp = dp_in ? bi : bx;
    *B_pp = (n_parts <= 1) ? bi : bx;
}

/* GPU and host memory of a plan, float32, one rounding per operation, in
 * exactly this order.  The paper leaves the estimate to the training
 * frameworks (Sec. 6); this is the mixed-precision Adam accounting of the
 * ZeRO paper it cites: 16 bytes of state per 2-byte parameter, partitioned
 * by stage, plus activations and a constant.
 *   Psi   = P_bytes / (t*p)
 *   kappa = 8 | 2+6/d | 1+7/d | 8/d   for ZeRO 0..3 without offload
 *           1 | 1/d                   for ZeRO 2,3 with offload
 *   S     = (mem_state*kappa)*Psi
 *   tok   = (mu*seq)*hidden ; lay = layers/p ; w = min(p, b/(d*mu))
 *   base  = ((tok*lay)/t)*w
 *   A     = mem_act*base                              without checkpointing
 *           mem_act_gc*base + (mem_act*tok)/t         with checkpointing
 *   M_gpu = (S + A) + mem_const
 *   H_host= ((mem_state*(7/d))*Psi)*g  with offload, else 0
 */
void memory_f32(const float *cf, const uint32_t *in, uint32_t d, uint32_t t, uint32_t p,
                uint32_t z, uint32_t gc, uint32_t off, float *M_gpu, float *H_host) {
    const float fd = (float)d, ft = (float)t;
    const float tp = (float)(t * p);
    const float Psi = cf[P_BYTES] / tp;
    float kappa;
    if (off) {
        kappa = (z == 2) ? 1.0f : 1.0f / fd;
    } else if (z == 0) {
        kappa = 8.0f;
    } else if (z == 1) {
        float q = 6.0f / fd; kappa = 2.0f + q;
    } else if (z == 2) {
        float q = 7.0f / fd; kappa = 1.0f + q;
    } else {
        kappa = 8.0f / fd;
    }
    float sk = cf[MEM_STATE] * kappa;
    const float S = sk * Psi;
    const uint32_t mu = in[MBATCH];
    const uint32_t n = in[GBATCH] / (d * mu);
    const uint32_t w = (p < n) ? p : n;
    float tok = (float)mu * cf[SEQ];
    tok = tok * cf[HIDDEN];
    const float lay = (float)(in[LAYERS] / p);
    float base = tok * lay;
    base = base / ft;
    base = base * (float)w;
    float A;
    if (gc) {
        float a1 = cf[MEM_ACT_GC] * base;
        float a2 = cf[MEM_ACT] * tok;
        a2 = a2 / ft;
        A = a1 + a2;
    } else {
        A = cf[MEM_ACT] * base;
    }
    float M = S + A;
    M = M + cf[MEM_CONST];
    *M_gpu = M;
    if (off) {
        float q = 7.0f / fd;
        float h = cf[MEM_STATE] * q;
        h = h * Psi;
        h = h * (float)(d * t * p);
        *H_host = h;
    } else {
        *H_host = 0.0f;
    }
}

/* Sec. 4, Eq. (1) and the paragraphs before it, for one candidate.
 * Pinned by tests/test_oracle_model.py: hand-computed sums with all overlap
 * exponents 1, the single-GPU closed form, volume special cases, V = 0 at
 * size 1, monotonicity in c for offload plans. */
/* th = the seven fittable parameters of Table 1 in double, in the order
 * k_bwd, k_sync, k_opt, k_opt_off, k_off, k_swap, k_const (the model fitting
 * varies them continuously; the float32 descriptor values convert exactly). */
enum { TH_BWD, TH_SYNC, TH_OPT, TH_OPT_OFF, TH_OFF, TH_SWAP, TH_CONST, N_TH };

uint32_t eval_candidate_th(const float *cf, const uint32_t *in_job, const ork_bounds *bounds,
                           const ork_env *env, uint32_t d, uint32_t t, uint32_t p, uint32_t v, uint32_t z,
                           uint32_t gc, uint32_t off, uint32_t c, float host_bytes, const double *th,
                           double *x, uint32_t n_parts = 0, const uint32_t *parts = nullptr) {
    /* the plan's micro-batch size is the job's times 2^v */
    const uint32_t in[N_INT] = {in_job[LAYERS], in_job[GBATCH], in_job[MBATCH] << v};
    for (int i = 0; i < ORK_N_TERMS; ++i) x[i] = 0.0;
    if (!option_valid(bounds, z, gc, off)) return 1u;

    const double b = in[GBATCH], mu = in[MBATCH], l = in[LAYERS];
    const double P = cf[P_BYTES], s = cf[SEQ], h = cf[HIDDEN], eb = cf[ELEM_BYTES];

    /* micro-batches per replica; pipeline plans run them as 1F1B
     * micro-batches, the others as gradient-accumulation steps */
    const double n = (double)(in[GBATCH] / (d * in[MBATCH]));
    const double m = (p > 1) ? n : 1.0;
    const double a = (p > 1) ? 1.0 : n;

    /* T_fwd: linear in per-GPU batch, tensor shard and layers per stage;
     * pipeline fill plus steady state (m + p - 1) */
    const double Tf_mb = (double)cf[T_FWD_SAMPLE] * mu / ((double)t * p);
    const double T_fwd = Tf_mb * (m + p - 1.0);
    /* T_bwd proportional to T_fwd; checkpointing recomputes one forward */
    const double T_bwd = th[TH_BWD] * T_fwd + (gc ? T_fwd : 0.0);

    /* communication volumes, zero when the corresponding size is 1 */
    const double V_dp = (d > 1) ? P * 2.0 * (d - 1.0) / ((double)d * t * p) : 0.0;
    const double V_tp = (t > 1) ? eb * 4.0 * 2.0 * (t - 1.0) * b * s * h * l / ((double)d * t) : 0.0;
    const double V_pp = (p > 1) ? eb * 2.0 * p * b * s * h / ((double)d * t) : 0.0;
    double B_dp, B_tp, B_pp;
    if (parts) bandwidths_placed(env, d, t, p, n_parts, parts, &B_dp, &B_tp, &B_pp);   /* the job's actual nodes */
    else bandwidths(env, d, t, p, &B_dp, &B_tp, &B_pp);                                 /* packed placement */
    const double T_dp = V_dp / B_dp, T_tp = V_tp / B_tp, T_pp = V_pp / B_pp;

    /* computation + communication; the accumulation form reduces to the 3D
     * form at a = 1 */
    const double sync = ork_f_overlap(th[TH_SYNC], T_bwd, T_dp);
    double T_cc;
    if (p > 1) T_cc = T_fwd + sync + T_tp + T_pp;
    else       T_cc = a * T_fwd + (a - 1.0) * T_bwd + sync + T_tp;

    /* optimizer and offloading */
    const double Psi = P / ((double)t * p);
    double T_opt, T_off = 0.0, T_oo;
    if (off) {
        T_opt = th[TH_OPT_OFF] * Psi / ((double)d * c);
        T_off = Psi / ((double)d * env->B_pcie);
        T_oo = ork_f_overlap(th[TH_OFF], T_dp, T_off) + ork_f_overlap(th[TH_SWAP], T_opt, T_off);
    } else {
        T_opt = th[TH_OPT] * Psi / ((z >= 1) ? (double)d : 1.0);
        T_oo = T_opt;
    }
    const double T_iter = T_cc + T_oo + th[TH_CONST];
    const double thr = b / T_iter;

    float M_gpu, H_host;
    memory_f32(cf, in, d, t, p, z, gc, off, &M_gpu, &H_host);
    uint32_t reason = 0;
    if (!(M_gpu <= env->gpu_mem_cap)) reason |= 2u;
    if (!(H_host <= host_bytes)) reason |= 4u;

    x[X_N] = n; x[X_M] = m; x[X_A] = a; x[X_TF_MB] = Tf_mb; x[X_T_FWD] = T_fwd; x[X_T_BWD] = T_bwd;
    x[X_V_DP] = V_dp; x[X_V_TP] = V_tp; x[X_V_PP] = V_pp; x[X_T_DP] = T_dp; x[X_T_TP] = T_tp;
    x[X_T_PP] = T_pp; x[X_T_CC] = T_cc; x[X_PSI] = Psi; x[X_T_OPT] = T_opt; x[X_T_OFF] = T_off;
    x[X_T_OO] = T_oo; x[X_T_ITER] = T_iter; x[X_THR] = thr; x[X_M_GPU] = M_gpu; x[X_H_HOST] = H_host;
    x[X_B_DP] = B_dp; x[X_B_TP] = B_tp; x[X_B_PP] = B_pp;
    return reason;
}

uint32_t eval_candidate(const float *cf, const uint32_t *in, const ork_bounds *bounds,
                        const ork_env *env, uint32_t d, uint32_t t, uint32_t p, uint32_t v, uint32_t z,
                        uint32_t gc, uint32_t off, uint32_t c, float host_bytes, double *x,
                        uint32_t n_parts = 0, const uint32_t *parts = nullptr) {
    const double th[N_TH] = {cf[K_BWD], cf[K_SYNC], cf[K_OPT], cf[K_OPT_OFF], cf[K_OFF], cf[K_SWAP], cf[K_CONST]};
    return eval_candidate_th(cf, in, bounds, env, d, t, p, v, z, gc, off, c, host_bytes, th, x, n_parts, parts);
}

int greedy_from(uint32_t n_jobs, const float *ref_thr, const ork_table *tb, const ork_grid *grid,
                uint64_t freeG, uint64_t freeC, float host_mem_gb, const float *best_thr,
                const uint32_t *best_plan, const float *curve_thr, std::vector<int64_t> &gi,
                std::vector<uint32_t> &ci, const std::vector<uint8_t> &waits, ork_assign *assign,
                double *total, double *min_gap);

int memory_step(uint32_t n_jobs, const float *ref_thr, const ork_table *tb, const ork_grid *grid, float host_mem_gb,
                const float *best_thr, const uint32_t *best_plan, const std::vector<int64_t> &gi,
                const std::vector<uint32_t> &ci, ork_assign *assign, double *total);

uint32_t cpus_of(const ork_grid *grid, uint32_t ci, uint32_t g) {
    return grid->cpu_mode ? grid->cpu_levels[ci] * g : grid->cpu_levels[ci];
}

/* host-memory tier in bytes (float32): GB * 2^30, times g in per-GPU mode */
float tier_bytes(const ork_grid *grid, uint32_t mi, uint32_t g) {
    float v = grid->mem_levels_gb[mi] * GIB;
    if (grid->mem_mode) v = v * (float)g;
    return v;
}

float tier_gb(const ork_grid *grid, uint32_t mi, uint32_t g) {
    float v = grid->mem_levels_gb[mi];
    if (grid->mem_mode) v = v * (float)g;
    return v;
}

template <typename T>
int best_plan_impl(const ork_table *tb, const ork_grid *grid, uint32_t job_begin, uint32_t job_end,
                   const T *thr, T *best_thr, uint32_t *best_plan, uint32_t n_threads) {
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    if (n_threads == 0) n_threads = 1;
    auto work = [&](uint32_t tid) {                       /* jobs are independent: threads take them in turns */
    for (uint32_t j = job_begin + tid; j < job_end; j += n_threads) {
        const uint64_t nt = tb->triple_off[j + 1] - tb->triple_off[j];
        const uint64_t ns = tb->seg_off[j + 1] - tb->seg_off[j];
        const uint64_t cbase = 16ull * rows * (tb->triple_off[j] - tb->triple_off[job_begin]);
        const uint64_t sbase = rows * (tb->seg_off[j] - tb->seg_off[job_begin]);
        for (uint64_t r = 0; r < rows; ++r) {
            for (uint64_t sg = 0; sg < ns; ++sg) {
                const uint64_t first = tb->seg_first[tb->seg_off[j] + sg];
                const uint64_t last = (sg + 1 < ns) ? tb->seg_first[tb->seg_off[j] + sg + 1] : nt;
                T bv = 0; uint32_t bp = ORK_NO_PLAN;
                for (uint64_t plan = first * 16; plan < last * 16; ++plan) {
                    const T v = thr[cbase + r * nt * 16 + plan];
                    if (v > bv) { bv = v; bp = (uint32_t)plan; }   /* strict: lowest index wins ties */
                }
                best_thr[sbase + r * ns + sg] = bv;
                best_plan[sbase + r * ns + sg] = bp;
            }
        }
    }
    };
    if (n_threads == 1) { work(0); return 0; }
    std::vector<std::thread> pool;
    for (uint32_t i = 0; i < n_threads; ++i) pool.emplace_back(work, i);
    for (auto &th : pool) th.join();
    return 0;
}

/* Free resources of the nodes and one job's first fit over them in node order
 * (Sec. 5.2, Algorithm 1, ScheduleJob): on each node the most GPUs k, up to
 * what the job still lacks, for which ceil(c*k/g) CPUs and mem*k/g GiB are free
 * there; the part is booked with floor(c*(done+k)/g) - floor(c*done/g) CPUs. */
struct NodeState {
    std::vector<uint32_t> freeG, freeC;
    std::vector<float> freeM;
    NodeState(uint32_t n, uint32_t g, uint32_t c, float m) : freeG(n, g), freeC(n, c), freeM(n, m) {}
    /* true and the parts when all g GPUs are found; nothing is booked */
    bool first_fit(uint32_t g, uint32_t c, float mem, std::vector<ork_place_entry> &parts) const {
        parts.clear();
        uint32_t done = 0;
        for (uint32_t n = 0; n < freeG.size() && done < g; ++n) {
            uint32_t k = std::min(freeG[n], g - done);
            for (; k > 0; --k) {                      /* the most GPUs whose CPUs and memory are free here */
                const uint64_t cpus = ((uint64_t)c * k + g - 1) / g;
                const float m = (mem * (float)k) / (float)g;
                if (cpus <= freeC[n] && m <= freeM[n]) break;
            }
            if (k == 0) continue;
            ork_place_entry e;
            e.node = n;
            e.g = k;
            e.c = (uint32_t)((uint64_t)c * (done + k) / g - (uint64_t)c * done / g);
            e.mem_gb = (mem * (float)k) / (float)g;
            parts.push_back(e);
            done += k;
        }
        return done == g;
    }
    void book(const std::vector<ork_place_entry> &parts) {
        for (const ork_place_entry &e : parts) {
            freeG[e.node] -= e.g;
            freeC[e.node] -= e.c;
            freeM[e.node] = freeM[e.node] - e.mem_gb;
        }
    }
};

/* What Algorithm 1's loop asks of a job's curves (Sec. 5.2, the paragraphs on slopes and on shrinking): the state the
 * jobs are in and, from it, a job's next step up and what it gives when it steps down, in GPUs and in CPU levels.
 * Shared by the loop over the cluster's totals and the loop over its nodes. */
struct Loop {
    uint32_t n_jobs;
    const float *ref_thr;
    const ork_table *tb;
    const ork_grid *grid;
    uint64_t G;                         /* GPUs of the cluster: no step goes beyond */
    const float *best_thr, *curve_thr;
    const uint8_t *state;
    const int32_t *floor_seg;
    const uint32_t *floor_c;
    std::vector<int64_t> gi;            /* what every job holds: index of its GPU count (-1 nothing) ... */
    std::vector<uint32_t> ci;           /* ... and its CPU level */

    Loop(uint32_t n, const float *ref, const ork_table *t, const ork_grid *g, uint64_t gpus, const float *best,
         const float *curve, const uint8_t *st, const int32_t *fs, const uint32_t *fc)
        : n_jobs(n), ref_thr(ref), tb(t), grid(g), G(gpus), best_thr(best), curve_thr(curve), state(st),
          floor_seg(fs), floor_c(fc), gi(n, -1), ci(n, 0) {}

    int64_t ns_of(uint32_t j) const { return (int64_t)(tb->seg_off[j + 1] - tb->seg_off[j]); }
    uint64_t g_at(uint32_t j, int64_t s) const { return s < 0 ? 0 : tb->seg_g[tb->seg_off[j] + s]; }
    uint64_t c_at(uint32_t j, uint32_t c, int64_t s) const { return s < 0 ? 0 : cpus_of(grid, c, (uint32_t)g_at(j, s)); }
    /* value of job j at CPU level c, highest memory tier, GPU count s (0 below the first) */
    float at(const float *arr, uint32_t j, uint32_t c, int64_t s) const {
        const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
        const uint32_t m_top = grid->n_mem - 1;
        return s < 0 ? 0.0f : arr[rows * tb->seg_off[j] + ((uint64_t)c * grid->n_mem + m_top) * ns_of(j) + s];
    }
    /* state 0: the job takes part; 2: it keeps exactly what it holds (it takes no step and gives nothing); anything
       else: it takes no part and holds nothing */
    bool part(uint32_t j) const { return !state || state[j] == 0; }
    bool holds(uint32_t j) const { return !state || state[j] == 0 || state[j] == 2; }
    /* the job's floor: a segment the job does not have counts as none, the CPU level is clamped to the grid */
    int64_t fl_s(uint32_t j) const {
        return (floor_seg && floor_seg[j] >= 0 && floor_seg[j] < ns_of(j)) ? floor_seg[j] : -1;
    }
    uint32_t fl_c(uint32_t j) const {
        return (fl_s(j) >= 0 && floor_c) ? std::min(floor_c[j], grid->n_cpu - 1) : 0u;
    }

    struct Step { bool any; int64_t tgt; uint32_t lvl; float slope, gain; uint64_t dg, dc; };
    /* the next GPU step of job j: to its floor while below it, else the larger count with the highest slope */
    Step up_gpu(uint32_t j) const {
        Step st = {false, -1, ci[j], 0.0f, 0.0f, 0, 0};
        const float cur = at(curve_thr, j, ci[j], gi[j]);
        if (fl_s(j) >= 0 && gi[j] < fl_s(j)) {
            const uint32_t lvl = std::max(ci[j], fl_c(j));
            const float v = at(curve_thr, j, lvl, fl_s(j));
            st.any = true; st.tgt = fl_s(j); st.lvl = lvl;
            st.dg = g_at(j, fl_s(j)) - g_at(j, gi[j]);
            st.dc = c_at(j, lvl, fl_s(j)) - c_at(j, ci[j], gi[j]);
            st.gain = (v - cur) / ref_thr[j];
            st.slope = st.gain / (float)st.dg;
            return st;
        }
        for (int64_t s = gi[j] + 1; s < ns_of(j); ++s) {
            const uint64_t dg = g_at(j, s) - g_at(j, gi[j]);
            if (g_at(j, s) > G) break;
            const float v = at(curve_thr, j, ci[j], s);
            if (!(v > cur)) continue;
            const float gain = (v - cur) / ref_thr[j];
            const float sl = gain / (float)dg;
            if (sl > st.slope) {
                st.any = true; st.tgt = s; st.slope = sl; st.gain = gain; st.dg = dg;
                st.dc = c_at(j, ci[j], s) - c_at(j, ci[j], gi[j]);
            }
        }
        return st;
    }
    Step up_cpu(uint32_t j) const {
        Step st = {false, gi[j], ci[j], 0.0f, 0.0f, 0, 0};
        if (gi[j] < 0) return st;
        const float cur = at(best_thr, j, ci[j], gi[j]);
        for (uint32_t c = ci[j] + 1; c < grid->n_cpu; ++c) {
            const uint64_t dc = c_at(j, c, gi[j]) - c_at(j, ci[j], gi[j]);
            const float v = at(best_thr, j, c, gi[j]);
            if (!(v > cur)) continue;
            const float gain = (v - cur) / ref_thr[j];
            const float sl = gain / (float)dc;
            if (sl > st.slope) { st.any = true; st.lvl = c; st.slope = sl; st.gain = gain; st.dc = dc; }
        }
        return st;
    }
    /* what job v gives when it steps down in GPUs: target segment (-1 = everything), loss, units */
    struct Give { bool any; int64_t tgt; float loss, slope; uint64_t dg, dc; };
    Give down_gpu(uint32_t v) const {
        Give gv = {false, -1, 0.0f, 0.0f, 0, 0};
        if (gi[v] < 0 || (fl_s(v) >= 0 && gi[v] <= fl_s(v))) return gv;
        const float V = at(curve_thr, v, ci[v], gi[v]);
        /* down to where the curve's value just below begins: the largest amount with a lower throughput, or, when
           the job holds more than it uses (same value just below), the smallest amount with the same throughput */
        const float want = at(curve_thr, v, ci[v], gi[v] - 1);
        int64_t t = -1;
        if (want > 0.0f) for (t = 0; at(curve_thr, v, ci[v], t) != want; ++t) {}
        if (fl_s(v) >= 0 && t < fl_s(v)) t = fl_s(v);
        gv.any = true; gv.tgt = t;
        gv.loss = (V - at(curve_thr, v, ci[v], t)) / ref_thr[v];
        gv.dg = g_at(v, gi[v]) - g_at(v, t);
        gv.dc = c_at(v, ci[v], gi[v]) - c_at(v, ci[v], t);
        gv.slope = gv.loss / (float)gv.dg;
        return gv;
    }
    Give down_cpu(uint32_t v) const {
        Give gv = {false, gi[v], 0.0f, 0.0f, 0, 0};
        const uint32_t lowest = (fl_s(v) >= 0) ? fl_c(v) : 0u;
        if (gi[v] < 0 || ci[v] == 0 || ci[v] <= lowest) return gv;
        gv.any = true;
        gv.loss = (at(best_thr, v, ci[v], gi[v]) - at(best_thr, v, ci[v] - 1, gi[v])) / ref_thr[v];
        gv.dc = c_at(v, ci[v], gi[v]) - c_at(v, ci[v] - 1, gi[v]);
        gv.slope = gv.loss / (float)gv.dc;
        return gv;
    }
};

}  // namespace

extern "C" {

/* Sec. 4.3 "Modeling overlapping": the definition, written out.
 * Pinned: k=1 gives x+y, large k approaches max, f(k;x,0)=x, f(k;x,x)=x*2^(1/k). */
double ork_f_overlap(double k, double x, double y) {
    return std::pow(std::pow(x, k) + std::pow(y, k), 1.0 / k);
}

/* Plan space of Sec. 3 (3D parallel sizes with d*t*p = g, Table 1) under the
 * partitioning constraints Fig. 6 alludes to: t a power of two up to tp_max,
 * p divides the layer count, d*mu*2^v divides the global batch for the
 * micro-batch shifts v that the bounds allow (Table 1 lists the number of
 * micro-batches m and of accumulation steps a among the plan's quantities).
 * Entries are (d, t, p, v), ordered by g, then t, p, v.
 * Pinned: brute force over [1..g]^3 in the tests; with constraints lifted the
 * count per g is the number of ordered factorisations into three factors. */
int ork_enumerate(uint32_t n_jobs, const uint32_t *ints, const ork_bounds *bounds,
                  uint32_t *triple_off, uint32_t *triples, uint64_t cap_triples,
                  uint32_t *seg_off, uint32_t *seg_g, uint32_t *seg_first, uint64_t cap_segs,
                  uint64_t *n_triples, uint64_t *n_segs, uint32_t n_threads) {
    /* every job on its own (the jobs are independent; threads take them in turns), then laid end to end */
    struct JobPlans { std::vector<uint32_t> dtpv, seg_g, seg_first; };
    std::vector<JobPlans> per_job(n_jobs);
    auto search = [&](uint32_t tid, uint32_t step) {
        for (uint32_t j = tid; j < n_jobs; j += step) {
            const uint32_t l = ints[j * 3 + LAYERS], b = ints[j * 3 + GBATCH], mu = ints[j * 3 + MBATCH];
            JobPlans &out = per_job[j];
            for (uint32_t g = 1; g <= bounds->g_max; ++g) {
                bool any = false;
                for (uint32_t t = 1; t <= 8 && t <= bounds->tp_max; t *= 2) {
                    for (uint32_t p = 1; p <= bounds->pp_max && p <= l; ++p) {
                        if (l % p != 0) continue;
                        if (g % (t * p) != 0) continue;
                        const uint32_t d = g / (t * p);
                        for (uint32_t v = 0; v < 4; ++v) {
                            if (!((bounds->mu_mask >> v) & 1u)) continue;
                            // n = b/(d*mu*2^v) micro-batches per replica: a whole number, at least one
                            if (mu == 0 || b == 0 || b % ((uint64_t)d * (mu << v)) != 0) continue;
                            if (!any) {
                                any = true;
                                out.seg_g.push_back(g);
                                out.seg_first.push_back((uint32_t)(out.dtpv.size() / 4));
                            }
                            out.dtpv.push_back(d); out.dtpv.push_back(t); out.dtpv.push_back(p); out.dtpv.push_back(v);
                        }
                    }
                }
            }
        }
    };
    if (n_threads <= 1) search(0, 1);
    else {
        std::vector<std::thread> pool;
        for (uint32_t i = 0; i < n_threads; ++i) pool.emplace_back(search, i, n_threads);
        for (auto &th : pool) th.join();
    }
    uint64_t nt = 0, ns = 0;
    const bool write = triple_off && triples && seg_off && seg_g && seg_first;
    bool overflow = false;
    for (uint32_t j = 0; j < n_jobs; ++j) {
        const JobPlans &in = per_job[j];
        if (write) { triple_off[j] = (uint32_t)nt; seg_off[j] = (uint32_t)ns; }
        const uint64_t jt = in.dtpv.size() / 4, js = in.seg_g.size();
        if (write) {
            if (nt + jt <= cap_triples) std::copy(in.dtpv.begin(), in.dtpv.end(), triples + nt * 4);
            else overflow = true;
            if (ns + js <= cap_segs) {
                std::copy(in.seg_g.begin(), in.seg_g.end(), seg_g + ns);
                std::copy(in.seg_first.begin(), in.seg_first.end(), seg_first + ns);
            } else overflow = true;
        }
        nt += jt; ns += js;
    }
    if (write) { triple_off[n_jobs] = (uint32_t)nt; seg_off[n_jobs] = (uint32_t)ns; }
    if (n_triples) *n_triples = nt;
    if (n_segs) *n_segs = ns;
    return overflow ? -1 : 0;
}

/* Host threads the machine offers (what the benchmark states beside the oracle's timings). */
uint32_t ork_host_cores(void) { return std::thread::hardware_concurrency(); }

uint32_t ork_eval_one(const float *coef17, const uint32_t *ints3, const ork_bounds *bounds,
                      const ork_env *env, uint32_t d, uint32_t t, uint32_t p, uint32_t v, uint32_t z,
                      uint32_t gc, uint32_t off, uint32_t c, float host_bytes, double *terms) {
    return eval_candidate(coef17, ints3, bounds, env, d, t, p, v, z, gc, off, c, host_bytes, terms);
}

/* One candidate whose GPUs are parts[0..n_parts) on consecutive nodes of its
 * placement (sum = d*t*p): the bandwidth of every communication group follows
 * where its ranks landed.  Pinned: hand cases of the bandwidth classes. */
uint32_t ork_eval_one_placed(const float *coef17, const uint32_t *ints3, const ork_bounds *bounds,
                             const ork_env *env, uint32_t d, uint32_t t, uint32_t p, uint32_t v, uint32_t z,
                             uint32_t gc, uint32_t off, uint32_t c, float host_bytes, uint32_t n_parts,
                             const uint32_t *parts, double *terms) {
    return eval_candidate(coef17, ints3, bounds, env, d, t, p, v, z, gc, off, c, host_bytes, terms, n_parts, parts);
}

/* Predicted throughput of measured runs ("samples") of one model type under
 * the parameter tuple th (Sec. 4 "Continuous model fitting": the fit compares
 * Eq. (1) with the collected data).  Sample i = plan (d,t,p, option code) on
 * cpus[i] CPUs; memory feasibility plays no part (the runs did happen).
 * Structurally invalid samples (d*mu does not divide b, p does not divide l)
 * give 0.  Same arithmetic as every other evaluation here. */
int ork_predict_f64(const float *coef17, const uint32_t *ints3, const ork_env *env, const double *th,
                    uint32_t n_samples, const uint32_t *d, const uint32_t *t, const uint32_t *p,
                    const uint32_t *mu_shift, const uint32_t *option, const uint32_t *cpus, double *thr,
                    double *t_iter) {
    const ork_bounds all = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xF, 0x3, 0x3, 0xF};
    double x[ORK_N_TERMS];
    for (uint32_t i = 0; i < n_samples; ++i) {
        const uint32_t o = option[i], z = o >> 2, gc = (o >> 1) & 1u, off = o & 1u;
        thr[i] = 0.0;
        if (t_iter) t_iter[i] = 0.0;
        const uint32_t v = mu_shift ? mu_shift[i] : 0u;
        if (d[i] == 0 || t[i] == 0 || p[i] == 0 || o > 15u || v > 3u) continue;
        if (ints3[GBATCH] % ((uint64_t)d[i] * (ints3[MBATCH] << v)) != 0 || ints3[LAYERS] % p[i] != 0) continue;
        if (off && cpus[i] == 0) continue;
        const uint32_t reason = eval_candidate_th(coef17, ints3, &all, env, d[i], t[i], p[i], v, z, gc, off, cpus[i],
                                                  INFINITY, th, x);
        if (reason & 1u) continue;
        thr[i] = x[X_THR];
        if (t_iter) t_iter[i] = x[X_T_ITER];
    }
    return 0;
}

/* The plain definition: every candidate evaluated from scratch. */
int ork_eval_jobs(uint32_t n_jobs, const float *coef, const uint32_t *ints,
                  const ork_bounds *bounds, const ork_table *tb, const ork_grid *grid,
                  const ork_env *env, uint32_t job_begin, uint32_t job_end,
                  double *thr, uint8_t *reason_out, uint32_t n_threads) {
    if (job_end > n_jobs || job_begin > job_end) return -1;
    if (n_threads == 0) n_threads = 1;
    const uint64_t rows_m = grid->n_mem;
    auto work = [&](uint32_t tid) {
        double x[ORK_N_TERMS];
        for (uint32_t j = job_begin + tid; j < job_end; j += n_threads) {
            const float *cf = coef + (uint64_t)j * N_COEF;
            const uint32_t *in = ints + (uint64_t)j * N_INT;
            const uint64_t nt = tb->triple_off[j + 1] - tb->triple_off[j];
            const uint64_t cbase = 16ull * grid->n_cpu * grid->n_mem *
                                   (tb->triple_off[j] - tb->triple_off[job_begin]);
            for (uint32_t ci = 0; ci < grid->n_cpu; ++ci)
            for (uint32_t mi = 0; mi < grid->n_mem; ++mi)
            for (uint64_t tl = 0; tl < nt; ++tl) {
                const uint32_t *tr = tb->triples + (tb->triple_off[j] + tl) * 4;
                const uint32_t d = tr[0], t = tr[1], p = tr[2], v = tr[3], g = d * t * p;
                for (uint32_t o = 0; o < 16; ++o) {
                    const uint32_t z = o >> 2, gc = (o >> 1) & 1u, off = o & 1u;
                    const uint32_t c = cpus_of(grid, ci, g);
                    const float hb = tier_bytes(grid, mi, g);
                    const uint32_t reason = eval_candidate(cf, in, bounds, env, d, t, p, v, z, gc, off, c, hb, x);
                    const uint64_t idx = cbase + ((ci * rows_m + mi) * nt + tl) * 16 + o;
                    thr[idx] = reason ? 0.0 : x[X_THR];
                    if (reason_out) reason_out[idx] = (uint8_t)reason;
                }
            }
        }
    };
    if (n_threads == 1) { work(0); return 0; }
    std::vector<std::thread> pool;
    for (uint32_t i = 0; i < n_threads; ++i) pool.emplace_back(work, i);
    for (auto &th : pool) th.join();
    return 0;
}

/* GetBestPlan of Sec. 5.2 / Algorithm 1: the best predicted throughput among
 * the feasible plans for a given resource amount; lowest plan index on exact
 * ties; no feasible plan gives (0, ORK_NO_PLAN).
 * Pinned: numpy argmax over a flat list in the tests. */
int ork_best_plan_f64(const ork_table *tb, const ork_grid *grid, uint32_t jb, uint32_t je,
                      const double *thr, double *best_thr, uint32_t *best_plan, uint32_t n_threads) {
    return best_plan_impl<double>(tb, grid, jb, je, thr, best_thr, best_plan, n_threads);
}
int ork_best_plan_f32(const ork_table *tb, const ork_grid *grid, uint32_t jb, uint32_t je,
                      const float *thr, float *best_thr, uint32_t *best_plan, uint32_t n_threads) {
    return best_plan_impl<float>(tb, grid, jb, je, thr, best_thr, best_plan, n_threads);
}

/* Resource sensitivity curve (Sec. 5.2, Fig. 6): for each GPU count the
 * maximum throughput achievable within that many GPUs, so the curve is flat
 * over counts that bring nothing; keeps the smallest count reaching the
 * maximum and its plan.  Pinned: numpy maximum.accumulate in the tests. */
int ork_curves_f32(const ork_table *tb, const ork_grid *grid, uint32_t jb, uint32_t je,
                   const float *best_thr, const uint32_t *best_plan,
                   float *curve_thr, uint32_t *curve_plan, uint32_t *curve_g) {
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    for (uint32_t j = jb; j < je; ++j) {
        const uint64_t ns = tb->seg_off[j + 1] - tb->seg_off[j];
        const uint64_t sbase = rows * (tb->seg_off[j] - tb->seg_off[jb]);
        for (uint64_t r = 0; r < rows; ++r) {
            float cur = 0.0f; uint32_t plan = ORK_NO_PLAN, gg = 0;
            for (uint64_t sg = 0; sg < ns; ++sg) {
                const uint64_t i = sbase + r * ns + sg;
                if (best_thr[i] > cur) { cur = best_thr[i]; plan = best_plan[i]; gg = tb->seg_g[tb->seg_off[j] + sg]; }
                curve_thr[i] = cur; curve_plan[i] = plan; curve_g[i] = gg;
            }
        }
    }
    return 0;
}

/* Minimum demand of guaranteed jobs (Sec. 5.2 "Scheduling algorithm design"):
 * the fewest resources, not above the request in any dimension, whose best
 * plan reaches the performance of the requested resources with the original
 * plan (base_thr).  "Fewest" is read as: fewest GPUs, then fewest CPUs, then
 * smallest memory tier.  If nothing qualifies the request itself is the
 * minimum.  Best-effort jobs have no minimum (segment -1).  A guaranteed job
 * whose request is below its smallest valid GPU count gets -1 as well.
 * Pinned: brute force over the same arrays in the tests, hand cases. */
int ork_min_res_f32(const ork_table *tb, const ork_grid *grid, uint32_t jb, uint32_t je,
                    const float *best_thr, const uint32_t *guaranteed, const uint32_t *req_g,
                    const uint32_t *req_c, const uint32_t *req_m, const float *base_thr,
                    int32_t *min_seg, uint32_t *min_c, uint32_t *min_m) {
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    for (uint32_t j = jb; j < je; ++j) {
        const uint32_t o = j - jb;
        min_seg[o] = -1; min_c[o] = 0; min_m[o] = 0;
        if (!guaranteed[j]) continue;
        const uint64_t ns = tb->seg_off[j + 1] - tb->seg_off[j];
        const uint64_t sbase = rows * (tb->seg_off[j] - tb->seg_off[jb]);
        int64_t s_req = -1;
        for (uint64_t s = 0; s < ns; ++s) if (tb->seg_g[tb->seg_off[j] + s] <= req_g[j]) s_req = (int64_t)s;
        if (s_req < 0) continue;
        const uint32_t c_req = req_c[j] < grid->n_cpu ? req_c[j] : grid->n_cpu - 1;
        const uint32_t m_req = req_m[j] < grid->n_mem ? req_m[j] : grid->n_mem - 1;
        bool found = false;
        for (int64_t s = 0; s <= s_req && !found; ++s)
            for (uint32_t c = 0; c <= c_req && !found; ++c)
                for (uint32_t m = 0; m <= m_req && !found; ++m) {
                    const float v = best_thr[sbase + ((uint64_t)c * grid->n_mem + m) * ns + s];
                    if (v > 0.0f && v >= base_thr[j]) {
                        min_seg[o] = (int32_t)s; min_c[o] = c; min_m[o] = m; found = true;
                    }
                }
        if (!found) { min_seg[o] = (int32_t)s_req; min_c[o] = c_req; min_m[o] = m_req; }
    }
    return 0;
}

/* Greedy marginal-gain allocation: a reading of Sec. 5.2 (slopes of the
 * curves, "slopes of GPUs and then CPUs", memory allocated last from the
 * chosen plan's estimate) with every job best-effort and the cluster as
 * totals.  Slopes are float32: ((v1 - v0) / ref_thr) / delta.
 *  GPU pass : repeatedly give the (job, larger GPU count) with the highest
 *             normalised throughput gain per GPU, at the lowest CPU level and
 *             the highest memory tier; ties -> smaller count, lower job index.
 *  CPU pass : same over CPU levels at the granted GPU count.
 *  Memory   : in job order, among the tiers that still fit, the one with the
 *             highest throughput (smallest such tier); none feasible -> the
 *             job is dropped and its GPUs/CPUs stay unused this round.
 * PARITY UNPINNED as a heuristic reading; the tests pin capacity invariants,
 * optimality on concave curves against exhaustive search, and hand cases. */
int ork_greedy_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *tb,
                   const ork_grid *grid, uint32_t G, uint32_t C, float host_mem_gb,
                   const float *best_thr, const uint32_t *best_plan,
                   const float *curve_thr, ork_assign *assign, double *total, double *min_gap) {
    return ork_policy_f32(n_jobs, ref_thr, tb, grid, G, C, host_mem_gb, best_thr, best_plan, curve_thr,
                          nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, assign, total, min_gap);
}

/* The greedy with service-level floors (Sec. 5.2: guaranteed jobs within their
 * tenant's quota are scheduled first with at least their minimum demand; the
 * remaining resources go to the jobs with the highest slopes).
 *  Privileged phase: guaranteed jobs in job order; a job whose minimum demand
 *  (GPUs, CPUs) fits its tenant's remaining quota and the free capacity is
 *  granted it; otherwise it waits for a later round and takes no part in this
 *  one.  Then the GPU pass, CPU pass and memory step of the greedy run from
 *  these floors; a job's GPU pass uses its floor's CPU level.
 * PARITY UNPINNED as a reading; pinned by invariants and hand cases. */
int ork_policy_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *tb,
                   const ork_grid *grid, uint32_t G, uint32_t C, float host_mem_gb,
                   const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                   const uint32_t *guaranteed, const uint32_t *tenant, const int32_t *min_seg,
                   const uint32_t *min_c, uint32_t n_tenants, const uint32_t *quota_g,
                   const uint32_t *quota_c, ork_assign *assign, double *total, double *min_gap) {
    std::vector<int64_t> gi(n_jobs, -1);
    std::vector<uint32_t> ci(n_jobs, 0);
    std::vector<uint8_t> waits(n_jobs, 0);
    uint64_t freeG = G, freeC = C;
    if (guaranteed) {                                       /* privileged phase */
        std::vector<uint64_t> qg(quota_g, quota_g + n_tenants), qc(quota_c, quota_c + n_tenants);
        for (uint32_t j = 0; j < n_jobs; ++j) {
            if (!guaranteed[j]) continue;
            waits[j] = 1;
            if (min_seg[j] < 0 || tenant[j] >= n_tenants) continue;
            const uint64_t g = tb->seg_g[tb->seg_off[j] + min_seg[j]];
            const uint64_t c = cpus_of(grid, min_c[j], (uint32_t)g);
            const uint32_t t = tenant[j];
            if (g <= qg[t] && c <= qc[t] && g <= freeG && c <= freeC) {
                qg[t] -= g; qc[t] -= c; freeG -= g; freeC -= c;
                gi[j] = min_seg[j]; ci[j] = min_c[j]; waits[j] = 0;
            }
        }
    }
    return greedy_from(n_jobs, ref_thr, tb, grid, freeG, freeC, host_mem_gb, best_thr, best_plan, curve_thr,
                       gi, ci, waits, assign, total, min_gap);
}

/* A round in which some jobs take no part (state 1) and some keep what they
 * hold (state 2: frozen at segment cur_seg and CPU level cur_c, e.g. because a
 * reconfiguration would cost them too much, Sec. 5.2 "Incorporating
 * reconfiguration penalty").  Frozen jobs are charged first; if they hold more
 * than the cluster has, nothing is left for the others.  Everything else is the
 * greedy.  Pinned: hand cases; all-normal equals the plain greedy. */
int ork_frozen_round_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *tb,
                         const ork_grid *grid, uint32_t G, uint32_t C, float host_mem_gb,
                         const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                         const uint8_t *state, const int32_t *cur_seg, const uint32_t *cur_c,
                         ork_assign *assign, double *total, double *min_gap) {
    std::vector<int64_t> gi(n_jobs, -1);
    std::vector<uint32_t> ci(n_jobs, 0);
    std::vector<uint8_t> skip(n_jobs, 0);
    uint64_t heldG = 0, heldC = 0;
    for (uint32_t j = 0; j < n_jobs; ++j) {
        skip[j] = state[j];
        if (state[j] == 2) {
            const uint64_t ns = tb->seg_off[j + 1] - tb->seg_off[j];
            if (cur_seg[j] < 0 || (uint64_t)cur_seg[j] >= ns || cur_c[j] >= grid->n_cpu) { skip[j] = 1; continue; }
            gi[j] = cur_seg[j]; ci[j] = cur_c[j];
            const uint32_t g = tb->seg_g[tb->seg_off[j] + cur_seg[j]];
            heldG += g; heldC += cpus_of(grid, cur_c[j], g);
        }
    }
    const uint64_t freeG = heldG < G ? G - heldG : 0, freeC = heldC < C ? C - heldC : 0;
    return greedy_from(n_jobs, ref_thr, tb, grid, freeG, freeC, host_mem_gb, best_thr, best_plan, curve_thr,
                       gi, ci, skip, assign, total, min_gap);
}

/* Sec. 5.2, Algorithm 1 (ScheduleJob): first fit over the nodes in order. */
int ork_place_f32(uint32_t n_jobs, const ork_assign *assign, uint32_t n_nodes, uint32_t gpus_per_node,
                  uint32_t cpus_per_node, float mem_per_node_gb, uint32_t *place_off,
                  ork_place_entry *entries, uint32_t *status) {
    NodeState nodes(n_nodes, gpus_per_node, cpus_per_node, mem_per_node_gb);
    uint32_t n_entries = 0;
    for (uint32_t j = 0; j < n_jobs; ++j) {
        place_off[j] = n_entries;
        status[j] = 0;
        if (assign[j].g == 0) continue;
        std::vector<ork_place_entry> parts;
        if (!nodes.first_fit(assign[j].g, assign[j].c, assign[j].mem_gb, parts)) { status[j] = 2; continue; }
        status[j] = 1;
        nodes.book(parts);
        for (const ork_place_entry &e : parts) entries[n_entries++] = e;
    }
    place_off[n_jobs] = n_entries;
    return 0;
}

/* Placement that feeds the plan (Sec. 5.2, Algorithm 1, ScheduleJob from the
 * placement record to the return: the job walks the nodes, and if what it
 * found satisfies at least its minimum demand the plan is selected given the
 * found placement, then memory is allocated from that plan's estimate; last
 * paragraph of Sec. 5.2: a job placed on several nodes is predicted with the
 * inter-node bandwidth).
 *  Jobs in index order, every node starts empty.  A job comes with the
 *  amounts an allocation decided (assign[j]: g GPUs = one of its valid counts,
 *  c CPUs = a CPU level at that count, mem_gb = a memory tier at that count).
 *  It tries first fit with these; when the nodes do not hold them it tries its
 *  next smaller valid GPU count (same CPU level and memory tier, so the
 *  amounts shrink with the grid's modes) that has a feasible plan there, and
 *  so on, but never below its floor (min_seg[j], -1 = none): Algorithm 1
 *  accepts what the search found as long as the minimum demand is met.
 *  A placed job's plan is searched again among the plans of its GPU count that
 *  are feasible at its CPUs and memory tier, each evaluated with the bandwidths
 *  of the actual node split (bandwidths_placed); best throughput, lowest plan
 *  index on ties.
 * out[j] = the amounts placed, the plan and its throughput (zeros / no plan
 * when the job got nothing); status 0 nothing to place, 1 placed, 2 placed
 * with fewer GPUs than asked, 3 not placed.  total = sum of thr / ref_thr.
 * best_thr (segment layout of all jobs) says which (count, level, tier) have a
 * feasible plan at all.
 *  With an earlier placement (prev_off, prev_entries; NULL: none) running jobs
 *  stay where they are (Algorithm 1's ScheduleJob adds to what a job holds): a
 *  job whose amounts are the ones its earlier parts add up to - the same GPUs
 *  and CPUs, and every part is what first fit books for these amounts on that
 *  split - keeps those parts; all kept jobs are booked before any other job
 *  looks for room, the others then take their turns in index order as above.
 *  Returns -1 when the kept parts do not fit the nodes (prev is then not a
 *  placement on these nodes).
 * PARITY UNPINNED as a reading; pinned by hand cases (a 3+1 split that flips
 * the best plan, a retry at a smaller count, the floor, jobs that stay) and by
 * brute force over the plans on generated rounds. */
int ork_place_plans(uint32_t n_jobs, const float *coef, const uint32_t *ints, const ork_bounds *bounds,
                    const ork_table *tb, const ork_grid *grid, const ork_env *env, const float *best_thr,
                    const ork_assign *assign, const int32_t *min_seg, const uint32_t *prev_off,
                    const ork_place_entry *prev_entries, uint32_t n_nodes, uint32_t gpus_per_node,
                    uint32_t cpus_per_node, float mem_per_node_gb, ork_assign *out, uint32_t *place_off,
                    ork_place_entry *entries, uint32_t *status, double *total) {
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    NodeState nodes(n_nodes, gpus_per_node, cpus_per_node, mem_per_node_gb);
    uint32_t n_entries = 0;
    double sum = 0.0;
    double x[ORK_N_TERMS];
    /* the jobs that stay: booked first, whatever their index */
    std::vector<uint8_t> kept(n_jobs, 0);
    if (prev_off && prev_entries) {
        for (uint32_t j = 0; j < n_jobs; ++j) {
            const uint32_t g = assign[j].g, c = assign[j].c;
            const float mem = assign[j].mem_gb;
            const uint32_t a = prev_off[j], b = prev_off[j + 1];
            if (g == 0 || a == b) continue;
            uint64_t done = 0;
            bool same = true;
            for (uint32_t i = a; i < b && same; ++i) {
                const ork_place_entry &e = prev_entries[i];
                if (e.node >= n_nodes || e.g == 0 || done + e.g > g) { same = false; break; }
                const uint32_t cpus = (uint32_t)((uint64_t)c * (done + e.g) / g - (uint64_t)c * done / g);
                const float m = (mem * (float)e.g) / (float)g;
                if (e.c != cpus || !(e.mem_gb == m)) same = false;
                done += e.g;
            }
            kept[j] = same && done == g;
        }
        for (uint32_t j = 0; j < n_jobs; ++j) {
            if (!kept[j]) continue;
            for (uint32_t i = prev_off[j]; i < prev_off[j + 1]; ++i) {
                const ork_place_entry &e = prev_entries[i];
                if (nodes.freeG[e.node] < e.g || nodes.freeC[e.node] < e.c || !(e.mem_gb <= nodes.freeM[e.node])) return -1;
                nodes.freeG[e.node] -= e.g;
                nodes.freeC[e.node] -= e.c;
                nodes.freeM[e.node] = nodes.freeM[e.node] - e.mem_gb;
            }
        }
    }
    for (uint32_t j = 0; j < n_jobs; ++j) {
        place_off[j] = n_entries;
        status[j] = 0;
        out[j] = ork_assign{0, 0, 0.0f, ORK_NO_PLAN, 0.0f};
        const uint32_t g0 = assign[j].g;
        if (g0 == 0) continue;
        const uint32_t s_off = tb->seg_off[j], ns = tb->seg_off[j + 1] - s_off;
        /* where the amounts sit in the grid: the GPU count among the job's counts, the CPU level and the tier */
        int64_t s0 = -1, ci = -1, mi = -1;
        for (uint32_t s = 0; s < ns; ++s) if (tb->seg_g[s_off + s] == g0) s0 = s;
        for (uint32_t c = 0; c < grid->n_cpu; ++c) if (cpus_of(grid, c, g0) == assign[j].c) ci = c;
        for (uint32_t m = 0; m < grid->n_mem; ++m) if (tier_gb(grid, m, g0) == assign[j].mem_gb) mi = m;
        if (s0 < 0 || ci < 0 || mi < 0) return -1;          /* not an allocation on this table and grid */
        if (!(best_thr[rows * s_off + ((uint64_t)ci * grid->n_mem + mi) * ns + s0] > 0.0f)) return -1;   /* no plan there */
        const int64_t s_min = (min_seg && min_seg[j] >= 0) ? min_seg[j] : 0;
        std::vector<ork_place_entry> parts;
        int64_t s = -1;
        if (kept[j]) {                                      /* stays where it is; its parts are booked already */
            parts.assign(prev_entries + prev_off[j], prev_entries + prev_off[j + 1]);
            s = s0;
        }
        for (int64_t s2 = s0; s2 >= 0 && s < 0; --s2) {     /* the amounts asked for, then smaller valid counts */
            if (s2 != s0) {
                if (s2 < s_min) break;                      /* never below the floor */
                if (!(best_thr[rows * s_off + ((uint64_t)ci * grid->n_mem + mi) * ns + s2] > 0.0f)) continue;
            }
            const uint32_t g = tb->seg_g[s_off + s2];
            if (nodes.first_fit(g, cpus_of(grid, (uint32_t)ci, g), tier_gb(grid, (uint32_t)mi, g), parts)) s = s2;
        }
        if (s < 0) { status[j] = 3; continue; }
        status[j] = (s == s0) ? 1 : 2;
        if (!kept[j]) nodes.book(parts);
        std::vector<uint32_t> split;
        for (const ork_place_entry &e : parts) { entries[n_entries++] = e; split.push_back(e.g); }
        /* GetBestPlan(j, placement): the plans of this GPU count with the bandwidths of this split */
        const uint32_t g = tb->seg_g[s_off + s], c = cpus_of(grid, (uint32_t)ci, g);
        const float hb = tier_bytes(grid, (uint32_t)mi, g);
        const uint32_t t_off = tb->triple_off[j], nt = tb->triple_off[j + 1] - t_off;
        const uint32_t first = tb->seg_first[s_off + s];
        const uint32_t last = ((uint32_t)s + 1 < ns) ? tb->seg_first[s_off + s + 1] : nt;
        double bv = 0.0; uint32_t bp = ORK_NO_PLAN;
        for (uint32_t tl = first; tl < last; ++tl) {
            const uint32_t *tr = tb->triples + (uint64_t)(t_off + tl) * 4;
            for (uint32_t o = 0; o < 16; ++o) {
                const uint32_t reason = eval_candidate(coef + (uint64_t)j * N_COEF, ints + (uint64_t)j * N_INT, bounds, env,
                                                       tr[0], tr[1], tr[2], tr[3], o >> 2, (o >> 1) & 1u, o & 1u, c, hb, x,
                                                       (uint32_t)split.size(), split.data());
                if (!reason && x[X_THR] > bv) { bv = x[X_THR]; bp = tl * 16 + o; }   /* strict: lowest index on ties */
            }
        }
        out[j] = ork_assign{g, c, tier_gb(grid, (uint32_t)mi, g), bp, (float)bv};
        sum += (double)(float)bv / (double)coef[(uint64_t)j * N_COEF + REF_THR];
    }
    place_off[n_jobs] = n_entries;
    if (total) *total = sum;
    return 0;
}

/* Algorithm 1's Schedule as the loop it is written as (Sec. 5.2, "Scheduling
 * algorithm design" and the paragraph on shrinking), from the state the jobs
 * are in: running jobs keep what they hold unless another job takes it.
 *   - Privileged jobs first, in job order: the jobs that have a floor
 *     (floor_seg >= 0) and hold fewer GPUs than it.  Then all other jobs that
 *     take part, sorted once by their GPU slope, then their CPU slope (both
 *     descending), then their index.
 *   - ScheduleJob(j), for GPUs and then for CPUs: while j has a next step (for
 *     a job below its floor: the step to the floor with the floor's CPU level;
 *     otherwise the larger amount with the highest slope, as in the greedy,
 *     whatever is free), the amount the step needs is gathered from what is
 *     free and then from the other jobs, always from the one with the lowest
 *     slope among those above their own floor (GetLowestSlopeOverMinJob; ties:
 *     lower index).  The reallocation unit of a job is the distance to its
 *     next useful amount: a job that gives steps down to the largest amount
 *     with a lower throughput (to the smallest amount with the same throughput
 *     when it holds more than it uses), never below its floor; its slope is
 *     the normalised throughput it loses per unit it gives.  A job may be
 *     shrunk when j's slope is higher than its slope, or when j is below its
 *     floor.  The step is committed when everything was found and, unless j is
 *     below its floor, j's gain exceeds what the others lose together;
 *     otherwise every job is put back and j's search in this resource ends.
 *     A GPU step must find its CPUs (at j's CPU level) free or freed by the
 *     same shrinks.
 *   - A job shrunk to nothing is preempted (best-effort jobs only: a job with
 *     a floor stops there).  Memory last, as in the greedy.
 * state[j] = 1 (or anything but 0 and 2): the job takes no part and holds
 * nothing; 2: it keeps exactly what it holds, takes no step and gives nothing
 * (a job that must not be reconfigured now, Sec. 5.2 "Incorporating
 * reconfiguration penalty").  n_moves = steps committed.  PARITY UNPINNED as a reading (the paper gives the outline);
 * pinned by hand cases for every rule above, by the greedy and the exhaustive
 * optimum on concave curves from an empty cluster, and by invariants. */
int ork_reschedule_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *tb, const ork_grid *grid,
                       uint32_t G, uint32_t C, float host_mem_gb, const float *best_thr,
                       const uint32_t *best_plan, const float *curve_thr, const uint8_t *state,
                       const int32_t *cur_seg, const uint32_t *cur_c, const int32_t *floor_seg,
                       const uint32_t *floor_c, ork_assign *assign, double *total, uint32_t *n_moves) {
    Loop L(n_jobs, ref_thr, tb, grid, G, best_thr, curve_thr, state, floor_seg, floor_c);
    std::vector<int64_t> &gi = L.gi;
    std::vector<uint32_t> &ci = L.ci;
    typedef Loop::Step Step;
    typedef Loop::Give Give;
    auto ns_of = [&](uint32_t j) { return L.ns_of(j); };
    auto g_at = [&](uint32_t j, int64_t s) { return L.g_at(j, s); };
    auto c_at = [&](uint32_t j, uint32_t c, int64_t s) { return L.c_at(j, c, s); };
    auto part = [&](uint32_t j) { return L.part(j); };
    auto fl_s = [&](uint32_t j) { return L.fl_s(j); };
    auto up_gpu = [&](uint32_t j) { return L.up_gpu(j); };
    auto up_cpu = [&](uint32_t j) { return L.up_cpu(j); };
    auto down_gpu = [&](uint32_t v) { return L.down_gpu(v); };
    auto down_cpu = [&](uint32_t v) { return L.down_cpu(v); };
    uint64_t heldG = 0, heldC = 0;
    for (uint32_t j = 0; j < n_jobs; ++j) {
        if (!L.holds(j) || cur_seg[j] < 0 || cur_seg[j] >= ns_of(j) || cur_c[j] >= grid->n_cpu) continue;
        gi[j] = cur_seg[j]; ci[j] = cur_c[j];
        heldG += g_at(j, gi[j]); heldC += c_at(j, ci[j], gi[j]);
    }
    uint64_t freeG = heldG < G ? G - heldG : 0, freeC = heldC < C ? C - heldC : 0;
    uint32_t moves = 0;

    auto schedule_job = [&](uint32_t j) {
        for (int res = 0; res < 2; ++res) {                 /* GPUs, then CPUs */
            for (;;) {
                const Step st = res == 0 ? up_gpu(j) : up_cpu(j);
                if (!st.any) break;
                const bool below_min = res == 0 && fl_s(j) >= 0 && gi[j] < fl_s(j);
                uint64_t availG = freeG, availC = freeC;
                std::vector<int64_t> keep_gi(gi);
                std::vector<uint32_t> keep_ci(ci);
                float lost = 0.0f;
                bool ok = true;
                while (res == 0 ? availG < st.dg : availC < st.dc) {
                    int64_t pick = -1; Give best = {false, -1, 0.0f, 0.0f, 0, 0};
                    for (uint32_t v = 0; v < n_jobs; ++v) {  /* GetLowestSlopeOverMinJob */
                        if (v == j || !part(v)) continue;
                        const Give gv = res == 0 ? down_gpu(v) : down_cpu(v);
                        if (!gv.any) continue;
                        if (pick < 0 || gv.slope < best.slope) { pick = v; best = gv; }
                    }
                    if (pick < 0 || !(below_min || st.slope > best.slope)) { ok = false; break; }
                    availG += best.dg; availC += best.dc; lost = lost + best.loss;
                    if (res == 0) { gi[pick] = best.tgt; if (best.tgt < 0) ci[pick] = 0; }
                    else ci[pick] -= 1;
                }
                if (ok && (availG < st.dg || availC < st.dc)) ok = false;
                if (ok && !below_min && !(st.gain > lost)) ok = false;
                if (!ok) { gi = keep_gi; ci = keep_ci; break; }
                freeG = availG - st.dg; freeC = availC - st.dc;
                if (res == 0) gi[j] = st.tgt;
                ci[j] = st.lvl;
                ++moves;
            }
        }
    };

    std::vector<uint8_t> first(n_jobs, 0);
    for (uint32_t j = 0; j < n_jobs; ++j)
        if (part(j) && fl_s(j) >= 0 && gi[j] < fl_s(j)) { first[j] = 1; schedule_job(j); }
    std::vector<uint32_t> order;
    std::vector<float> sg(n_jobs, 0.0f), sc(n_jobs, 0.0f);
    for (uint32_t j = 0; j < n_jobs; ++j)
        if (part(j) && !first[j]) { order.push_back(j); sg[j] = up_gpu(j).slope; sc[j] = up_cpu(j).slope; }
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        if (sg[a] != sg[b]) return sg[a] > sg[b];
        return sc[a] > sc[b];
    });
    for (uint32_t j : order) schedule_job(j);
    if (n_moves) *n_moves = moves;
    return memory_step(n_jobs, ref_thr, tb, grid, host_mem_gb, best_thr, best_plan, gi, ci, assign, total);
}

/* Algorithm 1 as printed: ScheduleJob searches the cluster node by node, and on each node the job to shrink is the one
 * with the lowest slope among the jobs on THAT node (GetLowestSlopeOverMinJob(n, resType)).  State, order, steps,
 * slopes, permit cases and commit rule are those of ork_reschedule_f32; what is new is where things are:
 *   - Every job that holds something has parts (node, GPUs), at most one per node, in ascending node order; they come
 *     in as an earlier placement (prev_off, prev_entries) and must add up to what the job holds.  The CPU levels must
 *     be CPUs per GPU (cpu_mode 1; otherwise -2): a part of k GPUs at level l holds cpu_levels[l] * k CPUs of its node.
 *   - A GPU step of job j walks the nodes in order.  On a node it first takes what is free (a GPU only together with
 *     its CPUs at the step's level), then, while it still lacks GPUs, asks for the job with the lowest slope among
 *     the other jobs with a part on this node that are above their own floor (lower index on ties); if that job may
 *     be shrunk (j's slope is higher, or j is below its floor) it steps down to its next useful amount, giving up
 *     GPUs of its part on this node first and, if its step is larger than that part, the rest from its other parts,
 *     the last one first (those become free where they are); j takes again.  No such job, or not permitted: next node.
 *     A step that raises the CPU level of a job that already holds parts (a step to a floor with a higher level)
 *     needs the additional CPUs of those parts free on their nodes.
 *   - A CPU step raises the level on every node the job is on: per node, what is free first, then the jobs on that
 *     node by lowest CPU slope, each giving one level (on all its nodes).
 *   - A step is committed when all of it was found and (unless j is below its floor) j gains more than the others
 *     lose; otherwise jobs and nodes are put back as they were and j's search in that resource ends.
 *   - Memory last, in job order: a tier costs every part its share (tier * k / g, float32) of its node's memory; among
 *     the tiers every part can pay, the highest throughput, the smallest such tier; none: the job is dropped.
 * Returns -1 when the state is not a placement on these nodes (parts that do not add up, a node that does not exist
 * or holds more than it has, parts out of order, CPUs that are not level * GPUs).
 * PARITY UNPINNED as a reading; pinned by the loop over totals (one node that holds the whole cluster), by hand cases
 * for every rule above and by invariants on generated rounds. */
int ork_reschedule_nodes_f32(uint32_t n_jobs, const float *ref_thr, const ork_table *tb, const ork_grid *grid,
                             uint32_t n_nodes, uint32_t gpus_per_node, uint32_t cpus_per_node, float mem_per_node_gb,
                             const float *best_thr, const uint32_t *best_plan, const float *curve_thr,
                             const uint8_t *state, const int32_t *cur_seg, const uint32_t *cur_c,
                             const int32_t *floor_seg, const uint32_t *floor_c, const uint32_t *prev_off,
                             const ork_place_entry *prev_entries, ork_assign *assign, uint32_t *place_off,
                             ork_place_entry *entries, double *total, uint32_t *n_moves) {
    if (grid->cpu_mode != 1) return -2;
    Loop L(n_jobs, ref_thr, tb, grid, (uint64_t)n_nodes * gpus_per_node, best_thr, curve_thr, state, floor_seg, floor_c);
    auto cpl = [&](uint32_t lvl) -> uint64_t { return grid->cpu_levels[lvl]; };
    /* where everything is: a job's parts (node -> GPUs), who is on a node, what a node has free */
    struct Where {
        std::vector<std::map<uint32_t, uint64_t>> parts;
        std::vector<std::set<uint32_t>> on_node;
        std::vector<uint64_t> freeG, freeC;
    } W;
    W.parts.resize(n_jobs); W.on_node.resize(n_nodes);
    W.freeG.assign(n_nodes, gpus_per_node); W.freeC.assign(n_nodes, cpus_per_node);
    auto add = [&](uint32_t j, uint32_t n, uint64_t k, uint64_t per_gpu) {          /* j gets k GPUs of node n */
        W.freeG[n] -= k; W.freeC[n] -= k * per_gpu;
        W.parts[j][n] += k; W.on_node[n].insert(j);
    };
    auto drop = [&](uint32_t v, uint32_t n, uint64_t k, uint64_t per_gpu) {         /* v gives k GPUs of node n back */
        W.freeG[n] += k; W.freeC[n] += k * per_gpu;
        if ((W.parts[v][n] -= k) == 0) { W.parts[v].erase(n); W.on_node[n].erase(v); }
    };

    for (uint32_t j = 0; j < n_jobs; ++j) {
        if (!L.holds(j) || cur_seg[j] < 0 || cur_seg[j] >= L.ns_of(j) || cur_c[j] >= grid->n_cpu) continue;
        L.gi[j] = cur_seg[j]; L.ci[j] = cur_c[j];
        if (!prev_off || !prev_entries) return -1;          /* a running job is somewhere */
        uint64_t sum = 0;
        int64_t last = -1;
        for (uint32_t i = prev_off[j]; i < prev_off[j + 1]; ++i) {
            const ork_place_entry &e = prev_entries[i];
            if (e.node >= n_nodes || (int64_t)e.node <= last || e.g == 0 || e.c != cpl(L.ci[j]) * e.g) return -1;
            if (e.g > W.freeG[e.node] || e.c > W.freeC[e.node]) return -1;
            add(j, e.node, e.g, cpl(L.ci[j]));
            last = e.node; sum += e.g;
        }
        if (sum != L.g_at(j, L.gi[j])) return -1;
    }
    uint32_t moves = 0;

    /* the most GPUs of node n that j can take now, up to what it lacks: a GPU comes with per_gpu CPUs */
    auto take = [&](uint32_t j, uint32_t n, uint64_t per_gpu, uint64_t &lack) {
        const uint64_t k = std::min(std::min(lack, W.freeG[n]), W.freeC[n] / per_gpu);
        if (k) { add(j, n, k, per_gpu); lack -= k; }
    };
    auto schedule_job = [&](uint32_t j) {
        for (;;) {                                          /* GPUs */
            const Loop::Step st = L.up_gpu(j);
            if (!st.any) break;
            const bool below_min = L.fl_s(j) >= 0 && L.gi[j] < L.fl_s(j);
            const Where keepW = W;
            const std::vector<int64_t> keep_gi(L.gi);
            const std::vector<uint32_t> keep_ci(L.ci);
            const uint64_t per_gpu = cpl(st.lvl);
            uint64_t lack = st.dg;
            float lost = 0.0f;
            bool ok = true;
            if (L.gi[j] >= 0 && st.lvl != L.ci[j]) {        /* its parts go to the step's level: their CPUs must be free */
                const uint64_t more = per_gpu - cpl(L.ci[j]);
                for (const auto &pk : W.parts[j]) {
                    if (W.freeC[pk.first] < more * pk.second) { ok = false; break; }
                    W.freeC[pk.first] -= more * pk.second;
                }
            }
            for (uint32_t n = 0; n < n_nodes && ok && lack > 0; ++n) {
                take(j, n, per_gpu, lack);
                while (lack > 0) {
                    int64_t pick = -1; Loop::Give best = {false, -1, 0.0f, 0.0f, 0, 0};
                    for (uint32_t v : W.on_node[n]) {       /* GetLowestSlopeOverMinJob(n, GPU); ascending index */
                        if (v == j || !L.part(v)) continue;
                        const Loop::Give gv = L.down_gpu(v);
                        if (!gv.any) continue;
                        if (pick < 0 || gv.slope < best.slope) { pick = v; best = gv; }
                    }
                    if (pick < 0 || !(below_min || st.slope > best.slope)) break;
                    const uint64_t per_v = cpl(L.ci[pick]);
                    uint64_t rest = best.dg;
                    const uint64_t here = std::min(rest, W.parts[pick][n]);
                    drop((uint32_t)pick, n, here, per_v); rest -= here;
                    while (rest > 0) {                      /* the rest from its other parts, the last one first */
                        auto it = W.parts[pick].end();
                        do { --it; } while (it->first == n);
                        const uint32_t m = it->first;
                        const uint64_t k = std::min(rest, it->second);
                        drop((uint32_t)pick, m, k, per_v); rest -= k;
                    }
                    lost = lost + best.loss;
                    L.gi[pick] = best.tgt; if (best.tgt < 0) L.ci[pick] = 0;
                    take(j, n, per_gpu, lack);
                }
            }
            if (ok && lack > 0) ok = false;
            if (ok && !below_min && !(st.gain > lost)) ok = false;
            if (!ok) { W = keepW; L.gi = keep_gi; L.ci = keep_ci; break; }
            L.gi[j] = st.tgt; L.ci[j] = st.lvl;
            ++moves;
        }
        for (;;) {                                          /* CPUs */
            const Loop::Step st = L.up_cpu(j);
            if (!st.any) break;
            const Where keepW = W;
            const std::vector<uint32_t> keep_ci(L.ci);
            const uint64_t more = cpl(st.lvl) - cpl(L.ci[j]);
            float lost = 0.0f;
            bool ok = true;
            for (const auto &pk : W.parts[j]) {
                const uint32_t n = pk.first;
                const uint64_t need = more * pk.second;
                while (ok && W.freeC[n] < need) {
                    int64_t pick = -1; Loop::Give best = {false, -1, 0.0f, 0.0f, 0, 0};
                    for (uint32_t v : W.on_node[n]) {       /* GetLowestSlopeOverMinJob(n, CPU) */
                        if (v == j || !L.part(v)) continue;
                        const Loop::Give gv = L.down_cpu(v);
                        if (!gv.any) continue;
                        if (pick < 0 || gv.slope < best.slope) { pick = v; best = gv; }
                    }
                    if (pick < 0 || !(st.slope > best.slope)) { ok = false; break; }
                    const uint64_t less = cpl(L.ci[pick]) - cpl(L.ci[pick] - 1);
                    for (const auto &qk : W.parts[pick]) W.freeC[qk.first] += less * qk.second;
                    L.ci[pick] -= 1;
                    lost = lost + best.loss;
                }
                if (!ok) break;
                W.freeC[n] -= need;
            }
            if (ok && !(st.gain > lost)) ok = false;
            if (!ok) { W = keepW; L.ci = keep_ci; break; }
            L.ci[j] = st.lvl;
            ++moves;
        }
    };

    std::vector<uint8_t> first(n_jobs, 0);
    for (uint32_t j = 0; j < n_jobs; ++j)
        if (L.part(j) && L.fl_s(j) >= 0 && L.gi[j] < L.fl_s(j)) { first[j] = 1; schedule_job(j); }
    std::vector<uint32_t> order;
    std::vector<float> sg(n_jobs, 0.0f), sc(n_jobs, 0.0f);
    for (uint32_t j = 0; j < n_jobs; ++j)
        if (L.part(j) && !first[j]) { order.push_back(j); sg[j] = L.up_gpu(j).slope; sc[j] = L.up_cpu(j).slope; }
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        if (sg[a] != sg[b]) return sg[a] > sg[b];
        return sc[a] > sc[b];
    });
    for (uint32_t j : order) schedule_job(j);
    if (n_moves) *n_moves = moves;

    /* memory, then the records */
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    std::vector<float> freeM(n_nodes, mem_per_node_gb);
    uint32_t n_entries = 0;
    double sum = 0.0;
    for (uint32_t j = 0; j < n_jobs; ++j) {
        place_off[j] = n_entries;
        assign[j] = ork_assign{0, 0, 0.0f, ORK_NO_PLAN, 0.0f};
        if (L.gi[j] < 0) continue;
        const uint64_t ns = L.ns_of(j);
        const uint32_t g = (uint32_t)L.g_at(j, L.gi[j]);
        float bv = 0.0f; int64_t bm = -1;
        for (uint32_t m = 0; m < grid->n_mem; ++m) {
            bool fits = true;
            for (const auto &pk : W.parts[j])
                if (!((tier_gb(grid, m, g) * (float)pk.second) / (float)g <= freeM[pk.first])) fits = false;
            if (!fits) continue;
            const float v = best_thr[rows * tb->seg_off[j] + ((uint64_t)L.ci[j] * grid->n_mem + m) * ns + L.gi[j]];
            if (v > bv) { bv = v; bm = m; }
        }
        if (bm < 0) continue;
        const float cost = tier_gb(grid, (uint32_t)bm, g);
        for (const auto &pk : W.parts[j]) {
            ork_place_entry e;
            e.node = pk.first; e.g = (uint32_t)pk.second; e.c = (uint32_t)(cpl(L.ci[j]) * pk.second);
            e.mem_gb = (cost * (float)pk.second) / (float)g;
            freeM[e.node] = freeM[e.node] - e.mem_gb;
            entries[n_entries++] = e;
        }
        assign[j].g = g; assign[j].c = cpus_of(grid, L.ci[j], g); assign[j].mem_gb = cost;
        assign[j].plan = best_plan[rows * tb->seg_off[j] + ((uint64_t)L.ci[j] * grid->n_mem + bm) * ns + L.gi[j]];
        assign[j].thr = bv;
        sum += (double)bv / (double)ref_thr[j];
    }
    place_off[n_jobs] = n_entries;
    if (total) *total = sum;
    return 0;
}

/* Who is privileged when Schedule runs from a running state (Sec. 5.2, "Scheduling algorithm design": the guaranteed
 * jobs whose demands are within their tenant's remaining quota are scheduled first; the quota usage of a job is its
 * minimum demand): the floors and states the loop takes.
 *   - A guaranteed job that holds something keeps taking part; its minimum demand (min_seg, min_c as ork_min_res_f32
 *     gives them; none when min_seg is not an index of its list or its tenant is unknown) is its floor and is charged
 *     to its tenant's quota before any queued job is looked at (a quota cannot go below zero).
 *   - Queued guaranteed jobs, in job order: a job whose minimum demand (GPUs, CPUs) fits what is left of its tenant's
 *     quota gets it as its floor - the loop then serves it first - and charges the quota; a job that does not fit, or
 *     has no minimum demand, waits: state 1.
 *   - Best-effort jobs have no floor.  A job whose state says it takes no part keeps that state and charges nothing.
 * PARITY UNPINNED as a reading; pinned by hand cases and, from an empty cluster, by the privileged phase of the
 * allocation from scratch (ork_policy_f32) when capacity is plentiful. */
int ork_privileged(uint32_t n_jobs, const ork_table *tb, const ork_grid *grid, const uint32_t *guaranteed,
                   const uint32_t *tenant, const int32_t *min_seg, const uint32_t *min_c, uint32_t n_tenants,
                   const uint32_t *quota_g, const uint32_t *quota_c, const uint8_t *state_in, const int32_t *cur_seg,
                   const uint32_t *cur_c, int32_t *floor_seg, uint32_t *floor_c, uint8_t *state_out) {
    std::vector<uint64_t> qg(quota_g, quota_g + n_tenants), qc(quota_c, quota_c + n_tenants);
    auto ns_of = [&](uint32_t j) { return (int64_t)(tb->seg_off[j + 1] - tb->seg_off[j]); };
    auto has_min = [&](uint32_t j) { return min_seg[j] >= 0 && min_seg[j] < ns_of(j) && tenant[j] < n_tenants; };
    auto demand = [&](uint32_t j, uint64_t &g, uint64_t &c) {
        g = tb->seg_g[tb->seg_off[j] + min_seg[j]];
        c = cpus_of(grid, std::min(min_c[j], grid->n_cpu - 1), (uint32_t)g);
    };
    auto holds = [&](uint32_t j) {
        const bool in = !state_in || state_in[j] == 0 || state_in[j] == 2;
        return in && cur_seg[j] >= 0 && cur_seg[j] < ns_of(j) && cur_c[j] < grid->n_cpu;
    };
    for (uint32_t j = 0; j < n_jobs; ++j) {
        floor_seg[j] = -1; floor_c[j] = 0;
        state_out[j] = state_in ? state_in[j] : 0;
        if (!guaranteed[j] || !holds(j) || !has_min(j)) continue;
        uint64_t g, c;
        demand(j, g, c);
        floor_seg[j] = min_seg[j]; floor_c[j] = std::min(min_c[j], grid->n_cpu - 1);
        qg[tenant[j]] -= std::min(qg[tenant[j]], g);
        qc[tenant[j]] -= std::min(qc[tenant[j]], c);
    }
    for (uint32_t j = 0; j < n_jobs; ++j) {
        if (!guaranteed[j] || holds(j) || state_out[j] != 0) continue;
        uint64_t g = 0, c = 0;
        if (has_min(j)) demand(j, g, c);
        if (has_min(j) && g <= qg[tenant[j]] && c <= qc[tenant[j]]) {
            floor_seg[j] = min_seg[j]; floor_c[j] = std::min(min_c[j], grid->n_cpu - 1);
            qg[tenant[j]] -= g; qc[tenant[j]] -= c;
        } else {
            state_out[j] = 1;
        }
    }
    return 0;
}

/* Slopes of the resource sensitivity curves (Sec. 5.2: the slope of a job's curve, per resource type, is the
 * throughput change per unit of the resource; Fig. 6).  A table of the steps the allocation rules take, for every
 * row (CPU level, memory tier) and GPU count of a job, cluster-independent:
 *   GPUs: from count s (or from nothing) to the larger count s' with the highest float32 slope
 *         ((curve(s') - curve(s)) / ref_thr) / (g(s') - g(s)), the smaller count among equal slopes; none: 0, -1.
 *   CPUs: at count s from level c to the level c' > c with the highest ((best(c') - best(c)) / ref_thr) / (CPUs(c') -
 *         CPUs(c)), the lower level among equals; none: 0, n_cpu.
 * Arrays in segment layout of jobs [jb, je) ([job][level][tier][count]); from0_* per job and row.
 * Pinned: hand values, concave curves (the next count, slopes falling), and the steps of the Schedule loop for a lone
 * job on a large empty cluster, which walk exactly this table. */
int ork_curve_slopes(const float *ref_thr, const ork_table *tb, const ork_grid *grid, uint32_t jb, uint32_t je,
                     const float *best_thr, const float *curve_thr, float *gpu_slope, int32_t *gpu_next,
                     float *from0_slope, int32_t *from0_next, float *cpu_slope, uint32_t *cpu_next) {
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    for (uint32_t j = jb; j < je; ++j) {
        const uint32_t s0 = tb->seg_off[j], ns = tb->seg_off[j + 1] - s0;
        const uint64_t base = rows * (s0 - tb->seg_off[jb]);
        for (uint32_t ci = 0; ci < grid->n_cpu; ++ci)
            for (uint32_t mi = 0; mi < grid->n_mem; ++mi) {
                const uint64_t row = base + ((uint64_t)ci * grid->n_mem + mi) * ns;
                for (int64_t s = -1; s < (int64_t)ns; ++s) {
                    const float cur = s < 0 ? 0.0f : curve_thr[row + s];
                    const uint32_t g = s < 0 ? 0u : tb->seg_g[s0 + s];
                    float top = 0.0f; int32_t nxt = -1;
                    for (uint32_t t = (uint32_t)(s + 1); t < ns; ++t) {
                        const float v = curve_thr[row + t];
                        if (!(v > cur)) continue;
                        float sl = (v - cur) / ref_thr[j];
                        sl = sl / (float)(tb->seg_g[s0 + t] - g);
                        if (sl > top) { top = sl; nxt = (int32_t)t; }
                    }
                    if (s < 0) {
                        from0_slope[rows * (j - jb) + (uint64_t)ci * grid->n_mem + mi] = top;
                        from0_next[rows * (j - jb) + (uint64_t)ci * grid->n_mem + mi] = nxt;
                    } else {
                        gpu_slope[row + s] = top; gpu_next[row + s] = nxt;
                    }
                }
                for (uint32_t s = 0; s < ns; ++s) {
                    const float cur = best_thr[row + s];
                    const uint32_t g = tb->seg_g[s0 + s];
                    float top = 0.0f; uint32_t nxt = grid->n_cpu;
                    for (uint32_t c = ci + 1; c < grid->n_cpu; ++c) {
                        const float v = best_thr[base + ((uint64_t)c * grid->n_mem + mi) * ns + s];
                        if (!(v > cur)) continue;
                        float sl = (v - cur) / ref_thr[j];
                        sl = sl / (float)(cpus_of(grid, c, g) - cpus_of(grid, ci, g));
                        if (sl > top) { top = sl; nxt = c; }
                    }
                    cpu_slope[row + s] = top; cpu_next[row + s] = nxt;
                }
            }
    }
    return 0;
}

}  // extern "C"

namespace {

/* The greedy proper, from a starting state: gi/ci = what every job holds
 * already, skip != 0 = the job neither gains GPUs nor CPUs in this round. */
int greedy_from(uint32_t n_jobs, const float *ref_thr, const ork_table *tb, const ork_grid *grid,
                uint64_t freeG, uint64_t freeC, float host_mem_gb, const float *best_thr,
                const uint32_t *best_plan, const float *curve_thr, std::vector<int64_t> &gi,
                std::vector<uint32_t> &ci, const std::vector<uint8_t> &waits, ork_assign *assign,
                double *total, double *min_gap) {
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    const uint32_t m_top = grid->n_mem - 1;
    double gap_min = INFINITY;

    auto ns_of = [&](uint32_t j) { return (uint64_t)(tb->seg_off[j + 1] - tb->seg_off[j]); };
    auto g_of = [&](uint32_t j, int64_t s) -> uint64_t { return s < 0 ? 0 : tb->seg_g[tb->seg_off[j] + s]; };
    auto at = [&](const float *arr, uint32_t j, uint32_t c, uint32_t m, uint64_t s) {
        return arr[rows * tb->seg_off[j] + ((uint64_t)c * grid->n_mem + m) * ns_of(j) + s];
    };
    auto cpu_cost = [&](uint32_t j, uint32_t c, int64_t s) -> uint64_t {
        return s < 0 ? 0 : cpus_of(grid, c, (uint32_t)g_of(j, s));
    };
    auto note_gap = [&](float win, float second) {
        if (second > 0.0f) { double gp = ((double)win - second) / win; if (gp < gap_min) gap_min = gp; }
    };

    /* GPU pass */
    for (;;) {
        float top = 0.0f, second = 0.0f; uint32_t tj = 0; int64_t ts = -1;
        for (uint32_t j = 0; j < n_jobs; ++j) {
            if (waits[j]) continue;
            const float cur = gi[j] < 0 ? 0.0f : at(curve_thr, j, ci[j], m_top, gi[j]);
            for (int64_t s = gi[j] + 1; s < (int64_t)ns_of(j); ++s) {
                const uint64_t dg = g_of(j, s) - g_of(j, gi[j]);
                if (dg > freeG) break;
                const float v = at(curve_thr, j, ci[j], m_top, s);
                if (!(v > cur)) continue;
                const uint64_t dc = cpu_cost(j, ci[j], s) - cpu_cost(j, ci[j], gi[j]);
                if (dc > freeC) continue;
                float sl = (v - cur) / ref_thr[j];
                sl = sl / (float)dg;
                if (sl > top) { second = top; top = sl; tj = j; ts = s; }
                else if (sl > second) second = sl;
            }
        }
        if (ts < 0) break;
        note_gap(top, second);
        freeG -= g_of(tj, ts) - g_of(tj, gi[tj]);
        freeC -= cpu_cost(tj, ci[tj], ts) - cpu_cost(tj, ci[tj], gi[tj]);
        gi[tj] = ts;
    }
    /* CPU pass */
    for (;;) {
        float top = 0.0f, second = 0.0f; uint32_t tj = 0; int64_t tc = -1;
        for (uint32_t j = 0; j < n_jobs; ++j) {
            if (gi[j] < 0 || waits[j]) continue;
            const float cur = at(best_thr, j, ci[j], m_top, gi[j]);
            for (uint32_t c = ci[j] + 1; c < grid->n_cpu; ++c) {
                const uint64_t dc = cpu_cost(j, c, gi[j]) - cpu_cost(j, ci[j], gi[j]);
                if (dc > freeC) break;
                const float v = at(best_thr, j, c, m_top, gi[j]);
                if (!(v > cur)) continue;
                float sl = (v - cur) / ref_thr[j];
                sl = sl / (float)dc;
                if (sl > top) { second = top; top = sl; tj = j; tc = c; }
                else if (sl > second) second = sl;
            }
        }
        if (tc < 0) break;
        note_gap(top, second);
        freeC -= cpu_cost(tj, (uint32_t)tc, gi[tj]) - cpu_cost(tj, ci[tj], gi[tj]);
        ci[tj] = (uint32_t)tc;
    }
    if (min_gap) *min_gap = gap_min;
    return memory_step(n_jobs, ref_thr, tb, grid, host_mem_gb, best_thr, best_plan, gi, ci, assign, total);
}

/* Memory, then output (Sec. 5.2: memory is allocated last, from the chosen plan's estimate): in job order, among the
 * tiers that still fit, the one with the highest throughput (smallest such tier); none feasible: the job is dropped. */
int memory_step(uint32_t n_jobs, const float *ref_thr, const ork_table *tb, const ork_grid *grid, float host_mem_gb,
                const float *best_thr, const uint32_t *best_plan, const std::vector<int64_t> &gi,
                const std::vector<uint32_t> &ci, ork_assign *assign, double *total) {
    const uint64_t rows = (uint64_t)grid->n_cpu * grid->n_mem;
    float freeM = host_mem_gb;
    double sum = 0.0;
    for (uint32_t j = 0; j < n_jobs; ++j) {
        ork_assign out = {0, 0, 0.0f, ORK_NO_PLAN, 0.0f};
        if (gi[j] >= 0) {
            const uint64_t ns = tb->seg_off[j + 1] - tb->seg_off[j];
            const uint32_t g = tb->seg_g[tb->seg_off[j] + gi[j]];
            float bv = 0.0f; int64_t bm = -1;
            for (uint32_t m = 0; m < grid->n_mem; ++m) {
                if (!(tier_gb(grid, m, g) <= freeM)) continue;
                const float v = best_thr[rows * tb->seg_off[j] + ((uint64_t)ci[j] * grid->n_mem + m) * ns + gi[j]];
                if (v > bv) { bv = v; bm = m; }
            }
            if (bm >= 0) {
                const float cost = tier_gb(grid, (uint32_t)bm, g);
                freeM = freeM - cost;
                out.g = g; out.c = cpus_of(grid, ci[j], g); out.mem_gb = cost;
                out.plan = best_plan[rows * tb->seg_off[j] + ((uint64_t)ci[j] * grid->n_mem + bm) * ns + gi[j]];
                out.thr = bv;
                sum += (double)bv / (double)ref_thr[j];
            }
        }
        assign[j] = out;
    }
    if (total) *total = sum;
    return 0;
}

}  // namespace
