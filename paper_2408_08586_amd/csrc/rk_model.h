// Device-side performance model (paper Sec. 4): everything a kernel needs to
// turn (job, triple, option, CPUs, memory tier) into a throughput and a
// feasibility verdict.  float32 throughout.  Both the materialising kernel and
// the fused kernel build their values from these functions only, so the two
// produce bit-identical numbers.
//
// The translation units are compiled with -ffp-contract=off: every written
// operation rounds once, which the memory estimate relies on (its verdicts
// must not depend on instruction selection).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "rubick.h"

struct JobDev {   // rk_jobs with restrict-qualified members
    const float *__restrict__ P_bytes, *__restrict__ seq, *__restrict__ hidden, *__restrict__ elem_bytes,
        *__restrict__ t_fwd_sample, *__restrict__ k_bwd, *__restrict__ k_sync, *__restrict__ k_opt,
        *__restrict__ k_opt_off, *__restrict__ k_off, *__restrict__ k_swap, *__restrict__ k_const,
        *__restrict__ mem_state, *__restrict__ mem_act, *__restrict__ mem_act_gc, *__restrict__ mem_const;
    const uint32_t *__restrict__ layers, *__restrict__ gbatch, *__restrict__ mbatch;
};

static inline JobDev job_dev(const rk_jobs *j) {
    return JobDev{j->P_bytes, j->seq, j->hidden, j->elem_bytes, j->t_fwd_sample, j->k_bwd, j->k_sync,
                  j->k_opt, j->k_opt_off, j->k_off, j->k_swap, j->k_const, j->mem_state, j->mem_act,
                  j->mem_act_gc, j->mem_const, j->layers, j->gbatch, j->mbatch};
}

struct GridDev {
    uint32_t n_cpu, cpu_mode, n_mem, mem_mode;
    uint32_t cpu_levels[RK_MAX_CPU_LEVELS];
    float mem_levels_gb[RK_MAX_MEM_LEVELS];
};

static inline GridDev grid_dev(const rk_alloc_grid *g) {
    GridDev d;
    d.n_cpu = g->n_cpu; d.cpu_mode = g->cpu_mode; d.n_mem = g->n_mem; d.mem_mode = g->mem_mode;
    for (int i = 0; i < RK_MAX_CPU_LEVELS; ++i) d.cpu_levels[i] = i < (int)g->n_cpu ? g->cpu_levels[i] : 0;
    for (int i = 0; i < RK_MAX_MEM_LEVELS; ++i) d.mem_levels_gb[i] = i < (int)g->n_mem ? g->mem_levels_gb[i] : 0.f;
    return d;
}

struct Job {      // one job's coefficients in registers
    float P, seq, hidden, eb, tfs, k_bwd, k_sync, k_opt, k_opt_off, k_off, k_swap, k_const;
    float m_state, m_act, m_act_gc, m_const;
    uint32_t layers, gbatch, mbatch;
};

__device__ __forceinline__ Job load_job(const JobDev &J, uint32_t j) {
    Job o;
    o.P = J.P_bytes[j]; o.seq = J.seq[j]; o.hidden = J.hidden[j]; o.eb = J.elem_bytes[j];
    o.tfs = J.t_fwd_sample[j]; o.k_bwd = J.k_bwd[j]; o.k_sync = J.k_sync[j]; o.k_opt = J.k_opt[j];
    o.k_opt_off = J.k_opt_off[j]; o.k_off = J.k_off[j]; o.k_swap = J.k_swap[j]; o.k_const = J.k_const[j];
    o.m_state = J.mem_state[j]; o.m_act = J.mem_act[j]; o.m_act_gc = J.mem_act_gc[j]; o.m_const = J.mem_const[j];
    o.layers = J.layers[j]; o.gbatch = J.gbatch[j]; o.mbatch = J.mbatch[j];
    return o;
}

__device__ __forceinline__ float fast_div(float a, float b) { return a * __builtin_amdgcn_rcpf(b); }

// Overlap of two stages (Sec. 4.3): (x^k + y^k)^(1/k), evaluated as
// M * 2^(log2(1 + r^k)/k) with M = max, r = min/max in [0,1], which neither
// overflows nor loses the small term.  inv_k = 1/k.
__device__ __forceinline__ float f_overlap(float k, float inv_k, float x, float y) {
    const float M = fmaxf(x, y), m = fminf(x, y);
    if (!(m > 0.f)) return M;
    const float r = fast_div(m, M);
    const float u = __builtin_amdgcn_exp2f(k * __builtin_amdgcn_logf(r));
    return M * __builtin_amdgcn_exp2f(__builtin_amdgcn_logf(1.f + u) * inv_k);
}

// Terms of a (job, triple) that do not depend on the option, CPUs or memory.
struct Triple {
    uint32_t d, t, p, g;
    float fd;
    float Tcc[2];        // computation + communication, by gc (Sec. 4.1)
    float Tdp;           // gradient synchronisation time
    float Psi;           // parameter bytes on one model-parallel shard
    float A[2];          // activation bytes by gc
    float b;             // global batch
};

// Bandwidths of the three kinds of communication groups.
struct Links { float dp, tp, pp; };

// Bottleneck bandwidths under a packed placement (TP ranks adjacent, then DP, then PP stages; the job starts at
// a node boundary and fills whole nodes): inside one node everything is intra-node; over several nodes a kind of
// group stays on the intra-node links only when whole groups tile a node.
__device__ __forceinline__ Links packed_links(const rk_env &E, uint32_t d, uint32_t t, uint32_t g) {
    const uint32_t N = E.gpus_per_node;
    Links L = {E.B_intra, E.B_intra, E.B_intra};
    if (g > N) {
        L.tp = (N % t == 0) ? E.B_intra : E.B_inter;
        L.dp = (N % (t * d) == 0) ? E.B_intra : E.B_inter;
        L.pp = E.B_inter;
    }
    return L;
}

// The same for a job whose nodes are known: edge_gcd = greatest common divisor of the GPU counts at which the
// job's slots cross from one node to the next (0 when it sits on one node).  Groups of w adjacent ranks all lie
// inside a node exactly when w divides every such count: w = t for tensor parallelism, t*d for data parallelism
// (its groups interleave over a whole pipeline stage); pipeline neighbours share a node only when the job does.
__device__ __forceinline__ Links placed_links(const rk_env &E, uint32_t d, uint32_t t, uint32_t edge_gcd) {
    Links L;
    L.tp = (edge_gcd % t == 0) ? E.B_intra : E.B_inter;
    L.dp = (edge_gcd % (t * d) == 0) ? E.B_intra : E.B_inter;
    L.pp = edge_gcd == 0 ? E.B_intra : E.B_inter;
    return L;
}

template <bool PLACED>
__device__ __forceinline__ Triple triple_terms_on(const Job &J, const rk_env &E, uint32_t packed, uint32_t edge_gcd) {
    Triple T;
    T.d = RK_TRIPLE_D(packed); T.t = RK_TRIPLE_T(packed); T.p = RK_TRIPLE_P(packed);
    T.g = T.d * T.t * T.p;
    const float fd = (float)T.d, ft = (float)T.t, fp = (float)T.p, ftp = (float)(T.t * T.p);
    T.fd = fd;
    T.b = (float)J.gbatch;
    const uint32_t mb = J.mbatch << RK_TRIPLE_V(packed);     // micro-batch size of this plan
    const uint32_t n = J.gbatch / (T.d * mb);                // micro-batches per replica
    const float fn = (float)n;
    const float fmu = (float)mb;

    // forward / backward of the pipeline fill + steady state, or of one accumulation step
    const float Tf_mb = fast_div(J.tfs * fmu, ftp);
    const float m = T.p > 1 ? fn : 1.f, a = T.p > 1 ? 1.f : fn;
    const float Tfwd = Tf_mb * (m + fp - 1.f);
    const float Tbwd0 = J.k_bwd * Tfwd;
    const float Tbwd1 = Tbwd0 + Tfwd;                        // checkpointing recomputes a forward

    const Links L = PLACED ? placed_links(E, T.d, T.t, edge_gcd) : packed_links(E, T.d, T.t, T.g);
    const float Bdp = L.dp, Btp = L.tp, Bpp = L.pp;
    const float bsh = (T.b * J.seq) * J.hidden;
    const float dt = fd * ft;
    T.Tdp = T.d > 1 ? fast_div(J.P * (2.f * (fd - 1.f)), (fd * ftp) * Bdp) : 0.f;
    const float Ttp = T.t > 1 ? fast_div(((J.eb * 8.f) * (ft - 1.f)) * (bsh * (float)J.layers), dt * Btp) : 0.f;
    const float Tpp = T.p > 1 ? fast_div(((J.eb * 2.f) * fp) * bsh, dt * Bpp) : 0.f;

    const float inv_ks = __builtin_amdgcn_rcpf(J.k_sync);
    const float sync0 = f_overlap(J.k_sync, inv_ks, Tbwd0, T.Tdp);
    const float sync1 = f_overlap(J.k_sync, inv_ks, Tbwd1, T.Tdp);
    if (T.p > 1) {
        const float c = Tfwd + Ttp + Tpp;
        T.Tcc[0] = c + sync0;
        T.Tcc[1] = c + sync1;
    } else {
        const float c = a * Tfwd + Ttp;
        T.Tcc[0] = c + (a - 1.f) * Tbwd0 + sync0;
        T.Tcc[1] = c + (a - 1.f) * Tbwd1 + sync1;
    }

    // memory: exact float32 sequence (documented in rubick.h)
    T.Psi = J.P / ftp;
    const uint32_t w = T.p < n ? T.p : n;
    float tok = fmu * J.seq;
    tok = tok * J.hidden;
    const float lay = (float)(J.layers / T.p);
    float base = tok * lay;
    base = base / ft;
    base = base * (float)w;
    T.A[0] = J.m_act * base;
    float a1 = J.m_act_gc * base;
    float a2 = J.m_act * tok;
    a2 = a2 / ft;
    T.A[1] = a1 + a2;
    return T;
}

// terms of a triple under the packed placement every candidate is evaluated with
__device__ __forceinline__ Triple triple_terms(const Job &J, const rk_env &E, uint32_t packed) {
    return triple_terms_on<false>(J, E, packed, 0u);
}

// GPU-memory verdict of a plan: true if it fits.
__device__ __forceinline__ bool gpu_mem_fits(const Job &J, const rk_env &E, const Triple &T,
                                             uint32_t z, uint32_t gc, uint32_t off) {
    float kappa;
    if (off) {
        kappa = (z == 2) ? 1.0f : 1.0f / T.fd;
    } else if (z == 0) {
        kappa = 8.0f;
    } else if (z == 1) {
        float q = 6.0f / T.fd; kappa = 2.0f + q;
    } else if (z == 2) {
        float q = 7.0f / T.fd; kappa = 1.0f + q;
    } else {
        kappa = 8.0f / T.fd;
    }
    float sk = J.m_state * kappa;
    float S = sk * T.Psi;
    float M = S + T.A[gc];
    M = M + J.m_const;
    return M <= E.gpu_mem_cap;
}

// Host bytes an offload plan needs (all GPUs of the job together).
__device__ __forceinline__ float host_bytes_needed(const Job &J, const Triple &T) {
    float q = 7.0f / T.fd;
    float h = J.m_state * q;
    h = h * T.Psi;
    h = h * (float)T.g;
    return h;
}

__device__ __forceinline__ float tier_bytes(const GridDev &G, uint32_t mi, uint32_t g) {
    float v = G.mem_levels_gb[mi] * 1073741824.0f;
    if (G.mem_mode) v = v * (float)g;
    return v;
}

// GiB a job of g GPUs books at memory tier mi
__device__ __forceinline__ float tier_gib(const GridDev &G, uint32_t mi, uint32_t g) {
    float v = G.mem_levels_gb[mi];
    if (G.mem_mode) v = v * (float)g;
    return v;
}

__device__ __forceinline__ uint32_t cpus_of(const GridDev &G, uint32_t ci, uint32_t g) {
    return G.cpu_mode ? G.cpu_levels[ci] * g : G.cpu_levels[ci];
}

// Throughput of a plan without offload (Eq. 1 with T_oo = T_opt).
__device__ __forceinline__ float thr_plain(const Job &J, const Triple &T, uint32_t z, uint32_t gc) {
    const float Topt = z ? fast_div(J.k_opt * T.Psi, T.fd) : J.k_opt * T.Psi;
    return fast_div(T.b, (T.Tcc[gc] + Topt) + J.k_const);
}

// Offload plans: the part of T_iter that does not depend on the CPUs ...
struct Offload {
    float base[2];       // T_cc + f(k_off; T_dp, T_off) + k_const, by gc
    float topt_num;      // k_opt_off * Psi / d ; T_opt = topt_num / c
    float Toff;
    float inv_kswap;
};

__device__ __forceinline__ Offload offload_terms(const Job &J, const rk_env &E, const Triple &T) {
    Offload O;
    O.Toff = fast_div(T.Psi, T.fd * E.B_pcie);
    const float foff = f_overlap(J.k_off, __builtin_amdgcn_rcpf(J.k_off), T.Tdp, O.Toff);
    O.base[0] = (T.Tcc[0] + foff) + J.k_const;
    O.base[1] = (T.Tcc[1] + foff) + J.k_const;
    O.topt_num = fast_div(J.k_opt_off * T.Psi, T.fd);
    O.inv_kswap = __builtin_amdgcn_rcpf(J.k_swap);
    return O;
}

// ... and the CPU-dependent part f(k_swap; T_opt(c), T_off).
__device__ __forceinline__ float swap_term(const Job &J, const Offload &O, uint32_t c) {
    return f_overlap(J.k_swap, O.inv_kswap, fast_div(O.topt_num, (float)c), O.Toff);
}

__device__ __forceinline__ float thr_offload(const Triple &T, const Offload &O, uint32_t gc, float swap) {
    return fast_div(T.b, O.base[gc] + swap);
}

// packed comparison key: larger throughput wins, then the lower plan index
__device__ __forceinline__ unsigned long long make_key(float thr, uint32_t plan) {
    return ((unsigned long long)__float_as_uint(thr) << 32) | (unsigned long long)(~plan);
}
__device__ __forceinline__ float key_thr(unsigned long long k) { return __uint_as_float((uint32_t)(k >> 32)); }
__device__ __forceinline__ uint32_t key_plan(unsigned long long k) {
    return (k >> 32) ? ~(uint32_t)k : RK_NO_PLAN;
}
