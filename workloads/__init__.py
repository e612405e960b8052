"""Seeded synthetic scheduling workloads (job descriptors, allocation grids, clusters).

This module is the only code shared by the CPU oracle and the HIP path: it
draws numbers and fills arrays, and contains none of the performance model's
arithmetic.  Every draw is a pure function of (seed, config, round, job, field)
through a counter-based generator (splitmix64 finaliser), so any job of any
configuration can be regenerated in isolation.

The five configurations stand in for the workload shapes of the paper's
evaluation (Sec. 7: seven Transformer models of 86M-30B parameters, a cluster
of 8 servers x 8 GPUs, a 406-job trace): only the shapes are used; no fitted
coefficient, trace record or dataset item is reproduced.

Job descriptor layout (Table 1 of the paper defines the symbols):
  coef  float32 [n_jobs, 17], columns COEF_FIELDS
  ints  uint32  [n_jobs, 3],  columns INT_FIELDS
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 0x52554249

COEF_FIELDS = (
    "P_bytes", "seq", "hidden", "elem_bytes", "t_fwd_sample",
    "k_bwd", "k_sync", "k_opt", "k_opt_off", "k_off", "k_swap", "k_const",
    "mem_state", "mem_act", "mem_act_gc", "mem_const", "ref_thr",
)
INT_FIELDS = ("layers", "gbatch", "mbatch")
N_COEF = len(COEF_FIELDS)
N_INT = len(INT_FIELDS)

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)


def _mix(x: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array."""
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        x = x ^ (x >> np.uint64(31))
    return x


def _key(seed: int, *parts) -> np.ndarray:
    """Chain (seed, part0, part1, ...) into one uint64 per broadcast element."""
    x = np.asarray(np.uint64(seed & 0xFFFFFFFFFFFFFFFF))
    with np.errstate(over="ignore"):
        for v in parts:
            v = np.asarray(v).astype(np.uint64)
            x = _mix(x + _GOLDEN * (v + np.uint64(1)))
    return x


def uniform(seed: int, *parts) -> np.ndarray:
    """U[0,1) double, one per broadcast element of `parts`."""
    return (_key(seed, *parts) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


@dataclass
class Grid:
    """Allocation grid: CPU levels and host-memory tiers (per job or per GPU)."""
    cpu_levels: np.ndarray           # uint32 [n_cpu], ascending, >= 1
    cpu_mode: int                    # 0: CPUs of the whole job; 1: CPUs per GPU
    mem_levels_gb: np.ndarray        # float32 [n_mem], ascending
    mem_mode: int                    # 0: GB for the whole job; 1: GB per GPU


@dataclass
class Env:
    B_intra: float = 400e9           # bytes/s, links inside a node
    B_inter: float = 100e9           # bytes/s, links between nodes
    B_pcie: float = 32e9             # bytes/s, GPU <-> host
    gpu_mem_cap: float = 80e9        # bytes
    gpus_per_node: int = 8


@dataclass
class Bounds:
    g_max: int
    tp_max: int = 8
    pp_max: int = 255
    zero_mask: int = 0xF             # bit z set: ZeRO stage z allowed
    gc_mask: int = 0x3               # bit v set: gradient checkpointing == v allowed
    off_mask: int = 0x3              # bit v set: offload == v allowed
    mu_mask: int = 0x1               # bit v set: micro-batches of mu * 2^v samples allowed (1 = the job's own mu only)


@dataclass
class Cluster:
    G: int
    C: int
    host_mem_gb: float


@dataclass
class Workload:
    name: str
    coef: np.ndarray                 # float32 [J, 17]
    ints: np.ndarray                 # uint32 [J, 3]
    bounds: Bounds
    grid: Grid
    env: Env
    cluster: Cluster
    meta: dict = field(default_factory=dict)

    @property
    def n_jobs(self) -> int:
        return int(self.coef.shape[0])

    def subset(self, idx) -> "Workload":
        idx = np.asarray(idx)
        return Workload(self.name + "[subset]", np.ascontiguousarray(self.coef[idx]),
                        np.ascontiguousarray(self.ints[idx]), self.bounds, self.grid,
                        self.env, self.cluster, dict(self.meta))


# field ids for the counter-based generator
_F_PARAMS, _F_BUCKET, _F_LAYERS, _F_BATCH, _F_MBATCH = 0, 1, 2, 3, 4
_F_COEF0 = 16                         # + column index of COEF_FIELDS


def _log_uniform(u, lo, hi):
    return np.exp(np.log(lo) + u * (np.log(hi) - np.log(lo)))


def draw_jobs(seed: int, config: int, rnd, job_ids, *, param_buckets, layer_choices,
              batch_choices=(32, 64, 128), mbatch_choices=(1, 2, 4), seq=2048):
    """Draw job descriptors.

    param_buckets: list of (probability, lo, hi) for the parameter count N
    (log-uniform inside a bucket).  `rnd` may be a scalar or an array aligned
    with job_ids (the round whose stream a job is drawn from).
    """
    job_ids = np.asarray(job_ids, dtype=np.uint64)
    rnd = np.broadcast_to(np.asarray(rnd, dtype=np.uint64), job_ids.shape)
    J = job_ids.shape[0]

    def u(fld):
        return uniform(seed, config, rnd, job_ids, fld)

    # parameter count
    ub = u(_F_BUCKET)
    un = u(_F_PARAMS)
    N = np.zeros(J)
    acc = 0.0
    chosen = np.zeros(J, dtype=bool)
    for prob, lo, hi in param_buckets:
        acc += prob
        sel = (~chosen) & (ub < acc + 1e-12)
        N[sel] = _log_uniform(un[sel], lo, hi)
        chosen |= sel
    lo, hi = param_buckets[-1][1], param_buckets[-1][2]
    N[~chosen] = _log_uniform(un[~chosen], lo, hi)

    def pick(fld, choices):
        c = np.asarray(choices)
        return c[np.minimum((u(fld) * len(c)).astype(np.int64), len(c) - 1)]

    layers = pick(_F_LAYERS, layer_choices).astype(np.uint32)
    gbatch = pick(_F_BATCH, batch_choices).astype(np.uint32)
    mbatch = pick(_F_MBATCH, mbatch_choices).astype(np.uint32)
    # hidden size from the usual transformer size relation N ~ 12 l h^2
    hidden = 128.0 * np.maximum(1.0, np.round(np.sqrt(N / (12.0 * layers)) / 128.0))

    nominal = {
        "P_bytes": 2.0 * N,
        "seq": np.full(J, float(seq)),
        "hidden": hidden,
        "elem_bytes": np.full(J, 2.0),
        "t_fwd_sample": 2.0 * N * seq / 1.5e14,
        "k_bwd": np.full(J, 2.0),
        "k_sync": np.full(J, 2.0),
        "k_opt": np.full(J, 5e-12),
        "k_opt_off": np.full(J, 5e-9),
        "k_off": np.full(J, 2.0),
        "k_swap": np.full(J, 2.0),
        "k_const": np.full(J, 0.05),
        "mem_state": np.full(J, 1.0),
        "mem_act": np.full(J, 34.0),
        "mem_act_gc": np.full(J, 2.0),
        "mem_const": np.full(J, float(2 ** 30)),
        # reference throughput used to normalise speedups: a nominal
        # samples/s figure for the model size (an input, not a prediction)
        "ref_thr": 1.5e14 / (6.0 * N * seq),
    }
    fixed = {"P_bytes", "seq", "hidden", "elem_bytes"}      # model constants, not fitted
    coef = np.zeros((J, N_COEF), dtype=np.float32)
    for col, name in enumerate(COEF_FIELDS):
        v = nominal[name]
        if name not in fixed:
            v = v * (0.5 + 1.5 * u(_F_COEF0 + col))
        coef[:, col] = v.astype(np.float32)
    ints = np.stack([layers, gbatch, mbatch], axis=1).astype(np.uint32)
    return np.ascontiguousarray(coef), np.ascontiguousarray(ints)


def _abs_levels(n):
    return np.arange(1, n + 1, dtype=np.uint32)


def tiny(seed: int = BASE_SEED) -> Workload:
    """8 jobs on one 8-GPU node; about 1e4 candidates."""
    coef, ints = draw_jobs(seed, 1, 0, np.arange(8), param_buckets=[(1.0, 0.1e9, 13e9)],
                           layer_choices=(12, 24, 32, 40))
    return Workload("tiny", coef, ints, Bounds(g_max=8),
                    Grid(_abs_levels(8), 0, np.array([64.0], np.float32), 0),
                    Env(), Cluster(8, 32, 512.0))


def paper_scale(seed: int = BASE_SEED) -> Workload:
    """64 jobs on 8 nodes x 8 GPUs (the size of the paper's testbed); about 1e6 candidates."""
    coef, ints = draw_jobs(seed, 2, 0, np.arange(64),
                           param_buckets=[(0.4, 0.1e9, 1.3e9), (0.4, 1.3e9, 13e9), (0.2, 13e9, 70e9)],
                           layer_choices=(12, 24, 32, 40))
    return Workload("paper_scale", coef, ints, Bounds(g_max=64),
                    Grid(_abs_levels(32), 0, np.array([64.0], np.float32), 0),
                    Env(), Cluster(64, 256, 4096.0))


_BIG = dict(param_buckets=[(1.0, 0.1e9, 175e9)], layer_choices=(24, 32, 48, 80, 96))
_RATIOS = np.array([1, 2, 4, 8, 16], dtype=np.uint32)


def large(seed: int = BASE_SEED) -> Workload:
    """1,000 jobs, 128 nodes x (8 GPUs, 128 CPUs, 2 TB); CPU levels are per-GPU ratios."""
    coef, ints = draw_jobs(seed, 3, 0, np.arange(1000), **_BIG)
    return Workload("large", coef, ints, Bounds(g_max=1024),
                    Grid(_RATIOS.copy(), 1, np.array([2048.0], np.float32), 0),
                    Env(), Cluster(1024, 128 * 128, 128 * 2048.0))


def stress(seed: int = BASE_SEED, n_jobs: int = 10000) -> Workload:
    """10,000 jobs, 4096 GPUs, full (g, CPU ratio, host-memory tier) grid."""
    coef, ints = draw_jobs(seed, 4, 0, np.arange(n_jobs), **_BIG)
    return Workload("stress", coef, ints, Bounds(g_max=4096),
                    Grid(_RATIOS.copy(), 1, np.array([0.0, 64.0, 256.0, 1024.0], np.float32), 0),
                    Env(), Cluster(4096, 512 * 128, 512 * 2048.0))


def what_if(round_index: int, seed: int = BASE_SEED, n_jobs: int = 500) -> Workload:
    """One of 256 independent what-if rounds: 500 jobs on about 512 GPUs.

    Capacity is perturbed by a uniform +-25 % and one job in ten is redrawn,
    both keyed by (seed, round)."""
    r = int(round_index)
    ids = np.arange(n_jobs)
    n_redraw = n_jobs // 10
    order = np.argsort(uniform(seed, 5, r, ids, 1000), kind="stable")
    rnd = np.zeros(n_jobs, dtype=np.uint64)
    rnd[order[:n_redraw]] = r + 1                      # stream 0 is the base job set
    coef, ints = draw_jobs(seed, 5, rnd, ids, **_BIG)
    ug = float(uniform(seed, 5, r, 0, 1001))
    uc = float(uniform(seed, 5, r, 0, 1002))
    G = int(round(512 * (1.0 + (ug - 0.5) * 0.5)))
    C = int(round(8192 * (1.0 + (uc - 0.5) * 0.5)))
    return Workload(f"what_if[{r}]", coef, ints, Bounds(g_max=512),
                    Grid(_RATIOS.copy(), 1, np.array([2048.0], np.float32), 0),
                    Env(), Cluster(G, C, 64 * 2048.0), {"round": r, "redrawn": np.sort(order[:n_redraw])})


def what_if_shared(n_rounds: int, seed: int = BASE_SEED, n_jobs: int = 500):
    """The same what-if rounds with every distinct job listed once: the jobs that
    a round does not redraw are the base jobs.  Returns (workload of the distinct
    jobs, round_off, round_jobs, clusters): slot i of round r is job
    round_jobs[round_off[r] + i], and what_if(r) equals the distinct jobs gathered
    by that slice."""
    ids = np.arange(n_jobs)
    base_coef, base_ints = draw_jobs(seed, 5, 0, ids, **_BIG)
    coefs, ints, round_jobs, clusters = [base_coef], [base_ints], [], []
    n_distinct = n_jobs
    first = None
    for r in range(n_rounds):
        w = what_if(r, seed, n_jobs)
        first = first or w
        red = w.meta["redrawn"]
        slots = ids.copy()
        slots[red] = n_distinct + np.arange(len(red))
        n_distinct += len(red)
        coefs.append(w.coef[red])
        ints.append(w.ints[red])
        round_jobs.append(slots)
        clusters.append(w.cluster)
    wl = Workload("what_if[shared]", np.concatenate(coefs), np.concatenate(ints), first.bounds, first.grid, first.env,
                  first.cluster)
    round_off = np.arange(n_rounds + 1, dtype=np.uint32) * n_jobs
    return wl, round_off, np.concatenate(round_jobs).astype(np.uint32), clusters


@dataclass
class SlaDraws:
    """Service-level side of a round (Sec. 5.2 / 7.1: guaranteed and best-effort
    jobs of several tenants).  Positions inside a job's plan space are given as
    uniform draws in [0,1); whoever holds the plan table maps them to indices."""
    guaranteed: np.ndarray           # uint32 [J], 0/1
    tenant: np.ndarray               # uint32 [J]
    u_seg: np.ndarray                # float64 [J]: position of the requested GPU count among the job's valid counts
    req_c: np.ndarray                # uint32 [J] requested CPU level
    req_m: np.ndarray                # uint32 [J] requested memory tier
    u_plan: np.ndarray               # float64 [J]: position of the original plan among the plans of that GPU count
    quota_g: np.ndarray              # uint32 [n_tenants]
    quota_c: np.ndarray              # uint32 [n_tenants]


def sla_draws(wl: Workload, seed: int = BASE_SEED, frac_guaranteed: float = 0.3, n_tenants: int = 6,
              quota_share: float = 1.0) -> SlaDraws:
    """Requests skewed to small GPU counts (most jobs ask for few GPUs, as in the
    paper's traces); tenant quotas sum to about quota_share of the cluster."""
    ids = np.arange(wl.n_jobs)
    guaranteed = (uniform(seed, 7, 0, ids, 1) < frac_guaranteed).astype(np.uint32)
    tenant = np.minimum((uniform(seed, 7, 0, ids, 2) * n_tenants).astype(np.uint32), n_tenants - 1)
    u_seg = uniform(seed, 7, 0, ids, 3) ** 2
    n_cpu, n_mem = len(wl.grid.cpu_levels), len(wl.grid.mem_levels_gb)
    req_c = np.minimum((uniform(seed, 7, 0, ids, 4) * n_cpu).astype(np.uint32), n_cpu - 1)
    req_m = np.minimum((uniform(seed, 7, 0, ids, 5) * n_mem).astype(np.uint32), n_mem - 1)
    u_plan = uniform(seed, 7, 0, ids, 6)
    w = 0.5 + uniform(seed, 7, 1, np.arange(n_tenants), 0)
    w = w / w.sum() * quota_share
    quota_g = np.floor(w * wl.cluster.G).astype(np.uint32)
    quota_c = np.floor(w * wl.cluster.C).astype(np.uint32)
    return SlaDraws(guaranteed, tenant, u_seg, req_c, req_m, u_plan, quota_g, quota_c)


@dataclass
class FitDraws:
    """Sampled test runs for the model fitting (Sec. 4 "Continuous model
    fitting": at least seven runs per model type, three of them with
    ZeRO-Offload).  Plans are given as positions in [0,1) inside the model's
    enumerated (d,t,p) list; whoever holds the plan table maps them to triples."""
    u_triple: np.ndarray             # float64 [J, S]
    option: np.ndarray               # uint32 [J, S] option code z*4 + gc*2 + off
    cpus: np.ndarray                 # uint32 [J, S] CPUs of the job in that run
    noise_z: np.ndarray              # float64 [J, S] standard normal: measured = true * exp(sigma * z)
    start_factor: np.ndarray         # float64 [J, 7] initial guess = true parameter * factor
    start_offsets: np.ndarray        # float64 [R, 7] extra starting points, offsets in the log-parameter space


def fit_draws(n_models: int, n_samples: int = 16, n_offload: int = 5, n_restarts: int = 4,
              seed: int = BASE_SEED) -> FitDraws:
    ids = np.arange(n_models)[:, None]
    k = np.arange(n_samples)[None, :]
    u_triple = uniform(seed, 8, 0, ids, 10 + k * 8)
    z = (uniform(seed, 8, 0, ids, 11 + k * 8) * 4).astype(np.uint32)
    gc = (uniform(seed, 8, 0, ids, 12 + k * 8) * 2).astype(np.uint32)
    off = np.broadcast_to(k < n_offload, z.shape).astype(np.uint32)
    z = np.where(off == 1, 2 + (z & 1), z).astype(np.uint32)             # offload needs stage 2 or 3
    option = (z * 4 + gc * 2 + off).astype(np.uint32)
    cpus = np.array([1, 2, 4, 8, 16, 32], np.uint32)[(uniform(seed, 8, 0, ids, 13 + k * 8) * 6).astype(np.int64)]
    u1, u2 = uniform(seed, 8, 0, ids, 14 + k * 8), uniform(seed, 8, 0, ids, 15 + k * 8)
    noise_z = np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)
    par = np.arange(7)[None, :]
    start_factor = np.exp((uniform(seed, 8, 1, ids, par) * 2.0 - 1.0) * np.log(2.0))
    r = np.arange(n_restarts)[:, None]
    a, b = uniform(seed, 8, 2, r, par * 2), uniform(seed, 8, 2, r, par * 2 + 1)
    start_offsets = 0.7 * np.sqrt(-2.0 * np.log(1.0 - a)) * np.cos(2.0 * np.pi * b)
    return FitDraws(u_triple, option, cpus, noise_z, start_factor, start_offsets)


def fit_sample_triples(draws: FitDraws, triple_off: np.ndarray, triples: np.ndarray):
    """Map the plan positions of the draws onto a plan table (CSR offsets and
    [n][3 or 4] unpacked triples): returns d, t, p as uint32 [J, S]."""
    J, S = draws.u_triple.shape
    t0 = np.asarray(triple_off[:J], np.int64)[:, None]
    nt = (np.asarray(triple_off[1:J + 1], np.int64) - np.asarray(triple_off[:J], np.int64))[:, None]
    idx = t0 + np.minimum((draws.u_triple * nt).astype(np.int64), np.maximum(nt - 1, 0))
    tr = np.asarray(triples)[idx]
    return tr[..., 0].astype(np.uint32), tr[..., 1].astype(np.uint32), tr[..., 2].astype(np.uint32)


@dataclass
class Trace:
    """Arrival trace for the cluster simulation (Sec. 7.1 / 7.4: a busy 12-hour
    window of a production trace, down-sampled to the cluster's size)."""
    arrival: np.ndarray              # float64 [J] seconds, ascending
    u_duration: np.ndarray           # float64 [J] in [0,1): position of the job's length in the length distribution
    delta: np.ndarray                # float64 [J] checkpoint-resume cost, seconds


def trace(n_jobs: int, horizon_s: float = 12 * 3600.0, seed: int = BASE_SEED) -> Trace:
    """Poisson arrivals over the horizon; lengths are mapped by the caller
    (heavy-tailed: most jobs short, a few long); checkpoint-resume 30-120 s."""
    ids = np.arange(n_jobs)
    gaps = -np.log(1.0 - uniform(seed, 9, 0, ids, 0))
    arrival = np.cumsum(gaps)
    arrival = arrival / arrival[-1] * horizon_s * (1.0 - 1.0 / max(n_jobs, 1))
    return Trace(arrival, uniform(seed, 9, 0, ids, 1), 30.0 + 90.0 * uniform(seed, 9, 0, ids, 2))


def job_lengths_s(u: np.ndarray) -> np.ndarray:
    """Job length in seconds on its reference allocation: log-uniform from 5 minutes to 8 hours."""
    return 300.0 * np.exp(u * np.log(8 * 3600.0 / 300.0))


def trace_scale(seed: int = BASE_SEED, n_jobs: int = 406) -> Workload:
    """The shape of the paper's trace experiment: 406 jobs on 8 nodes x 8 GPUs (models as in paper_scale)."""
    coef, ints = draw_jobs(seed, 6, 0, np.arange(n_jobs),
                           param_buckets=[(0.4, 0.1e9, 1.3e9), (0.4, 1.3e9, 13e9), (0.2, 13e9, 70e9)],
                           layer_choices=(12, 24, 32, 40))
    return Workload("trace_scale", coef, ints, Bounds(g_max=64),
                    Grid(_abs_levels(32), 0, np.array([64.0], np.float32), 0),
                    Env(), Cluster(64, 256, 4096.0))


CONFIGS = {"tiny": tiny, "paper_scale": paper_scale, "large": large, "stress": stress}
