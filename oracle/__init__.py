"""ctypes access to the CPU oracle (oracle/rk_oracle.cpp).

TEST INFRASTRUCTURE ONLY.  May be imported by tests/, by the smoke check and
by the CPU-baseline leg of the benchmark; never by the GPU library or its
Python binding.  Imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rk_oracle.cpp")
_HDR = os.path.join(_HERE, "rk_oracle.h")
_LIB = os.path.join(_HERE, "librk_oracle.so")

NO_PLAN = 0xFFFFFFFF
N_TERMS = 24
TERMS = ("n", "m", "a", "Tf_mb", "T_fwd", "T_bwd", "V_dp", "V_tp", "V_pp", "T_dp", "T_tp",
         "T_pp", "T_cc", "Psi", "T_opt", "T_off", "T_oo", "T_iter", "thr", "M_gpu", "H_host",
         "B_dp", "B_tp", "B_pp")


_LIB_SAN = os.path.join(_HERE, "librk_oracle_san.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with g++ (strict IEEE: no contraction, no fast-math).

    sanitize=True builds a second library with AddressSanitizer and
    UndefinedBehaviorSanitizer (CPU only).  A process can load it only when the
    sanitizer runtime is loaded first (LD_PRELOAD=$(g++ -print-file-name=libasan.so));
    setting RK_ORACLE_SANITIZE=1 makes lib() pick it."""
    out = _LIB_SAN if sanitize else _LIB
    stale = (not os.path.exists(out)
             or os.path.getmtime(out) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", "-pthread", "-Wall"]
        if sanitize:
            cmd += ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
        subprocess.run(cmd + ["-o", out, _SRC], check=True, cwd=_HERE)
    return out


class _Env(C.Structure):
    _fields_ = [("B_intra", C.c_float), ("B_inter", C.c_float), ("B_pcie", C.c_float),
                ("gpu_mem_cap", C.c_float), ("gpus_per_node", C.c_uint32)]


class _Grid(C.Structure):
    _fields_ = [("n_cpu", C.c_uint32), ("cpu_levels", C.c_void_p), ("cpu_mode", C.c_uint32),
                ("n_mem", C.c_uint32), ("mem_levels_gb", C.c_void_p), ("mem_mode", C.c_uint32)]


class _Bounds(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("g_max", "tp_max", "pp_max", "zero_mask", "gc_mask", "off_mask", "mu_mask")]


class _Table(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("triple_off", "triples", "seg_off", "seg_g", "seg_first")]


ASSIGN_DTYPE = np.dtype([("g", np.uint32), ("c", np.uint32), ("mem_gb", np.float32),
                         ("plan", np.uint32), ("thr", np.float32)])

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build(sanitize=os.environ.get("RK_ORACLE_SANITIZE") == "1"))
        _lib.ork_host_cores.restype = C.c_uint32
        _lib.ork_f_overlap.restype = C.c_double
        _lib.ork_f_overlap.argtypes = [C.c_double] * 3
        _lib.ork_eval_one.restype = C.c_uint32
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _env(env):
    return _Env(env.B_intra, env.B_inter, env.B_pcie, env.gpu_mem_cap, env.gpus_per_node)


def _bounds(b):
    return _Bounds(b.g_max, b.tp_max, b.pp_max, b.zero_mask, b.gc_mask, b.off_mask, getattr(b, "mu_mask", 1))


class _GridHolder:
    def __init__(self, grid):
        self.cpu = np.ascontiguousarray(grid.cpu_levels, dtype=np.uint32)
        self.mem = np.ascontiguousarray(grid.mem_levels_gb, dtype=np.float32)
        self.c = _Grid(len(self.cpu), _p(self.cpu), grid.cpu_mode, len(self.mem), _p(self.mem), grid.mem_mode)
        self.rows = len(self.cpu) * len(self.mem)


class Table:
    """Plan table produced by enumerate(); numpy arrays."""

    def __init__(self, triple_off, triples, seg_off, seg_g, seg_first):
        self.triple_off, self.triples = triple_off, triples
        self.seg_off, self.seg_g, self.seg_first = seg_off, seg_g, seg_first
        self.c = _Table(_p(triple_off), _p(triples), _p(seg_off), _p(seg_g), _p(seg_first))

    @property
    def n_jobs(self):
        return len(self.triple_off) - 1

    def n_candidates(self, rows, jb=0, je=None):
        je = self.n_jobs if je is None else je
        return 16 * rows * int(self.triple_off[je] - self.triple_off[jb])

    def n_segments(self, rows, jb=0, je=None):
        je = self.n_jobs if je is None else je
        return rows * int(self.seg_off[je] - self.seg_off[jb])


def f_overlap(k, x, y):
    return lib().ork_f_overlap(float(k), float(x), float(y))


def host_cores() -> int:
    """Host threads the machine offers (std::thread::hardware_concurrency)."""
    return int(lib().ork_host_cores())


def enumerate_plans(ints, bounds, n_threads=1) -> Table:
    ints = np.ascontiguousarray(ints, dtype=np.uint32)
    J = ints.shape[0]
    nt, ns = C.c_uint64(0), C.c_uint64(0)
    b = _bounds(bounds)
    lib().ork_enumerate(C.c_uint32(J), _p(ints), C.byref(b), None, None, C.c_uint64(0), None, None, None,
                        C.c_uint64(0), C.byref(nt), C.byref(ns), C.c_uint32(n_threads))
    triple_off = np.zeros(J + 1, np.uint32)
    triples = np.zeros((max(nt.value, 1), 4), np.uint32)
    seg_off = np.zeros(J + 1, np.uint32)
    seg_g = np.zeros(max(ns.value, 1), np.uint32)
    seg_first = np.zeros(max(ns.value, 1), np.uint32)
    rc = lib().ork_enumerate(C.c_uint32(J), _p(ints), C.byref(b), _p(triple_off), _p(triples),
                             C.c_uint64(nt.value), _p(seg_off), _p(seg_g), _p(seg_first),
                             C.c_uint64(ns.value), C.byref(nt), C.byref(ns), C.c_uint32(n_threads))
    assert rc == 0
    return Table(triple_off, triples[:nt.value], seg_off, seg_g[:ns.value], seg_first[:ns.value])


def eval_one(coef_row, ints_row, bounds, env, d, t, p, z, gc, off, c, host_bytes, v=0):
    """One candidate -> (reason bits, dict of every intermediate term); v = micro-batch shift of the plan."""
    cf = np.ascontiguousarray(coef_row, dtype=np.float32)
    it = np.ascontiguousarray(ints_row, dtype=np.uint32)
    terms = np.zeros(N_TERMS, np.float64)
    b, e = _bounds(bounds), _env(env)
    reason = lib().ork_eval_one(_p(cf), _p(it), C.byref(b), C.byref(e), C.c_uint32(d), C.c_uint32(t),
                                C.c_uint32(p), C.c_uint32(v), C.c_uint32(z), C.c_uint32(gc), C.c_uint32(off),
                                C.c_uint32(c), C.c_float(host_bytes), _p(terms))
    return int(reason), dict(zip(TERMS, terms.tolist()))


def eval_jobs(coef, ints, bounds, table, grid, env, jb=0, je=None, want_reason=True, n_threads=1):
    coef = np.ascontiguousarray(coef, dtype=np.float32)
    ints = np.ascontiguousarray(ints, dtype=np.uint32)
    J = coef.shape[0]
    je = J if je is None else je
    gh = _GridHolder(grid)
    n = table.n_candidates(gh.rows, jb, je)
    thr = np.zeros(n, np.float64)
    reason = np.zeros(n, np.uint8) if want_reason else None
    b, e = _bounds(bounds), _env(env)
    rc = lib().ork_eval_jobs(C.c_uint32(J), _p(coef), _p(ints), C.byref(b), C.byref(table.c), C.byref(gh.c),
                             C.byref(e), C.c_uint32(jb), C.c_uint32(je), _p(thr), _p(reason),
                             C.c_uint32(n_threads))
    assert rc == 0
    return thr, reason


def best_plan(table, grid, thr, jb=0, je=None, n_threads=1):
    """Segmented argmax; dtype of thr (float64 or float32) selects the precision."""
    je = table.n_jobs if je is None else je
    gh = _GridHolder(grid)
    n = table.n_segments(gh.rows, jb, je)
    thr = np.ascontiguousarray(thr)
    assert thr.dtype in (np.float32, np.float64)
    assert thr.size == table.n_candidates(gh.rows, jb, je)
    best_thr = np.zeros(n, thr.dtype)
    best_idx = np.zeros(n, np.uint32)
    fn = lib().ork_best_plan_f64 if thr.dtype == np.float64 else lib().ork_best_plan_f32
    rc = fn(C.byref(table.c), C.byref(gh.c), C.c_uint32(jb), C.c_uint32(je), _p(thr), _p(best_thr), _p(best_idx),
            C.c_uint32(n_threads))
    assert rc == 0
    return best_thr, best_idx


def curves(table, grid, best_thr, best_idx, jb=0, je=None):
    je = table.n_jobs if je is None else je
    gh = _GridHolder(grid)
    best_thr = np.ascontiguousarray(best_thr, dtype=np.float32)
    best_idx = np.ascontiguousarray(best_idx, dtype=np.uint32)
    n = table.n_segments(gh.rows, jb, je)
    assert best_thr.size == n and best_idx.size == n
    ct, cp, cg = np.zeros(n, np.float32), np.zeros(n, np.uint32), np.zeros(n, np.uint32)
    rc = lib().ork_curves_f32(C.byref(table.c), C.byref(gh.c), C.c_uint32(jb), C.c_uint32(je),
                              _p(best_thr), _p(best_idx), _p(ct), _p(cp), _p(cg))
    assert rc == 0
    return ct, cp, cg


def greedy(ref_thr, table, grid, cluster, best_thr, best_idx, curve_thr):
    gh = _GridHolder(grid)
    J = table.n_jobs
    ref_thr = np.ascontiguousarray(ref_thr, dtype=np.float32)
    best_thr = np.ascontiguousarray(best_thr, dtype=np.float32)
    best_idx = np.ascontiguousarray(best_idx, dtype=np.uint32)
    curve_thr = np.ascontiguousarray(curve_thr, dtype=np.float32)
    assign = np.zeros(J, ASSIGN_DTYPE)
    total, gap = C.c_double(0), C.c_double(0)
    rc = lib().ork_greedy_f32(C.c_uint32(J), _p(ref_thr), C.byref(table.c), C.byref(gh.c),
                              C.c_uint32(cluster.G), C.c_uint32(cluster.C), C.c_float(cluster.host_mem_gb),
                              _p(best_thr), _p(best_idx), _p(curve_thr), _p(assign),
                              C.byref(total), C.byref(gap))
    assert rc == 0
    return assign, total.value, gap.value


def schedule_round(wl, n_threads=1):
    """The whole path on a workload: enumerate -> evaluate (float64) -> argmax
    (float64) -> round to float32 -> curves -> greedy.  Returns a dict."""
    table = enumerate_plans(wl.ints, wl.bounds, n_threads=n_threads)
    thr, reason = eval_jobs(wl.coef, wl.ints, wl.bounds, table, wl.grid, wl.env, n_threads=n_threads)
    bt64, bp = best_plan(table, wl.grid, thr, n_threads=n_threads)
    bt = bt64.astype(np.float32)
    ct, cp, cg = curves(table, wl.grid, bt, bp)
    assign, total, gap = greedy(wl.coef[:, 16], table, wl.grid, wl.cluster, bt, bp, ct)
    return dict(table=table, thr=thr, reason=reason, best_thr64=bt64, best_thr=bt, best_plan=bp,
                curve_thr=ct, curve_plan=cp, curve_g=cg, assign=assign, total=total, min_gap=gap)


def min_res(table, grid, best_thr, guaranteed, req_g, req_c, req_m, base_thr, jb=0, je=None):
    """Minimum demand of guaranteed jobs -> (segment index or -1, CPU level, memory tier) per job of the range."""
    je = table.n_jobs if je is None else je
    gh = _GridHolder(grid)
    best_thr = np.ascontiguousarray(best_thr, dtype=np.float32)
    u = lambda a: np.ascontiguousarray(a, dtype=np.uint32)
    guaranteed, req_g, req_c, req_m = u(guaranteed), u(req_g), u(req_c), u(req_m)
    base_thr = np.ascontiguousarray(base_thr, dtype=np.float32)
    n = je - jb
    seg, c, m = np.zeros(n, np.int32), np.zeros(n, np.uint32), np.zeros(n, np.uint32)
    rc = lib().ork_min_res_f32(C.byref(table.c), C.byref(gh.c), C.c_uint32(jb), C.c_uint32(je), _p(best_thr),
                               _p(guaranteed), _p(req_g), _p(req_c), _p(req_m), _p(base_thr), _p(seg), _p(c), _p(m))
    assert rc == 0
    return seg, c, m


def policy(ref_thr, table, grid, cluster, best_thr, best_idx, curve_thr, guaranteed, tenant, min_seg, min_c,
           quota_g, quota_c):
    """Greedy with service-level floors and tenant quotas."""
    gh = _GridHolder(grid)
    J = table.n_jobs
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    u = lambda a: np.ascontiguousarray(a, dtype=np.uint32)
    ref_thr, best_thr, curve_thr = f(ref_thr), f(best_thr), f(curve_thr)
    best_idx, guaranteed, tenant, min_c, quota_g, quota_c = u(best_idx), u(guaranteed), u(tenant), u(min_c), u(quota_g), u(quota_c)
    min_seg = np.ascontiguousarray(min_seg, dtype=np.int32)
    assign = np.zeros(J, ASSIGN_DTYPE)
    total, gap = C.c_double(0), C.c_double(0)
    rc = lib().ork_policy_f32(C.c_uint32(J), _p(ref_thr), C.byref(table.c), C.byref(gh.c), C.c_uint32(cluster.G),
                              C.c_uint32(cluster.C), C.c_float(cluster.host_mem_gb), _p(best_thr), _p(best_idx),
                              _p(curve_thr), _p(guaranteed), _p(tenant), _p(min_seg), _p(min_c),
                              C.c_uint32(len(quota_g)), _p(quota_g), _p(quota_c), _p(assign),
                              C.byref(total), C.byref(gap))
    assert rc == 0
    return assign, total.value, gap.value


from . import fitting  # noqa: E402  (model fitting on top of the functions above)


def frozen_round(ref_thr, table, grid, cluster, best_thr, best_idx, curve_thr, state, cur_seg, cur_c):
    """Greedy round with per-job state: 0 takes part, 1 takes no part, 2 keeps (cur_seg, cur_c)."""
    gh = _GridHolder(grid)
    J = table.n_jobs
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    ref_thr, best_thr, curve_thr = f(ref_thr), f(best_thr), f(curve_thr)
    best_idx = np.ascontiguousarray(best_idx, dtype=np.uint32)
    state = np.ascontiguousarray(state, dtype=np.uint8)
    cur_seg = np.ascontiguousarray(cur_seg, dtype=np.int32)
    cur_c = np.ascontiguousarray(cur_c, dtype=np.uint32)
    assign = np.zeros(J, ASSIGN_DTYPE)
    total, gap = C.c_double(0), C.c_double(0)
    rc = lib().ork_frozen_round_f32(C.c_uint32(J), _p(ref_thr), C.byref(table.c), C.byref(gh.c), C.c_uint32(cluster.G),
                                    C.c_uint32(cluster.C), C.c_float(cluster.host_mem_gb), _p(best_thr), _p(best_idx),
                                    _p(curve_thr), _p(state), _p(cur_seg), _p(cur_c), _p(assign), C.byref(total),
                                    C.byref(gap))
    assert rc == 0
    return assign, total.value, gap.value


def reschedule(ref_thr, table, grid, cluster, best_thr, best_idx, curve_thr, cur_seg, cur_c, floor_seg=None, floor_c=None,
               state=None):
    """Algorithm 1's Schedule as a loop from the jobs' present state -> (records, total, steps committed)."""
    gh = _GridHolder(grid)
    J = table.n_jobs
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    ref_thr, best_thr, curve_thr = f(ref_thr), f(best_thr), f(curve_thr)
    best_idx = np.ascontiguousarray(best_idx, dtype=np.uint32)
    cur_seg = np.ascontiguousarray(cur_seg, dtype=np.int32)
    cur_c = np.ascontiguousarray(cur_c, dtype=np.uint32)
    state = None if state is None else np.ascontiguousarray(state, dtype=np.uint8)
    floor_seg = None if floor_seg is None else np.ascontiguousarray(floor_seg, dtype=np.int32)
    floor_c = None if floor_c is None else np.ascontiguousarray(floor_c, dtype=np.uint32)
    assign = np.zeros(J, ASSIGN_DTYPE)
    total, moves = C.c_double(0), C.c_uint32(0)
    rc = lib().ork_reschedule_f32(C.c_uint32(J), _p(ref_thr), C.byref(table.c), C.byref(gh.c), C.c_uint32(cluster.G),
                                  C.c_uint32(cluster.C), C.c_float(cluster.host_mem_gb), _p(best_thr), _p(best_idx),
                                  _p(curve_thr), _p(state), _p(cur_seg), _p(cur_c), _p(floor_seg), _p(floor_c), _p(assign),
                                  C.byref(total), C.byref(moves))
    assert rc == 0
    return assign, total.value, moves.value


PLACE_DTYPE = np.dtype([("node", np.uint32), ("g", np.uint32), ("c", np.uint32), ("mem_gb", np.float32)])


def place(assign, n_nodes, gpus_per_node, cpus_per_node, mem_per_node_gb):
    """Node-level placement of an allocation: (place_off, entries, status)."""
    assign = np.ascontiguousarray(assign, dtype=ASSIGN_DTYPE)
    J = assign.size
    place_off = np.zeros(J + 1, np.uint32)
    entries = np.zeros(max(int(assign["g"].astype(np.uint64).sum()), 1), PLACE_DTYPE)
    status = np.zeros(J, np.uint32)
    rc = lib().ork_place_f32(C.c_uint32(J), _p(assign), C.c_uint32(n_nodes), C.c_uint32(gpus_per_node),
                             C.c_uint32(cpus_per_node), C.c_float(mem_per_node_gb), _p(place_off), _p(entries),
                             _p(status))
    assert rc == 0
    return place_off, entries[:int(place_off[J])].copy(), status


def eval_one_placed(coef_row, ints_row, bounds, env, d, t, p, z, gc, off, c, host_bytes, parts, v=0):
    """One candidate on a placement: parts = GPUs on the consecutive nodes the job sits on."""
    cf = np.ascontiguousarray(coef_row, dtype=np.float32)
    it = np.ascontiguousarray(ints_row, dtype=np.uint32)
    parts = np.ascontiguousarray(parts, dtype=np.uint32)
    assert int(parts.sum()) == d * t * p
    terms = np.zeros(N_TERMS, np.float64)
    b, e = _bounds(bounds), _env(env)
    lib().ork_eval_one_placed.restype = C.c_uint32
    reason = lib().ork_eval_one_placed(_p(cf), _p(it), C.byref(b), C.byref(e), C.c_uint32(d), C.c_uint32(t),
                                       C.c_uint32(p), C.c_uint32(v), C.c_uint32(z), C.c_uint32(gc), C.c_uint32(off),
                                       C.c_uint32(c), C.c_float(host_bytes), C.c_uint32(len(parts)), _p(parts), _p(terms))
    return int(reason), dict(zip(TERMS, terms.tolist()))


def place_plans(coef, ints, bounds, table, grid, env, best_thr, assign, n_nodes, gpus_per_node, cpus_per_node,
                mem_per_node_gb, min_seg=None, prev=None):
    """Placement that feeds the plan -> (placed records, place_off, entries, status, total).
    prev = (place_off, entries) of an earlier placement: jobs whose amounts are unchanged stay on their nodes."""
    coef = np.ascontiguousarray(coef, dtype=np.float32)
    ints = np.ascontiguousarray(ints, dtype=np.uint32)
    best_thr = np.ascontiguousarray(best_thr, dtype=np.float32)
    assign = np.ascontiguousarray(assign, dtype=ASSIGN_DTYPE)
    J = assign.size
    gh = _GridHolder(grid)
    ms = None if min_seg is None else np.ascontiguousarray(min_seg, dtype=np.int32)
    out = np.zeros(J, ASSIGN_DTYPE)
    place_off = np.zeros(J + 1, np.uint32)
    entries = np.zeros(max(int(assign["g"].astype(np.uint64).sum()), 1), PLACE_DTYPE)
    status = np.zeros(J, np.uint32)
    total = C.c_double(0)
    b, e = _bounds(bounds), _env(env)
    p_off = None if prev is None else np.ascontiguousarray(prev[0], dtype=np.uint32)
    p_ent = None if prev is None else np.ascontiguousarray(prev[1], dtype=PLACE_DTYPE)
    if prev is not None:
        assert p_off.size == J + 1 and int(p_off[J]) <= max(p_ent.size, 0) and np.all(np.diff(p_off.astype(np.int64)) >= 0)
        if p_ent.size == 0:
            p_ent = np.zeros(1, PLACE_DTYPE)
    rc = lib().ork_place_plans(C.c_uint32(J), _p(coef), _p(ints), C.byref(b), C.byref(table.c), C.byref(gh.c), C.byref(e),
                               _p(best_thr), _p(assign), _p(ms), _p(p_off), _p(p_ent), C.c_uint32(n_nodes), C.c_uint32(gpus_per_node),
                               C.c_uint32(cpus_per_node), C.c_float(mem_per_node_gb), _p(out), _p(place_off), _p(entries),
                               _p(status), C.byref(total))
    assert rc == 0, "the records are not an allocation on this table and grid, or the kept parts do not fit the nodes"
    return out, place_off, entries[:int(place_off[J])].copy(), status, total.value


def reschedule_nodes(ref_thr, table, grid, n_nodes, gpus_per_node, cpus_per_node, mem_per_node_gb, best_thr, best_idx,
                     curve_thr, cur_seg, cur_c, prev, floor_seg=None, floor_c=None, state=None):
    """Algorithm 1's Schedule with the node-by-node search of ScheduleJob, from the jobs' present state and
    placement prev = (place_off, entries) -> (records, place_off, entries, total, steps committed), or None when
    the state is not a placement on these nodes."""
    gh = _GridHolder(grid)
    J = table.n_jobs
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    ref_thr, best_thr, curve_thr = f(ref_thr), f(best_thr), f(curve_thr)
    best_idx = np.ascontiguousarray(best_idx, dtype=np.uint32)
    cur_seg = np.ascontiguousarray(cur_seg, dtype=np.int32)
    cur_c = np.ascontiguousarray(cur_c, dtype=np.uint32)
    state = None if state is None else np.ascontiguousarray(state, dtype=np.uint8)
    floor_seg = None if floor_seg is None else np.ascontiguousarray(floor_seg, dtype=np.int32)
    floor_c = None if floor_c is None else np.ascontiguousarray(floor_c, dtype=np.uint32)
    p_off = None if prev is None else np.ascontiguousarray(prev[0], dtype=np.uint32)
    p_ent = None if prev is None else np.ascontiguousarray(prev[1], dtype=PLACE_DTYPE)
    if prev is not None:
        assert p_off.size == J + 1
        if np.any(np.diff(p_off.astype(np.int64)) < 0) or int(p_off.max()) > p_ent.size:
            return None                                      # offsets that are no index into the entries
        if p_ent.size == 0:
            p_ent = np.zeros(1, PLACE_DTYPE)
    assign = np.zeros(J, ASSIGN_DTYPE)
    place_off = np.zeros(J + 1, np.uint32)
    entries = np.zeros(max(n_nodes * gpus_per_node, 1), PLACE_DTYPE)
    total, moves = C.c_double(0), C.c_uint32(0)
    rc = lib().ork_reschedule_nodes_f32(C.c_uint32(J), _p(ref_thr), C.byref(table.c), C.byref(gh.c), C.c_uint32(n_nodes),
                                        C.c_uint32(gpus_per_node), C.c_uint32(cpus_per_node), C.c_float(mem_per_node_gb),
                                        _p(best_thr), _p(best_idx), _p(curve_thr), _p(state), _p(cur_seg), _p(cur_c),
                                        _p(floor_seg), _p(floor_c), _p(p_off), _p(p_ent), _p(assign), _p(place_off),
                                        _p(entries), C.byref(total), C.byref(moves))
    assert rc != -2, "the grid's CPU levels must be CPUs per GPU"
    if rc == -1:
        return None
    assert rc == 0
    return assign, place_off, entries[:int(place_off[J])].copy(), total.value, moves.value


def privileged(table, grid, guaranteed, tenant, min_seg, min_c, quota_g, quota_c, cur_seg, cur_c, state=None):
    """Floors and states for the Schedule loops from the service levels -> (floor_seg, floor_c, state)."""
    gh = _GridHolder(grid)
    J = table.n_jobs
    u32 = lambda a: np.ascontiguousarray(a, dtype=np.uint32)
    guaranteed, tenant, min_c, quota_g, quota_c, cur_c = (u32(a) for a in (guaranteed, tenant, min_c, quota_g, quota_c, cur_c))
    min_seg, cur_seg = np.ascontiguousarray(min_seg, dtype=np.int32), np.ascontiguousarray(cur_seg, dtype=np.int32)
    state = None if state is None else np.ascontiguousarray(state, dtype=np.uint8)
    floor_seg, floor_c, out = np.zeros(J, np.int32), np.zeros(J, np.uint32), np.zeros(J, np.uint8)
    rc = lib().ork_privileged(C.c_uint32(J), C.byref(table.c), C.byref(gh.c), _p(guaranteed), _p(tenant), _p(min_seg), _p(min_c),
                              C.c_uint32(quota_g.size), _p(quota_g), _p(quota_c), _p(state), _p(cur_seg), _p(cur_c),
                              _p(floor_seg), _p(floor_c), _p(out))
    assert rc == 0
    return floor_seg, floor_c, out


def curve_slopes(ref_thr, table, grid, best_thr, curve_thr, jb=0, je=None):
    """The slope table of the curves -> dict(gpu_slope, gpu_next, from0_slope, from0_next, cpu_slope, cpu_next)."""
    je = table.n_jobs if je is None else je
    gh = _GridHolder(grid)
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    ref_thr, best_thr, curve_thr = f(ref_thr), f(best_thr), f(curve_thr)
    rows = len(grid.cpu_levels) * len(grid.mem_levels_gb)
    n = rows * int(table.seg_off[je] - table.seg_off[jb])
    out = dict(gpu_slope=np.zeros(n, np.float32), gpu_next=np.zeros(n, np.int32),
               from0_slope=np.zeros(rows * (je - jb), np.float32), from0_next=np.zeros(rows * (je - jb), np.int32),
               cpu_slope=np.zeros(n, np.float32), cpu_next=np.zeros(n, np.uint32))
    rc = lib().ork_curve_slopes(_p(ref_thr), C.byref(table.c), C.byref(gh.c), C.c_uint32(jb), C.c_uint32(je), _p(best_thr),
                                _p(curve_thr), _p(out["gpu_slope"]), _p(out["gpu_next"]), _p(out["from0_slope"]),
                                _p(out["from0_next"]), _p(out["cpu_slope"]), _p(out["cpu_next"]))
    assert rc == 0
    return out


from . import simulator  # noqa: E402
