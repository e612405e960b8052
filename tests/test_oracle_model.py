"""Pins for the CPU oracle's performance model (paper Sec. 4, Eq. 1).

Everything here checks the oracle against something other than itself: the
hand-worked fixture under tests/golden, closed forms of the overlap function,
special cases of the volume formulas, and exact power-of-two memory cases.
"""
import json
import math
import os

import numpy as np
import pytest

import workloads
from workloads import COEF_FIELDS

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_cases.json")
GIB = float(2 ** 30)


def make_job(spec, mem=None):
    vals = dict(elem_bytes=2, mem_state=1, mem_act=34, mem_act_gc=2, mem_const=GIB, ref_thr=1)
    vals.update(spec)
    if mem:
        vals.update(mem)
    coef = np.array([vals[n] for n in COEF_FIELDS], dtype=np.float32)
    ints = np.array([vals["layers"], vals["gbatch"], vals["mbatch"]], dtype=np.uint32)
    return coef, ints


BOUNDS = workloads.Bounds(g_max=64)
BIG_CAP = 1e30


def run(orc, coef, ints, env, d, t, p, z=0, gc=0, off=0, c=1, host=BIG_CAP, bounds=BOUNDS):
    return orc.eval_one(coef, ints, bounds, env, d, t, p, z, gc, off, c, host)


def test_f_overlap_closed_forms(orc):
    # Sec. 4.3: k = 1 is the plain sum, k -> infinity tends to the maximum
    assert orc.f_overlap(1.0, 0.3, 0.9) == pytest.approx(1.2, rel=1e-15)
    assert orc.f_overlap(2.0, 3.0, 4.0) == pytest.approx(5.0, rel=1e-15)
    assert orc.f_overlap(64.0, 2.0, 5.0) == pytest.approx(5.0, rel=0.02)
    assert orc.f_overlap(64.0, 5.0, 5.0) == pytest.approx(5.0 * 2 ** (1 / 64), rel=1e-12)
    assert orc.f_overlap(3.0, 7.0, 0.0) == pytest.approx(7.0, rel=1e-15)
    assert orc.f_overlap(3.0, 0.0, 0.0) == 0.0
    for k in (1.0, 1.7, 2.0, 3.3, 4.0):
        assert orc.f_overlap(k, 0.2, 1.3) == orc.f_overlap(k, 1.3, 0.2)
        assert orc.f_overlap(k, 1.5, 1.5) == pytest.approx(1.5 * 2 ** (1 / k), rel=1e-14)
        # between max and sum, decreasing in k
        v = orc.f_overlap(k, 0.2, 1.3)
        assert 1.3 <= v <= 1.5 + 1e-15
    assert orc.f_overlap(1.5, 1.0, 2.0) > orc.f_overlap(2.5, 1.0, 2.0)


def test_hand_cases(orc):
    g = json.load(open(GOLD))
    env = workloads.Env(B_intra=g["env"]["B_intra"], B_inter=g["env"]["B_inter"], B_pcie=g["env"]["B_pcie"],
                        gpu_mem_cap=BIG_CAP, gpus_per_node=g["env"]["gpus_per_node"])
    cases = [(g["job"], c) for c in g["cases"]]
    oc = dict(g["overlap_case"])
    job2 = dict(g["job"]); job2.update(oc["job_override"]); oc["name"] = "overlap"
    cases.append((job2, oc))
    for job, case in cases:
        coef, ints = make_job(job)
        reason, x = run(orc, coef, ints, env, case["d"], case["t"], case["p"], case["z"], case["gc"],
                        case["off"], case["c"])
        assert reason == 0, case["name"]
        for key, want in case["expect"].items():
            # inputs pass through float32 (1e-10, 0.08 ... are not exact): 1e-6 relative
            assert x[key] == pytest.approx(want, rel=2e-6, abs=1e-12), (case["name"], key)


def test_single_gpu_closed_form(orc):
    # d = t = p = 1 without options: a = b/mu accumulation steps of forward +
    # backward, the whole-model optimizer step, the constant (Sec. 4, GA form)
    wl = workloads.tiny()
    for j in range(wl.n_jobs):
        cf, it = wl.coef[j].astype(np.float64), wl.ints[j]
        reason, x = run(orc, wl.coef[j], wl.ints[j], wl.env, 1, 1, 1)
        a = int(it[1]) // int(it[2])
        name = {n: i for i, n in enumerate(COEF_FIELDS)}
        want = a * cf[name["t_fwd_sample"]] * int(it[2]) * (1.0 + cf[name["k_bwd"]]) \
            + cf[name["k_opt"]] * cf[name["P_bytes"]] + cf[name["k_const"]]
        assert x["T_iter"] == pytest.approx(want, rel=1e-13)
        assert x["thr"] == pytest.approx(int(it[1]) / want, rel=1e-13)
        assert x["V_dp"] == 0 and x["V_tp"] == 0 and x["V_pp"] == 0


def test_volume_special_cases(orc):
    env = workloads.Env(gpu_mem_cap=BIG_CAP)
    job = dict(P_bytes=6e9, seq=512, hidden=768, elem_bytes=2, t_fwd_sample=0.01, k_bwd=2, k_sync=1,
               k_opt=1e-11, k_opt_off=1e-9, k_off=1, k_swap=1, k_const=0.1, layers=12, gbatch=4096, mbatch=1)
    coef, ints = make_job(job)
    P, b, s, h, l = 6e9, 4096, 512, 768, 12
    # ring all-reduce on two replicas moves exactly the gradient size
    _, x = run(orc, coef, ints, env, 2, 1, 1)
    assert x["V_dp"] == pytest.approx(P, rel=1e-7)
    assert x["V_tp"] == 0 and x["V_pp"] == 0
    # many replicas: tends to twice the gradient shard
    _, x = run(orc, coef, ints, env, 4096, 2, 3, bounds=workloads.Bounds(g_max=1 << 20))
    assert x["V_dp"] == pytest.approx(2 * P / 6 * (4095 / 4096), rel=1e-7)
    # two tensor-parallel ranks, one replica: 4 * elem * b s h l
    _, x = run(orc, coef, ints, env, 1, 2, 1)
    assert x["V_tp"] == pytest.approx(4 * 2 * b * s * h * l, rel=1e-7)
    assert x["V_dp"] == 0 and x["V_pp"] == 0
    # tensor-parallel traffic is not divided by the pipeline size
    _, x1 = run(orc, coef, ints, env, 1, 2, 1)
    _, x3 = run(orc, coef, ints, env, 1, 2, 3)
    assert x1["V_tp"] == x3["V_tp"]
    # pipeline: 2 p elem b s h / (d t), nothing at p = 1
    _, x = run(orc, coef, ints, env, 2, 2, 3)
    assert x["V_pp"] == pytest.approx(2 * 3 * 2 * b * s * h / 4, rel=1e-7)
    _, x = run(orc, coef, ints, env, 2, 2, 1)
    assert x["V_pp"] == 0


def test_bandwidth_rule(orc):
    env = workloads.Env(B_intra=4e11, B_inter=1e11, gpu_mem_cap=BIG_CAP, gpus_per_node=8)
    job = dict(P_bytes=6e9, seq=512, hidden=768, t_fwd_sample=0.01, k_bwd=2, k_sync=1, k_opt=1e-11,
               k_opt_off=1e-9, k_off=1, k_swap=1, k_const=0.1, layers=12, gbatch=4096, mbatch=1)
    coef, ints = make_job(job)
    f32 = lambda v: float(np.float32(v))
    # inside a node everything uses the fast links
    _, x = run(orc, coef, ints, env, 2, 2, 2)
    assert (x["B_dp"], x["B_tp"], x["B_pp"]) == (f32(4e11), f32(4e11), f32(4e11))
    # 16 GPUs, t*d = 8 tiles a node: only the pipeline crosses nodes
    _, x = run(orc, coef, ints, env, 2, 4, 2)
    assert (x["B_dp"], x["B_tp"], x["B_pp"]) == (f32(4e11), f32(4e11), f32(1e11))
    # 16 GPUs, data parallel group spans nodes
    _, x = run(orc, coef, ints, env, 4, 4, 1)
    assert (x["B_dp"], x["B_tp"]) == (f32(1e11), f32(4e11))
    # a TP group that does not tile a node is charged the slow links
    env6 = workloads.Env(B_intra=4e11, B_inter=1e11, gpu_mem_cap=BIG_CAP, gpus_per_node=6)
    _, x = run(orc, coef, ints, env6, 4, 4, 1)
    assert x["B_tp"] == f32(1e11)


def test_options_change_only_what_they_should(orc):
    wl = workloads.paper_scale()
    env = workloads.Env(gpu_mem_cap=BIG_CAP)
    j = 5
    cf, it = wl.coef[j], wl.ints[j]
    base = run(orc, cf, it, env, 2, 2, 2)[1]
    # checkpointing adds exactly one forward to the backward pass
    gc = run(orc, cf, it, env, 2, 2, 2, gc=1)[1]
    assert gc["T_bwd"] == pytest.approx(base["T_bwd"] + base["T_fwd"], rel=1e-14)
    assert gc["T_fwd"] == base["T_fwd"] and gc["T_opt"] == base["T_opt"]
    # ZeRO divides the optimizer step by d and leaves the rest alone; stages agree in time
    z1 = run(orc, cf, it, env, 2, 2, 2, z=1)[1]
    assert z1["T_opt"] == pytest.approx(base["T_opt"] / 2, rel=1e-14)
    assert z1["T_cc"] == base["T_cc"]
    for z in (2, 3):
        assert run(orc, cf, it, env, 2, 2, 2, z=z)[1]["T_iter"] == z1["T_iter"]
    # ZeRO on a single replica is the same time as no ZeRO
    assert run(orc, cf, it, env, 1, 2, 2, z=2)[1]["T_iter"] == run(orc, cf, it, env, 1, 2, 2)[1]["T_iter"]
    # offload: more CPUs shorten only the optimizer; speed-up of doubling is between 1x and 2x
    o4 = run(orc, cf, it, env, 2, 1, 1, z=2, off=1, c=4)[1]
    o8 = run(orc, cf, it, env, 2, 1, 1, z=2, off=1, c=8)[1]
    assert o8["T_opt"] == pytest.approx(o4["T_opt"] / 2, rel=1e-14)
    assert o8["T_cc"] == o4["T_cc"] and o8["T_off"] == o4["T_off"]
    assert 1.0 < o8["thr"] / o4["thr"] < 2.0
    # offload without partitioned gradients is not a plan
    assert run(orc, cf, it, env, 2, 1, 1, z=0, off=1)[0] == 1
    assert run(orc, cf, it, env, 2, 1, 1, z=1, off=1)[0] == 1
    # option masks
    nb = workloads.Bounds(g_max=64, zero_mask=0b0101, gc_mask=0b01, off_mask=0b01)
    assert run(orc, cf, it, env, 2, 1, 1, z=1, bounds=nb)[0] == 1
    assert run(orc, cf, it, env, 2, 1, 1, z=2, bounds=nb)[0] == 0
    assert run(orc, cf, it, env, 2, 1, 1, gc=1, bounds=nb)[0] == 1
    assert run(orc, cf, it, env, 2, 1, 1, z=2, off=1, bounds=nb)[0] == 1


def test_memory_exact_power_of_two_cases(orc):
    # all quantities are powers of two, so float32 arithmetic is exact and the
    # expected byte counts below are literal
    env = workloads.Env(gpu_mem_cap=BIG_CAP)
    mem = dict(mem_state=1, mem_act=32, mem_act_gc=2, mem_const=GIB)
    job = dict(P_bytes=float(2 ** 33), seq=1024, hidden=1024, t_fwd_sample=0.01, k_bwd=2, k_sync=1,
               k_opt=1e-11, k_opt_off=1e-9, k_off=1, k_swap=1, k_const=0.1, layers=8, gbatch=64, mbatch=2)
    coef, ints = make_job(job, mem)
    # d=4 t=1 p=2: Psi = 2^32; n = 64/(4*2) = 8, in flight min(2, 8) = 2; tok = 2^21; layers/stage 4
    # base = 2^21*4/1*2 = 2^24 ; A = 32*2^24 = 2^29
    _, x = run(orc, coef, ints, env, 4, 1, 2, z=0)
    assert x["Psi"] == 2 ** 32
    assert x["M_gpu"] == 8 * 2 ** 32 + 2 ** 29 + 2 ** 30
    assert x["H_host"] == 0
    _, x = run(orc, coef, ints, env, 4, 1, 2, z=1)          # 2 + 6/4 = 3.5
    assert x["M_gpu"] == 3.5 * 2 ** 32 + 2 ** 29 + 2 ** 30
    _, x = run(orc, coef, ints, env, 4, 1, 2, z=2)          # 1 + 7/4 = 2.75
    assert x["M_gpu"] == 2.75 * 2 ** 32 + 2 ** 29 + 2 ** 30
    _, x = run(orc, coef, ints, env, 4, 1, 2, z=3)          # 8/4 = 2
    assert x["M_gpu"] == 2 * 2 ** 32 + 2 ** 29 + 2 ** 30
    # checkpointing: 2*2^24 kept + one layer recomputed 32*2^21
    _, x = run(orc, coef, ints, env, 4, 1, 2, z=3, gc=1)
    assert x["M_gpu"] == 2 * 2 ** 32 + (2 ** 25 + 2 ** 26) + 2 ** 30
    # offload: GPU keeps the 2-byte weights (z2) or their shard (z3); host gets 7/d per GPU
    _, x = run(orc, coef, ints, env, 4, 1, 2, z=2, off=1)
    assert x["M_gpu"] == 2 ** 32 + 2 ** 29 + 2 ** 30
    assert x["H_host"] == (7 / 4) * 2 ** 32 * 8
    _, x = run(orc, coef, ints, env, 4, 1, 2, z=3, off=1)
    assert x["M_gpu"] == 2 ** 30 + 2 ** 29 + 2 ** 30
    # tensor parallel halves the activations, mem_state scales the state only
    _, x = run(orc, coef, ints, env, 4, 2, 1, z=0)           # Psi = 2^32, lay = 8, w = 1: base = 2^21*8/2 = 2^23
    assert x["M_gpu"] == 8 * 2 ** 32 + 32 * 2 ** 23 + 2 ** 30
    # fewer micro-batches than stages: only n = 64/(16*2) = 2 are in flight, not p = 4
    _, x = run(orc, coef, ints, env, 16, 1, 4, z=0)          # Psi = 2^31, lay = 2: base = 2^21*2*2 = 2^23
    assert x["n"] == 2 and x["M_gpu"] == 8 * 2 ** 31 + 32 * 2 ** 23 + 2 ** 30
    coef2, _ = make_job(job, dict(mem, mem_state=2))
    _, x = run(orc, coef2, ints, env, 4, 2, 1, z=0)
    assert x["M_gpu"] == 16 * 2 ** 32 + 32 * 2 ** 23 + 2 ** 30


def test_memory_thresholds_and_reason_bits(orc):
    mem = dict(mem_state=1, mem_act=32, mem_act_gc=2, mem_const=GIB)
    job = dict(P_bytes=float(2 ** 33), seq=1024, hidden=1024, t_fwd_sample=0.01, k_bwd=2, k_sync=1,
               k_opt=1e-11, k_opt_off=1e-9, k_off=1, k_swap=1, k_const=0.1, layers=8, gbatch=64, mbatch=2)
    coef, ints = make_job(job, mem)
    need = 2 ** 32 + 2 ** 29 + 2 ** 30            # z2 + offload on d=4,t=1,p=2 (previous test)
    host = (7 / 4) * 2 ** 32 * 8
    ok = workloads.Env(gpu_mem_cap=float(need))
    tight = workloads.Env(gpu_mem_cap=float(need - 512))
    assert run(orc, coef, ints, ok, 4, 1, 2, z=2, off=1, host=host)[0] == 0      # equality is feasible
    assert run(orc, coef, ints, tight, 4, 1, 2, z=2, off=1, host=host)[0] == 2
    assert run(orc, coef, ints, ok, 4, 1, 2, z=2, off=1, host=host - 4096)[0] == 4
    assert run(orc, coef, ints, tight, 4, 1, 2, z=2, off=1, host=0.0)[0] == 6
    # a plan that keeps nothing on the host fits a zero-byte tier
    assert run(orc, coef, ints, workloads.Env(gpu_mem_cap=BIG_CAP), 4, 1, 2, z=2, host=0.0)[0] == 0


def test_seven_billion_on_one_gpu_needs_offload(orc):
    # Sec. 7.2 (changing resource limits): on one 80 GB GPU a 7B-parameter
    # model trains only with ZeRO-Offload; Sec. 2.2: capping host memory below
    # the offloaded state makes that fail too.
    env = workloads.Env()
    N = 7e9
    job = dict(P_bytes=2 * N, seq=2048, hidden=4096, t_fwd_sample=0.2, k_bwd=2, k_sync=2, k_opt=5e-12,
               k_opt_off=5e-9, k_off=2, k_swap=2, k_const=0.05, layers=32, gbatch=32, mbatch=1)
    coef, ints = make_job(job)
    feasible = []
    for o in range(16):
        z, gc, off = o >> 2, (o >> 1) & 1, o & 1
        reason, _ = run(orc, coef, ints, env, 1, 1, 1, z=z, gc=gc, off=off, c=8, host=256 * GIB)
        if reason == 0:
            feasible.append((z, gc, off))
    assert feasible and all(off == 1 for _, _, off in feasible)
    reason, x = run(orc, coef, ints, env, 1, 1, 1, z=2, gc=1, off=1, c=8, host=64 * GIB)
    assert reason == 4 and x["H_host"] == pytest.approx(7 * 14e9, rel=1e-6)


def test_micro_batch_shift_of_a_plan(orc):
    """Sec. 4.1 "Gradient Accumulation", Table 1 (m, a belong to the plan): a plan
    with shift v runs micro-batches of mu * 2^v samples."""
    env = workloads.Env(B_intra=1e11, B_inter=1e10, B_pcie=1e10, gpu_mem_cap=BIG_CAP, gpus_per_node=8)
    spec = dict(P_bytes=4e9, seq=1024, hidden=2048, t_fwd_sample=0.002, k_bwd=2.0, k_sync=1.0, k_opt=1e-12, k_opt_off=1e-9,
                k_off=2.0, k_swap=2.0, k_const=0.25, layers=8, gbatch=64, mbatch=2)
    coef, ints = make_job(spec)
    f32 = lambda x: float(np.float32(x))                    # the descriptor and the environment hold float32 values
    tfs, k_opt, b_intra = f32(0.002), f32(1e-12), f32(1e11)
    run_v = lambda d, t, p, v, **kw: orc.eval_one(coef, ints, BOUNDS, env, d, t, p, kw.get("z", 0), kw.get("gc", 0), 0, 1,
                                                   BIG_CAP, v=v)[1]
    # one GPU: a * Tf_mb is the whole batch whatever the micro-batch size, and so is the iteration time
    for v in (0, 1, 2, 3):
        x = run_v(1, 1, 1, v)
        assert x["a"] == 64 / (2 * 2 ** v) and x["m"] == 1
        assert x["Tf_mb"] == pytest.approx(tfs * 2 * 2 ** v, rel=1e-12)
        assert x["T_iter"] == pytest.approx(64 * tfs * 3 + k_opt * 4e9 + 0.25, rel=1e-12)
    # data parallel over 4 GPUs, no overlap (k_sync = 1): T = a*Tf + a*Tb + T_dp, again the same for every size ...
    t_dp = 4e9 * 2 * 3 / 4 / b_intra
    for v in (0, 1, 2):
        x = run_v(4, 1, 1, v)
        assert x["a"] == 16 / (2 * 2 ** v)
        assert x["T_cc"] == pytest.approx(16 * tfs * 3 + t_dp, rel=1e-12)
    # ... but with overlap the last backward pass hides more of the synchronisation when it is longer:
    # T_cc = a*Tf + (a-1)*Tb + f(k; Tb, T_dp) with Tb = 2*Tf, Tf = t_fwd_sample * mu * 2^v
    coef2, _ = make_job(dict(spec, k_sync=3.0))
    prev = None
    for v in (0, 1, 2):
        x = orc.eval_one(coef2, ints, BOUNDS, env, 4, 1, 1, 0, 0, 0, 1, BIG_CAP, v=v)[1]
        tf = tfs * 2 * 2 ** v
        a = 16 / (2 * 2 ** v)
        want = a * tf + (a - 1) * 2 * tf + (((2 * tf) ** 3 + t_dp ** 3) ** (1 / 3))
        assert x["T_cc"] == pytest.approx(want, rel=1e-12)
        assert prev is None or x["T_cc"] < prev
        prev = x["T_cc"]
    # pipeline: m = b / (d * mu * 2^v) micro-batches, fill + steady state (m + p - 1)
    for v in (0, 1):
        x = run_v(2, 1, 4, v)
        m = 64 / (2 * 2 * 2 ** v)
        assert x["m"] == m and x["a"] == 1
        assert x["T_fwd"] == pytest.approx(tfs * 2 * 2 ** v / 4 * (m + 3), rel=1e-12)
    # activations grow with the micro-batch: exact float32 bytes for powers of two (no checkpointing)
    m0 = run_v(1, 1, 1, 0)["M_gpu"]
    m2 = run_v(1, 1, 1, 2)["M_gpu"]
    act0 = 34 * (2 * 1024 * 2048) * 8
    assert m0 == 8 * 4e9 + act0 + GIB and m2 == 8 * 4e9 + 4 * act0 + GIB
    # the shifted plan equals the unshifted plan of a job whose own micro-batch is larger, term by term
    _, ints8 = make_job(dict(spec, mbatch=8))
    a_ = orc.eval_one(coef, ints, BOUNDS, env, 2, 2, 2, 1, 1, 0, 1, BIG_CAP, v=2)[1]
    b_ = orc.eval_one(coef, ints8, BOUNDS, env, 2, 2, 2, 1, 1, 0, 1, BIG_CAP, v=0)[1]
    assert a_ == b_
