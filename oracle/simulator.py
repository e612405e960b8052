"""Discrete-time cluster simulation on the CPU oracle (paper Sec. 7.4: a
discrete-time simulator replays job traces through the scheduling policy;
Sec. 5.2, paragraph on the reconfiguration penalty: the rule compares
(T - N*delta)/T with a threshold of 0.97).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.

Every tick of length dt, at time t = k*dt:
  1. a job is active when it has arrived (arrival <= t) and is not finished;
  2. an active job that runs is frozen for this tick unless one more
     reconfiguration keeps (T - (N+1)*delta) > gate*T, with T the time it has
     held resources and N its reconfigurations so far (the division-free form
     of the paper's ratio);
  3. one round over the resource sensitivity curves (computed once: they do
     not depend on the cluster's state): inactive jobs take no part, frozen
     jobs keep their GPUs and CPUs.  policy "greedy": the from-scratch greedy
     with the frozen jobs charged first; policy "loop": Algorithm 1's Schedule
     loop from what the jobs hold (running jobs keep it unless a job with a
     higher slope takes it; the policy is triggered every tick); policy
     "nodes": the same loop with ScheduleJob searching node by node, from the
     placement the last tick left (nodes = (n, GPUs, CPUs, GiB per node));
  4. a running job whose (GPUs, CPUs, plan) changed while it keeps running is
     reconfigured: N += 1 and delta seconds of checkpoint-resume are owed;
     starting from or stopping at zero GPUs is free;
  5. a job that holds GPUs first pays owed seconds out of the tick, then
     trains: progress += thr * (dt - paid); it finishes inside the tick at
     t + paid + remaining/thr.
All times and progress are float64, the throughput is the round's float32.

Readings (the paper gives the ratio and the threshold only): what T and N
count, that the gate is applied before the round by freezing, that starts and
preemptions are free, the tick structure.  PARITY UNPINNED as a reading; pinned
by closed forms for lone jobs, hand cases for the gate and conservation laws.
"""
from __future__ import annotations

import numpy as np

from . import PLACE_DTYPE, frozen_round, reschedule, reschedule_nodes


def level_of(grid, c, g):
    """CPU level whose cost at g GPUs is c (the first one)."""
    for i, lv in enumerate(grid.cpu_levels):
        if (int(lv) * int(g) if grid.cpu_mode else int(lv)) == int(c):
            return i
    raise ValueError("no CPU level costs %d at %d GPUs" % (c, g))


def simulate(ref_thr, table, grid, cluster, best_thr, best_plan, curve_thr, arrival, work, delta, dt, n_ticks,
             gate=0.97, trace=False, policy="greedy", nodes=None):
    J = table.n_jobs
    arrival, work, delta = (np.asarray(a, np.float64) for a in (arrival, work, delta))
    dt, gate = float(dt), float(gate)
    done = np.zeros(J, bool)
    g_prev, c_prev = np.zeros(J, np.uint32), np.zeros(J, np.uint32)
    plan_prev = np.full(J, 0xFFFFFFFF, np.uint32)
    seg_prev, lvl_prev = np.full(J, -1, np.int32), np.zeros(J, np.uint32)
    held = np.zeros(J, np.float64)            # T: time with resources
    n_reconf = np.zeros(J, np.uint32)         # N
    owed = np.zeros(J, np.float64)            # checkpoint-resume seconds still to pay
    progress = np.zeros(J, np.float64)
    finish = np.full(J, -1.0, np.float64)
    gpus_in_use = np.zeros(n_ticks, np.uint32)
    totals = np.zeros(n_ticks, np.float64)
    frozen_count = np.zeros(n_ticks, np.uint32)
    history, placements = [], []
    where = (np.zeros(J + 1, np.uint32), np.zeros(0, PLACE_DTYPE))       # nobody is anywhere yet
    for k in range(n_ticks):
        t = float(k) * dt
        active = (arrival <= t) & ~done
        running = active & (g_prev > 0)
        with np.errstate(invalid="ignore"):                 # an infinite gate times a zero time
            may_move = held - (n_reconf.astype(np.float64) + 1.0) * delta > gate * held
        frozen = running & ~may_move
        state = np.where(~active, 1, np.where(frozen, 2, 0)).astype(np.uint8)
        if policy == "nodes":
            res = reschedule_nodes(ref_thr, table, grid, *nodes, best_thr, best_plan, curve_thr, seg_prev, lvl_prev, where,
                                   state=state)
            assert res is not None, "what the jobs hold and where they are have come apart"
            assign, p_off, p_ent, total, _ = res
            where = (p_off, p_ent)
        elif policy == "loop":
            assign, total, _ = reschedule(ref_thr, table, grid, cluster, best_thr, best_plan, curve_thr, seg_prev, lvl_prev,
                                          state=state)
        else:
            assign, total, _ = frozen_round(ref_thr, table, grid, cluster, best_thr, best_plan, curve_thr, state, seg_prev,
                                            lvl_prev)
        gpus_in_use[k] = assign["g"].sum()
        totals[k] = total
        frozen_count[k] = frozen.sum()
        for j in np.flatnonzero(active):
            g, c, plan, thr = int(assign["g"][j]), int(assign["c"][j]), int(assign["plan"][j]), float(assign["thr"][j])
            if g_prev[j] > 0 and g > 0 and (g != g_prev[j] or c != c_prev[j] or plan != plan_prev[j]):
                n_reconf[j] += 1
                owed[j] = owed[j] + delta[j]
            if g > 0:
                held[j] = held[j] + dt
                paid = min(owed[j], dt)
                owed[j] = owed[j] - paid
                train = dt - paid
                gain = thr * train
                if progress[j] + gain >= work[j]:
                    finish[j] = t + paid + (work[j] - progress[j]) / thr
                    progress[j] = work[j]
                    done[j] = True
                    g = 0
                else:
                    progress[j] = progress[j] + gain
            if g > 0:
                seg = int(np.searchsorted(table.seg_g[table.seg_off[j]:table.seg_off[j + 1]], g))
                g_prev[j], c_prev[j], plan_prev[j], seg_prev[j], lvl_prev[j] = g, c, plan, seg, level_of(grid, c, g)
            else:
                g_prev[j], c_prev[j], plan_prev[j], seg_prev[j], lvl_prev[j] = 0, 0, 0xFFFFFFFF, -1, 0
        if trace:
            history.append(assign.copy())
            placements.append(where)
    out = dict(finish=finish, n_reconf=n_reconf, progress=progress, held=held, gpus_in_use=gpus_in_use, totals=totals,
               frozen=frozen_count)
    if trace:
        out["history"] = history
        out["placements"] = placements
    return out
