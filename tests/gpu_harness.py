"""Helpers for the GPU tests: run the library's entry points on a workload and
bring the results back as numpy arrays.  Allocation and marshalling only."""
from __future__ import annotations

import numpy as np

import paper_2408_08586_amd as rk


class DeviceRun:
    def __init__(self, wl, device="cuda:0"):
        import torch
        self.torch = torch
        self.wl = wl
        self.device = device
        self.ctx = rk.rk_create(0)
        self.jobs = rk.Jobs(wl.coef, wl.ints, device)
        self.bounds = rk.make_bounds(wl.bounds)
        self.grid = rk.make_grid(wl.grid)
        self.env = rk.make_env(wl.env)
        self.cluster = rk.make_cluster(wl.cluster)
        self.n_rows = len(wl.grid.cpu_levels) * len(wl.grid.mem_levels_gb)
        self.table = None

    def close(self):
        rk.rk_destroy(self.ctx)

    def f32(self, n):
        return self.torch.empty(max(int(n), 4), dtype=self.torch.float32, device=self.device)

    def i32(self, n):
        return self.torch.empty(max(int(n), 4), dtype=self.torch.int32, device=self.device)

    def enumerate(self):
        self.table = rk.enumerate_to_table(self.ctx, self.jobs, self.bounds, self.device)
        return self.table

    def table_numpy(self):
        t = self.table
        return dict(triple_off=rk.u32(t.triple_off), triples=t.unpack_triples(), seg_off=rk.u32(t.seg_off),
                    seg_g=rk.u32(t.seg_g)[:t.n_segs], seg_first=rk.u32(t.seg_first)[:t.n_segs])

    def eval(self, jb=0, je=None, want_feas=True):
        je = self.wl.n_jobs if je is None else je
        n = self.table.n_candidates(self.n_rows, jb, je)
        thr = self.f32(n)
        feas = self.torch.empty(max(n, 16), dtype=self.torch.uint8, device=self.device) if want_feas else None
        need = rk.rk_eval_candidates(self.ctx, self.jobs, self.table.c, self.grid, self.env, jb, je, thr, feas)
        assert need == n
        return thr, feas, n

    def best(self, thr, jb=0, je=None):
        je = self.wl.n_jobs if je is None else je
        n = self.table.n_segments(self.n_rows, jb, je)
        bt, bp = self.f32(n), self.i32(n)
        need = rk.rk_best_plan(self.ctx, self.table.c, self.grid, jb, je, thr, bt, bp)
        assert need == n
        return bt, bp, n

    def eval_best(self, jb=0, je=None, want_feas=True):
        """Evaluation and best plan in one pass: (thr, feas, best_thr, best_plan, candidates, segment entries)."""
        je = self.wl.n_jobs if je is None else je
        n = self.table.n_candidates(self.n_rows, jb, je)
        ns = self.table.n_segments(self.n_rows, jb, je)
        thr, bt, bp = self.f32(n), self.f32(ns), self.i32(ns)
        feas = self.torch.empty(max(n, 16), dtype=self.torch.uint8, device=self.device) if want_feas else None
        rk.rk_eval_best_plan(self.ctx, self.jobs, self.table.c, self.grid, self.env, jb, je, thr, bt, bp, feas=feas)
        return thr, feas, bt, bp, n, ns

    def curves(self, bt, bp, jb=0, je=None):
        je = self.wl.n_jobs if je is None else je
        n = self.table.n_segments(self.n_rows, jb, je)
        ct, cp, cg = self.f32(n), self.i32(n), self.i32(n)
        rk.rk_curves(self.ctx, self.table.c, self.grid, jb, je, bt, bp, ct, cp, cg)
        return ct, cp, cg

    def fused(self, jb=0, je=None, want_best=True):
        je = self.wl.n_jobs if je is None else je
        n = self.table.n_segments(self.n_rows, jb, je)
        bt, bp = (self.f32(n), self.i32(n)) if want_best else (None, None)
        ct, cp, cg = self.f32(n), self.i32(n), self.i32(n)
        rk.rk_job_curves(self.ctx, self.jobs, self.table.c, self.grid, self.env, jb, je, bt, bp, ct, cp, cg)
        return bt, bp, ct, cp, cg, n

    def allocate(self, bt, bp, ct, cluster=None, jb=0, je=None):
        je = self.wl.n_jobs if je is None else je
        assign = rk.new_assign(je - jb, self.device)
        total = self.f32(1)
        rk.rk_allocate(self.ctx, self.jobs.ref_thr, self.table.c, self.grid,
                       self.cluster if cluster is None else cluster, jb, je, bt, bp, ct, assign, total)
        rk.rk_sync(self.ctx)
        return rk.assign_to_numpy(assign), float(total[0].item())

    def schedule_round(self):
        assign = rk.new_assign(self.wl.n_jobs, self.device)
        total = self.f32(1)
        rk.rk_schedule_round(self.ctx, self.jobs, self.bounds, self.grid, self.env, self.cluster, assign, total)
        rk.rk_sync(self.ctx)
        return rk.assign_to_numpy(assign), float(total[0].item())

    def dev_f32(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device)

    def dev_u32(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).to(self.device)

    def host(self, t, n=None):
        a = t.cpu().numpy()
        return a if n is None else a[:n]
