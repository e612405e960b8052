"""Host-side checks of the C ABI: the built library exports every function the
header declares, the Python binding mirrors the struct layouts, and the entry
points reject a null context without touching a device."""
import ctypes as C
import os
import re
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "rubick.h")


@pytest.fixture(scope="module")
def rk():
    import paper_2408_08586_amd as rk
    if not os.path.exists(rk.LIB_PATH):
        from paper_2408_08586_amd import build
        build.build(verbose=False)
    rk.load_library()
    return rk


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rk_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported(rk):
    names = declared_functions()
    assert {"rk_enumerate_plans", "rk_eval_candidates", "rk_best_plan", "rk_job_curves", "rk_schedule_round"} <= set(names)
    lib = rk.load_library()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in rubick.h but not exported"
    assert set(rk.EXPORTS) == set(names)
    for n in names:
        assert callable(getattr(rk, n)), f"binding lacks {n}"


def test_struct_layouts_match_the_header(rk):
    structs = ["rk_jobs", "rk_plan_bounds", "rk_plan_table", "rk_alloc_grid", "rk_env", "rk_cluster", "rk_assign", "rk_sla", "rk_samples", "rk_fit_options", "rk_fit_result", "rk_trace", "rk_sim_options", "rk_sim_result", "rk_nodes", "rk_place_entry", "rk_place_result", "rk_job_state"]
    prog = ['#include <stdio.h>', '#include <stddef.h>', '#include "rubick.h"', 'int main(void){']
    for s in structs:
        prog.append(f'printf("{s} %zu\\n", sizeof({s}));')
    fields = {"rk_plan_table": ["cap_triples", "h_triple_off", "n_triples", "n_jobs", "option_mask"],
              "rk_alloc_grid": ["cpu_mode", "n_mem", "mem_levels_gb", "mem_mode"],
              "rk_jobs": ["P_bytes", "ref_thr", "layers", "mbatch"],
              "rk_assign": ["mem_gb", "plan", "thr"],
              "rk_sla": ["tenant", "base_thr", "n_tenants", "quota_g", "quota_c"],
              "rk_samples": ["cpus", "thr", "max_samples"],
              "rk_fit_options": ["refit_threshold", "n_starts", "start_offsets"],
              "rk_fit_result": ["k_const", "theta", "rmsle_after", "iters"],
              "rk_trace": ["work", "delta"], "rk_sim_options": ["n_ticks", "gate"],
              "rk_sim_result": ["n_reconf", "held", "totals", "frozen"],
              "rk_nodes": ["gpus_per_node", "cpus_per_node", "mem_per_node_gb"],
              "rk_place_entry": ["node", "g", "c", "mem_gb"],
              "rk_place_result": ["n_placed", "n_failed", "in_order"],
              "rk_job_state": ["cur_seg", "cur_c", "floor_seg", "floor_c"]}
    for s, fs in fields.items():
        for f in fs:
            prog.append(f'printf("{s}.{f} %zu\\n", offsetof({s}, {f}));')
    prog.append("return 0;}")
    with tempfile.TemporaryDirectory() as d:
        src, exe = os.path.join(d, "a.c"), os.path.join(d, "a.out")
        open(src, "w").write("\n".join(prog))
        subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), src, "-o", exe], check=True)
        out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    want = dict(line.split() for line in out.strip().splitlines())
    py = {"rk_jobs": rk.rk_jobs, "rk_plan_bounds": rk.rk_plan_bounds, "rk_plan_table": rk.rk_plan_table,
          "rk_alloc_grid": rk.rk_alloc_grid, "rk_env": rk.rk_env, "rk_cluster": rk.rk_cluster, "rk_sla": rk.rk_sla,
          "rk_samples": rk.rk_samples, "rk_fit_options": rk.rk_fit_options, "rk_fit_result": rk.rk_fit_result,
          "rk_trace": rk.rk_trace, "rk_sim_options": rk.rk_sim_options, "rk_sim_result": rk.rk_sim_result,
          "rk_nodes": rk.rk_nodes, "rk_place_result": rk.rk_place_result, "rk_job_state": rk.rk_job_state}
    for s, cls in py.items():
        assert C.sizeof(cls) == int(want[s]), s
        for f in fields.get(s, []):
            assert getattr(cls, f).offset == int(want[f"{s}.{f}"]), f"{s}.{f}"
    assert rk.PLACE_DTYPE.itemsize == int(want["rk_place_entry"])
    for f in fields["rk_place_entry"]:
        assert rk.PLACE_DTYPE.fields[f][1] == int(want[f"rk_place_entry.{f}"])
    assert rk.ASSIGN_DTYPE.itemsize == int(want["rk_assign"])
    for f in fields["rk_assign"]:
        assert rk.ASSIGN_DTYPE.fields[f][1] == int(want[f"rk_assign.{f}"])


def test_null_context_is_rejected(rk):
    lib = rk.load_library()
    null = C.c_void_p(0)
    assert lib.rk_sync(null) == rk.RK_ERR_INVALID_ARG
    assert lib.rk_destroy(null) == rk.RK_ERR_INVALID_ARG
    assert lib.rk_create(null, 0, null) == rk.RK_ERR_INVALID_ARG
    assert lib.rk_enumerate_plans(null, null, null, null) == rk.RK_ERR_INVALID_ARG
    assert lib.rk_schedule_round(null, null, null, null, null, null, null, null) == rk.RK_ERR_INVALID_ARG
    assert rk.rk_last_error(null) == "null context"


def test_product_path_has_no_oracle_or_cpu_fallback():
    pkg = os.path.join(ROOT, "paper_2408_08586_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "rk_oracle" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert bench.count("import oracle") == 1        # only inside cpu_baseline()


def test_missing_library_fails_loudly(rk, monkeypatch):
    monkeypatch.setattr(rk, "_lib", None)
    monkeypatch.setattr(rk, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "librubick.so"))
    with pytest.raises(RuntimeError):
        rk.load_library()
