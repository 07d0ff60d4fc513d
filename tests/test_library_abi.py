"""The C-ABI library loads and exports every entry point include/*.h declares (no GPU needed),
and the host-side validation answers without touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2508_21613_amd import binding as B
from paper_2508_21613_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(chm_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_entry_point_is_exported():
    names = declared_functions()
    assert "chm_load_scenario" in names and "chm_score_plans" in names and "chm_search_best" in names
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.SYMBOLS) == names


def test_struct_layouts_match_the_header(tmp_path):
    """sizes and field offsets of every structure of the binding against what a C compiler makes of include/chm.h"""
    import subprocess
    structs = {"chm_scenario_desc": B.Desc, "chm_family": B.Family, "chm_space": B.Space, "chm_best": B.Best,
               "chm_timing": B.Timing, "chm_selection": B.Selection, "chm_replan_desc": B.ReplanDesc, "chm_replan_plan": B.ReplanPlan}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "chm.h"', '#include "chm_measure.h"', 'int main(void) {']
    for cname, cls in structs.items():
        lines.append('  printf("%s %%zu\\n", sizeof(%s));' % (cname, cname))
        for field, _ in cls._fields_:
            lines.append('  printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (cname, field, cname, field))
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)], check=True)
    want = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, cls in structs.items():
        assert C.sizeof(cls) == int(want[cname]), cname
        for field, _ in cls._fields_:
            assert getattr(cls, field).offset == int(want["%s.%s" % (cname, field)]), (cname, field)
    assert C.sizeof(B.Family) == 32 and C.sizeof(B.Space) == 8 + 3 * 32 + 8


def test_error_strings_and_argument_checks_need_no_device():
    assert B.strerror(0) == "ok" and "memory" in B.strerror(B.ERR_NO_FEASIBLE)
    sc = synth.small_random(1)
    for key, val in [("L", 0), ("L", 129), ("PP", 0), ("DP", 17), ("M", 257), ("failed_nodes", [0, 0]),
                     ("failed_nodes", [10 ** 6]), ("horizon_steps", 0), ("mem_cap_mib", 0), ("comm_us", -1),
                     ("fwd_us", np.zeros(sc["L"], np.int32))]:
        with pytest.raises(B.ChmError) as e:
            B.Scenario(dict(sc, **{key: val}))
        assert e.value.code == B.ERR_ARG, key
    wide = synth.scenario(128, 32, 2, 4, np.ones(128, np.int32), np.ones(128, np.int32), np.ones(128, np.int32),
                          [0], 0, 1000)
    with pytest.raises(B.ChmError) as e:
        B.Scenario(wide)
    assert e.value.code == B.ERR_OVERFLOW
    assert B.lib().chm_plan_space(None, None) == B.ERR_ARG
    assert B.lib().chm_search_best(None, 7, None, None) == B.ERR_ARG
    assert B.lib().chm_score_plans(None, 0, 0, None, None) == B.ERR_ARG


def test_no_cpu_fallback_without_a_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.ChmError) as e:
        B.Scenario(synth.small_random(1))
    assert e.value.code == B.ERR_HIP
    with pytest.raises(B.ChmError) as e:
        B.replan(synth.replan_case(5, 10, 3, 3, [4], 12, (1, 4), (1, 6)), stream=0)
    assert e.value.code == B.ERR_HIP


def test_objective_comparison_is_exact():
    """Optimization Problem: (H - t_trans) / t_step, compared without rounding"""
    from fractions import Fraction
    rng = np.random.default_rng(3)
    for _ in range(2000):
        H = int(rng.integers(1, 2 ** 50))
        a = {"t_step_us": int(rng.integers(1, 2 ** 40)), "t_trans_us": int(rng.integers(0, 2 ** 50))}
        b = {"t_step_us": int(rng.integers(1, 2 ** 40)), "t_trans_us": int(rng.integers(0, 2 ** 50))}
        fa, fb = Fraction(H - a["t_trans_us"], a["t_step_us"]), Fraction(H - b["t_trans_us"], b["t_step_us"])
        assert B.compare_objective(a, b, H) == (fa > fb) - (fa < fb)
    # differences far below double precision, and exact ties
    big = 2 ** 61
    assert B.compare_objective({"t_step_us": big, "t_trans_us": 0}, {"t_step_us": big + 1, "t_trans_us": 0}, big) == 1
    assert B.compare_objective({"t_step_us": 3, "t_trans_us": 10}, {"t_step_us": 6, "t_trans_us": 0}, 20) == 0
    assert B.compare_objective({"t_step_us": 2, "t_trans_us": 40}, {"t_step_us": 1, "t_trans_us": 30}, 20) == 0   # -10 and -10
    assert B.compare_objective({"t_step_us": 2, "t_trans_us": 50}, {"t_step_us": 1, "t_trans_us": 30}, 20) == -1  # -15 and -10
    with pytest.raises(B.ChmError):
        B.compare_objective({"t_step_us": 0, "t_trans_us": 0}, {"t_step_us": 1, "t_trans_us": 0}, 5)


def test_replan_argument_checks_need_no_device():
    rp = synth.replan_case(5, 10, 3, 3, [4], 12, (1, 4), (1, 6))
    for key, val in [("L", 0), ("old_pp", 0), ("old_dp", 17), ("dp_min", 0), ("dp_max", 17), ("pp_min", 0), ("pp_max", 33),
                     ("micro_batches", 0), ("horizon_us", 0), ("failed_nodes", [1, 1]), ("failed_nodes", [9]), ("mem_cap_mib", 0),
                     ("allreduce_us", -1), ("fwd_us", np.zeros(10, np.int32))]:
        with pytest.raises(B.ChmError) as e:
            B.replan(dict(rp, **{key: val}), stream=0)
        assert e.value.code == B.ERR_ARG, key
