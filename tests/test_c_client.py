"""The boundary from plain C: tests/capi/plan_from_c.c is compiled with gcc as strict C99 against
include/mgwfbp.h, linked with the library and run; its output is compared with the CPU oracle."""
import os
import subprocess

import pytest

from oracle import planner as op
from paper_1811_11141_amd import binding as mg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_is_c99_and_planner_runs_from_c(tmp_path, golden):
    exe = str(tmp_path / "plan_from_c")
    libdir = os.path.dirname(mg.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "capi", "plan_from_c.c"), "-o", exe,
           "-L", libdir, "-l:libmgwfbp.so", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, (run.stdout, run.stderr[-2000:])
    rows = {l.split()[0]: l.split() for l in run.stdout.strip().splitlines()}
    p, tb, a, b = [2500000] * 3, [0.9] * 3, 1.0, 1.0e-6
    t_best, _ = op.brute_force(p, tb, 0.0, a, b)
    t_wfbp = op.wfbp_timeline(p, tb, 0.0, a, b)[1]
    t_rule = op.simulate(p, tb, 0.0, a, b, op.algorithm1(p, tb, 0.0, a, b))
    t_single = op.simulate(p, tb, 0.0, a, b, [2, 3])
    assert float(rows["optimal"][4]) == t_best and int(rows["optimal"][2]) == 2
    assert float(rows["theorem1"][4]) == t_rule
    assert float(rows["wfbp"][4]) == t_wfbp == float(rows["optimal"][6]) and int(rows["wfbp"][2]) == 3
    assert float(rows["single"][4]) == t_single and int(rows["single"][2]) == 1
    # the hand-worked example's three values (Theorem 1's rule is not optimal here)
    ex = golden["hand_worked_three_layers"]
    assert ex["p"] == p and ex["tb_ms"] == tb
    assert t_best == pytest.approx(32.9) and t_rule == pytest.approx(33.7) and t_wfbp == pytest.approx(33.9)
    a8, b8 = op.table2_cost("ring", 8, 0.04526, 8.0e-7, 0.0)
    assert float(rows["ring8"][2]) == pytest.approx(a8, rel=1e-15) and float(rows["ring8"][4]) == pytest.approx(b8, rel=1e-15)
    assert a8 == pytest.approx(0.63364)        # Section V-A: 633.64 us start-up on 8 nodes
