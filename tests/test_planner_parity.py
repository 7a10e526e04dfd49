"""Host logic of the library (planner, plan tables, error paths) against the CPU oracle.
No GPU is needed: nothing here launches a kernel."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import planner as op
from paper_1811_11141_amd import binding as mg
from paper_1811_11141_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def plan_for(w, mode, a=None, b=None, tf=0.0):
    return mg.mgwfbp_plan(w.p, w.tb_ms, tf, w.a_ms if a is None else a,
                          w.b_ms_per_byte if b is None else b, w.n_workers, mode)


def oracle_args(w, a=None, b=None, tf=0.0):
    return (w.p.tolist(), w.tb_ms.tolist(), tf, w.a_ms if a is None else a,
            w.b_ms_per_byte if b is None else b)


def test_library_exports_every_declared_symbol():
    """Every function any header under include/ declares is exported by the built library, and
    the binding lists exactly those names (the method's in mgwfbp.h, the benchmark's probes in
    mgwfbp_probe.h)."""
    import glob
    lib = C.CDLL(mg.LIB_PATH)
    seen = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        hdr = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)      # declarations, not prose
        declared = set(re.findall(r"\b(mgwfbp_[a-z0-9_]+)\s*\(", hdr))
        assert declared, path
        want = mg.PROBE_EXPORTS if path.endswith("mgwfbp_probe.h") else mg.EXPORTS
        assert declared == set(want), (path, declared ^ set(want))
        for name in declared:
            assert hasattr(lib, name), name
        seen |= declared
    assert seen == set(mg.EXPORTS) | set(mg.PROBE_EXPORTS)


def test_optimal_equals_brute_force_tiny_nets():
    """Config 1: L = 8, all 128 partitions, many seeds; the optimum value is unique."""
    mismatched_greedy = 0
    for seed in range(120):
        w = wl.tiny_workload(seed)
        args = oracle_args(w)
        t_best, _ = op.brute_force(*args)
        pl = plan_for(w, mg.MODE_OPTIMAL)
        inf = pl.info()
        assert inf["t_iter_ms"] == t_best, seed
        # the plan the library returns really has that cost under the oracle's evaluator
        assert op.simulate(*args, pl.merged_layers()) == t_best
        assert inf["t_iter_wfbp_ms"] == op.wfbp_timeline(*args)[1]
        g = plan_for(w, mg.MODE_PAPER_GREEDY)
        mismatched_greedy += g.info()["t_iter_ms"] > t_best
    assert mismatched_greedy > 0        # Theorem 1's rule is not always optimal


@pytest.mark.parametrize("L", [1, 2, 3, 5, 11])
def test_optimal_equals_brute_force_other_sizes(L):
    rng = np.random.default_rng(100 + L)
    for _ in range(25 if L < 11 else 6):
        w = wl.tiny_workload(int(rng.integers(1 << 30)), L=L)
        a = float(rng.choice([0.0, 0.05, 0.5, 2.0, 20.0]))
        b = float(rng.choice([0.0, 1e-6, 1e-4]))
        tf = float(rng.uniform(0, 5))
        args = oracle_args(w, a, b, tf)
        pl = plan_for(w, mg.MODE_OPTIMAL, a, b, tf)
        assert pl.info()["t_iter_ms"] == op.brute_force(*args)[0]


def test_optimal_equals_brute_force_twelve_layers():
    """L = 12: 2048 partitions, the largest size the brute force is asked for."""
    for seed in (1, 2, 3):
        w = wl.tiny_workload(seed, L=12)
        for a in (0.1, 0.5, 2.0):
            pl = plan_for(w, mg.MODE_OPTIMAL, a=a)
            assert pl.info()["t_iter_ms"] == op.brute_force(*oracle_args(w, a=a))[0]


def test_plan_properties_hypothesis():
    """Random shapes and cost constants: optimal <= rule of Theorem 1 <= WFBP, optimal <= single,
    the returned plan costs what it claims under the oracle's evaluator, groups are contiguous."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=150, deadline=None, derandomize=True)
    @given(st.lists(st.tuples(st.integers(1, 10**7), st.floats(0.0, 5.0)), min_size=1, max_size=40),
           st.floats(0.0, 3.0), st.floats(0.0, 1e-5), st.floats(0.0, 10.0))
    def check(layers, a, b, tf):
        p = [x[0] for x in layers]
        tb = [x[1] for x in layers]
        L = len(p)
        args = (p, tb, tf, a, b)
        res = {}
        for mode in (mg.MODE_OPTIMAL, mg.MODE_PAPER_GREEDY, mg.MODE_WFBP, mg.MODE_SINGLE):
            pl = mg.mgwfbp_plan(p, tb, tf, a, b, 8, mode)
            inf = pl.info()
            assert inf["t_iter_ms"] == op.simulate(*args, pl.merged_layers())
            gol = inf["group_of_layer"].tolist()
            assert gol[L - 1] == 0 and all(gol[l] - gol[l + 1] in (0, 1) for l in range(L - 1))
            assert int(inf["group_elems"].sum()) == sum(p)
            res[mode] = inf["t_iter_ms"]
        tol = 1e-12 * max(1.0, res[mg.MODE_WFBP])
        assert res[mg.MODE_OPTIMAL] <= res[mg.MODE_PAPER_GREEDY] + tol
        assert res[mg.MODE_PAPER_GREEDY] <= res[mg.MODE_WFBP] + tol
        assert res[mg.MODE_OPTIMAL] <= res[mg.MODE_SINGLE] + tol
        assert mg.mgwfbp_plan(p, tb, tf, a, b, 8, mg.MODE_PAPER_GREEDY).merged_layers() == op.algorithm1(*args)

    check()


def test_every_partition_evaluates_like_the_oracle():
    w = wl.tiny_workload(5, L=6)
    args = oracle_args(w)
    for m in op.all_merge_sets(6):
        pl = mg.mgwfbp_plan_explicit(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, 4, m)
        assert pl.info()["t_iter_ms"] == op.simulate(*args, m)
        assert pl.merged_layers() == sorted(m, reverse=True)
        assert [[l + 1 for l in g] for g in pl.groups()] == op.groups_from_merged(6, m)


def test_greedy_mode_is_algorithm1():
    rng = np.random.default_rng(21)
    for _ in range(300):
        L = int(rng.integers(1, 14))
        w = wl.tiny_workload(int(rng.integers(1 << 30)), L=L)
        a = float(rng.choice([0.05, 0.5, 1.0, 2.0]))
        pl = plan_for(w, mg.MODE_PAPER_GREEDY, a=a)
        assert pl.merged_layers() == op.algorithm1(*oracle_args(w, a=a))


def test_golden_cases_through_the_library(golden):
    ex = golden["hand_worked_three_layers"]
    mk = lambda mode: mg.mgwfbp_plan(ex["p"], ex["tb_ms"], 0.0, ex["a_ms"], ex["b_ms_per_byte"], 8, mode)
    assert mk(mg.MODE_OPTIMAL).info()["t_iter_ms"] == pytest.approx(ex["optimum"], rel=1e-12)
    assert mk(mg.MODE_OPTIMAL).merged_layers() == [2]
    g = mk(mg.MODE_PAPER_GREEDY)
    assert g.merged_layers() == ex["theorem1_merged"]
    assert g.info()["t_iter_ms"] == pytest.approx(ex["t_iter"]["3,2"], rel=1e-12)
    assert mk(mg.MODE_WFBP).info()["t_iter_ms"] == pytest.approx(ex["t_iter"][""], rel=1e-12)
    assert mk(mg.MODE_SINGLE).info()["t_iter_ms"] == pytest.approx(ex["t_iter"]["3,2"], rel=1e-12)
    for c in golden["hand_worked_traces"]["cases"]:
        pl = mg.mgwfbp_plan(c["p"], c["tb_ms"], 0.0, c["a_ms"], c["b_ms_per_byte"], 8,
                            mg.MODE_PAPER_GREEDY)
        assert pl.merged_layers() == c["merged"]
        assert pl.info()["t_iter_ms"] == pytest.approx(c["t_iter"], rel=1e-12)


def test_modes_wfbp_and_single_and_offsets():
    w = wl.tiny_workload(9)
    L = w.L
    wf = plan_for(w, mg.MODE_WFBP).info()
    assert wf["n_groups"] == L
    assert wf["group_of_layer"].tolist() == list(range(L - 1, -1, -1))
    assert wf["group_elems"].tolist() == w.p[::-1].tolist()
    assert wf["t_iter_ms"] == wf["t_iter_wfbp_ms"]
    sg = plan_for(w, mg.MODE_SINGLE).info()
    assert sg["n_groups"] == 1 and int(sg["group_elems"][0]) == w.P
    # arrival order: the top layer sits at offset 0, no padding between layers
    off = 0
    for l in range(L - 1, -1, -1):
        assert int(sg["offset_in_group"][l]) == off
        off += int(w.p[l])
    assert sg["t_iter_ms"] == pytest.approx(sum(w.tb_ms) + w.a_ms + w.b_ms_per_byte * 4 * w.P, rel=1e-12)


def test_timeline_matches_eq6_to_8():
    w = wl.tiny_workload(10)
    pl = plan_for(w, mg.MODE_WFBP)
    tl = pl.timeline()
    args = oracle_args(w)
    assert tl["mu_b"].tolist() == op.backward_finish(w.tb_ms.tolist(), 0.0)
    tau_c, t_iter = op.wfbp_timeline(*args)
    assert tl["group_start"].tolist() == tau_c[::-1]
    assert tl["group_finish"][-1] == t_iter


def test_cnn_plans_are_consistent():
    for name in wl.CNN_WORKLOADS:
        w = wl.cnn_workload(name)
        args = oracle_args(w)
        opt, gr = plan_for(w, mg.MODE_OPTIMAL), plan_for(w, mg.MODE_PAPER_GREEDY)
        t_opt, t_gr = opt.info()["t_iter_ms"], gr.info()["t_iter_ms"]
        t_wf = op.wfbp_timeline(*args)[1]
        t_single = op.simulate(*args, range(2, w.L + 1))
        assert t_opt == op.simulate(*args, opt.merged_layers())
        assert gr.merged_layers() == op.algorithm1(*args)
        assert t_opt <= t_gr <= t_wf * (1 + 1e-12)
        assert t_opt <= t_single
        inf = opt.info()
        assert int(inf["group_elems"].sum()) == w.P


@pytest.mark.parametrize("name", ["resnet50", "googlenet", "alexnet", "vgg16"])
@pytest.mark.parametrize("a_ms,g_eff", [(0.1, 2e12), (0.5, 2e12), (2.0, 2e12), (0.5, 2e13), (0.02, 2e14)])
def test_full_size_plans_admit_no_better_neighbour(name, a_ms, g_eff):
    """Where brute force cannot go (L up to 161): necessary conditions of optimality, all
    evaluated by the oracle's simulate.  No plan reached by toggling one layer (for the short
    nets: any two layers) of the optimal merge set, no random merge set, and none of the named
    plans (no merging, single group, Theorem 1's rule) finishes earlier."""
    w = wl.cnn_workload(name, a_ms=a_ms, g_eff=g_eff)
    args = oracle_args(w)
    pl = plan_for(w, mg.MODE_OPTIMAL)
    m_opt = set(pl.merged_layers())
    t_opt = pl.info()["t_iter_ms"]
    assert t_opt == op.simulate(*args, m_opt)
    cand = list(range(2, w.L + 1))
    for l in cand:
        assert op.simulate(*args, m_opt ^ {l}) >= t_opt, f"toggling layer {l} is better"
    if w.L <= 32:
        for i, l1 in enumerate(cand):
            for l2 in cand[i + 1:]:
                assert op.simulate(*args, m_opt ^ {l1, l2}) >= t_opt, (l1, l2)
    rng = np.random.default_rng(w.L)
    for _ in range(300):
        density = rng.random()
        m = {l for l in cand if rng.random() < density}
        assert op.simulate(*args, m) >= t_opt
    assert op.simulate(*args, op.algorithm1(*args)) >= t_opt
    assert op.wfbp_timeline(*args)[1] >= t_opt and op.simulate(*args, cand) >= t_opt


def test_error_paths():
    lib = mg.raw()
    p = (C.c_uint64 * 3)(10, 20, 30)
    tb = (C.c_double * 3)(1.0, 1.0, 1.0)
    h = C.c_void_p()
    call = lambda L=3, pp=p, tt=tb, tf=0.0, a=0.5, b=1e-6, N=4, mode=0, out=C.byref(h): \
        lib.mgwfbp_plan(L, pp, tt, tf, a, b, N, mode, out)
    assert call(L=0) == mg.EINVAL and "L" in mg.last_error()
    assert call(N=0) == mg.EINVAL
    assert call(pp=None) == mg.EINVAL
    assert call(tt=None) == mg.EINVAL
    assert call(a=-1.0) == mg.EINVAL
    assert call(b=float("nan")) == mg.EINVAL
    assert call(tf=float("inf")) == mg.EINVAL
    assert call(mode=9) == mg.EINVAL
    assert call(out=None) == mg.EINVAL
    assert call(pp=(C.c_uint64 * 3)(10, 0, 30)) == mg.EINVAL and "p_elems[1]" in mg.last_error()
    assert call(tt=(C.c_double * 3)(1.0, -2.0, 1.0)) == mg.EINVAL
    # sizes whose byte counts would leave 64 bits: one layer, or the sum, beyond 2^40 elements
    assert call(pp=(C.c_uint64 * 3)(10, 2**40 + 1, 30)) == mg.EINVAL and "2^40" in mg.last_error()
    assert call(pp=(C.c_uint64 * 3)(2**39, 2**39, 1)) == mg.EINVAL and "p_elems[0..2]" in mg.last_error()
    assert call(pp=(C.c_uint64 * 3)(2**64 - 1, 2**64 - 1, 2)) == mg.EINVAL
    assert h.value is None
    assert call() == mg.OK and h.value
    # launches before bind are a state error; no kernel is launched
    assert lib.mgwfbp_pack_reduce_unpack(h, -1, None, 0, None) == mg.ESTATE
    assert lib.mgwfbp_step(h, -1, 0.1, 0.9, None, 0, None) == mg.ESTATE
    assert lib.mgwfbp_bind(h, None, None, None, None) == mg.EINVAL
    n = C.c_size_t()
    assert lib.mgwfbp_workspace_bytes(h, 7, C.byref(n)) == mg.EINVAL
    assert lib.mgwfbp_workspace_bytes(h, -1, C.byref(n)) == mg.OK and n.value == 5 * 64 * 4
    assert lib.mgwfbp_plan_set_option(h, mg.OPT_TILE_ELEMS, 1000) == mg.EINVAL
    assert lib.mgwfbp_plan_set_option(h, mg.OPT_TILE_ELEMS, 4096) == mg.OK
    assert lib.mgwfbp_plan_set_option(h, 99, 1) == mg.EINVAL
    for bad in (-2, 1, 7, 12):
        assert lib.mgwfbp_plan_set_option(h, mg.OPT_UPDATE_WGS_PER_CU, bad) == mg.EINVAL
    for good in (-1, 0, 8, 11):
        assert lib.mgwfbp_plan_set_option(h, mg.OPT_UPDATE_WGS_PER_CU, good) == mg.OK
    assert lib.mgwfbp_plan_info(None, None, None, None, None, None, None) == mg.EINVAL
    merged = (C.c_uint8 * 3)(1, 0, 0)
    h2 = C.c_void_p()
    assert lib.mgwfbp_plan_explicit(3, p, tb, 0.0, 0.5, 1e-6, 4, merged, C.byref(h2)) == mg.EINVAL
    lib.mgwfbp_plan_destroy(h)
    lib.mgwfbp_plan_destroy(None)


def test_fit_cost_and_table2_match_oracle(golden):
    ex = golden["allreduce_example"]
    a, b = mg.mgwfbp_fit_cost(ex["bytes"], ex["ms"])
    assert a == pytest.approx(1.2, rel=1e-9) and b == pytest.approx(1.5e-6, rel=1e-9)
    rng = np.random.default_rng(31)
    for _ in range(20):
        n = int(rng.integers(2, 40))
        x = rng.uniform(1e2, 1e9, size=n)
        y = rng.uniform(0, 2) + rng.uniform(1e-9, 1e-5) * x + rng.normal(0, 0.02, size=n)
        a_o, b_o = op.fit_cost(x.tolist(), y.tolist())
        a_l, b_l = mg.mgwfbp_fit_cost(x, y)
        assert a_l == pytest.approx(a_o, rel=1e-7, abs=1e-9) and b_l == pytest.approx(b_o, rel=1e-7)
    with pytest.raises(mg.MgwfbpError):
        mg.mgwfbp_fit_cost([5.0, 5.0], [1.0, 2.0])
    for name in mg.TABLE2:
        for n in (2, 4, 8, 64):
            a_l, b_l = mg.mgwfbp_table2_cost(name, n, 0.04526, 8e-7, 1e-8)
            a_o, b_o = op.table2_cost(name, n, 0.04526, 8e-7, 1e-8)
            assert a_l == pytest.approx(a_o, rel=1e-12) and b_l == pytest.approx(b_o, rel=1e-12)
    rs = golden["ring_startup"]
    for n, us in zip(rs["nodes"], rs["startup_us"]):
        assert mg.mgwfbp_table2_cost("ring", n, rs["alpha_us"], 0.0, 0.0)[0] == pytest.approx(us, abs=5e-3)


def test_scaling_curve_matches_oracle():
    """Section V-C style simulation on the ResNet-50 / GoogLeNet shaped traces, 10GbE constants of
    Section V-A (alpha = 45.26 us, 10 Gb/s): the library's curve equals the oracle's plan-by-plan
    evaluation, merging never loses to either baseline, and no latency and infinite bandwidth
    give linear speedup."""
    alpha, beta, gamma = 0.04526, 8e-7, 0.0
    nodes = [1, 2, 4, 8, 16, 32, 64]
    for name in ("resnet50", "googlenet"):
        w = wl.cnn_workload(name)
        p, tb = w.p.tolist(), w.tb_ms.tolist()
        tf = 0.5 * sum(tb)
        curves = {}
        for label, mode in (("wfbp", mg.MODE_WFBP), ("single", mg.MODE_SINGLE),
                            ("theorem1", mg.MODE_PAPER_GREEDY), ("optimal", mg.MODE_OPTIMAL)):
            t, s = mg.mgwfbp_scaling_curve(w.p, w.tb_ms, tf, "ring", alpha, beta, gamma, nodes, mode)
            curves[label] = (t, s)
            for i, n in enumerate(nodes):
                a, b = op.table2_cost("ring", n, alpha, beta, gamma)
                if label == "wfbp":
                    m = []
                elif label == "single":
                    m = range(2, w.L + 1)
                elif label == "theorem1":
                    m = op.algorithm1(p, tb, tf, a, b)
                else:
                    m = mg.mgwfbp_plan(w.p, w.tb_ms, tf, a, b, n, mg.MODE_OPTIMAL).merged_layers()
                t_o = op.simulate(p, tb, tf, a, b, m)
                assert t[i] == pytest.approx(t_o, rel=1e-12)
                assert s[i] == pytest.approx(op.speedup(n, tf, sum(tb), t_o), rel=1e-12)
        for i in range(len(nodes)):
            assert curves["optimal"][1][i] >= curves["wfbp"][1][i] * (1 - 1e-12)
            assert curves["optimal"][1][i] >= curves["single"][1][i] * (1 - 1e-12)
            assert curves["optimal"][1][i] >= curves["theorem1"][1][i] * (1 - 1e-12)
        assert curves["optimal"][1][0] == pytest.approx(1.0, rel=1e-12)      # one worker: a = b = 0
        _, s_free = mg.mgwfbp_scaling_curve(w.p, w.tb_ms, tf, "ring", 0.0, 0.0, 0.0, nodes, mg.MODE_OPTIMAL)
        assert np.allclose(s_free, nodes, rtol=1e-12)


def test_experiments_scaling_table_is_host_only_and_consistent():
    """The scaling table of the experiments module: same numbers as the oracle's Table II costs,
    planning and Eq. 4, and the communication left outside the computation is t_iter - (t_f + t_b)."""
    from paper_1811_11141_amd import experiments as ex

    tab = ex.scaling("googlenet", workers=(4, 16, 64))
    w = wl.cnn_workload("googlenet")
    tf, tb_total = tab["t_f_ms"], float(w.tb_ms.sum())
    for i, n in enumerate(tab["workers"]):
        a, b = op.table2_cost("ring", n, tab["alpha_ms"], tab["beta_ms_per_byte"], 0.0)
        args = (w.p.tolist(), w.tb_ms.tolist(), tf, a, b)
        t_wfbp = op.wfbp_timeline(*args)[1]
        assert tab["modes"]["wfbp"]["t_iter_ms"][i] == pytest.approx(t_wfbp, rel=1e-12)
        assert tab["modes"]["wfbp"]["speedup"][i] == pytest.approx(op.speedup(n, tf, tb_total, t_wfbp), rel=1e-12)
        t_rule = op.simulate(*args, op.algorithm1(*args))
        assert tab["modes"]["theorem1"]["t_iter_ms"][i] == pytest.approx(t_rule, rel=1e-12)
        for m in tab["modes"].values():
            assert m["not_overlapped_ms"][i] == pytest.approx(m["t_iter_ms"][i] - tf - tb_total, abs=1e-9)
            assert m["not_overlapped_ms"][i] >= -1e-9
        assert tab["modes"]["optimal"]["t_iter_ms"][i] <= min(t_wfbp, t_rule) * (1 + 1e-12)


def test_tie_between_equal_plans_keeps_the_smaller_groups(golden):
    """include/mgwfbp.h documents the tie rule of the optimal mode: among plans of equal t_iter
    the one with smaller groups.  The hand-worked tie case (merging layer 2 into 1 or not both
    give 5.0 ms) must therefore come back unmerged, like Theorem 1's strict inequality."""
    c = [x for x in golden["hand_worked_traces"]["cases"] if x["note"].startswith("exact tie")][0]
    args = (c["p"], c["tb_ms"], 0.0, c["a_ms"], c["b_ms_per_byte"])
    assert op.simulate(*args, [2]) == op.simulate(*args, []) == c["t_iter"]
    for mode in (mg.MODE_OPTIMAL, mg.MODE_PAPER_GREEDY):
        pl = mg.mgwfbp_plan(np.array(c["p"], dtype=np.uint64), np.array(c["tb_ms"]), 0.0, c["a_ms"],
                            c["b_ms_per_byte"], 4, mode)
        assert pl.merged_layers() == [] and pl.info()["n_groups"] == 2
        assert pl.info()["t_iter_ms"] == c["t_iter"]


def _exhaustive_recurrence(p, tb, tf, a, b):
    """Eq. 19-23 as a recurrence over 'the lowest layer of a message', every candidate message
    tried (no early exit), ties to the shorter message.  Returns (t_iter, merged layers)."""
    L = len(p)
    mu_b = op.backward_finish(tb, tf)
    best = [0.0] * (L + 1)
    top = [0] * L
    for k in range(L - 1, -1, -1):
        best_t, best_j, n_bytes = float("inf"), k, 0
        for j in range(k, L):
            n_bytes += op.BYTES_PER_PARAM * p[j]
            t = max(best[j + 1], mu_b[k]) + op.t_ar(a, b, n_bytes)
            if t < best_t:
                best_t, best_j = t, j
        best[k], top[k] = best_t, best_j
    merged, k = [], 0
    while k < L:
        merged += list(range(k + 2, top[k] + 2))      # paper numbering: layers k+2 .. top+1 ride down
        k = top[k] + 1
    return best[0], sorted(merged)


def test_early_exit_of_the_exact_planner_changes_nothing():
    """The library stops growing a message once no longer one can be strictly better.  The same
    recurrence without any early exit (checked here against brute force first) must give the same
    merged set, also where many plans tie exactly (small-integer times) and on nets far beyond
    brute force in the compute-bound, mixed and communication-bound regimes."""
    rng = np.random.default_rng(77)
    for _ in range(60):                                   # the exhaustive recurrence is itself exact
        L = int(rng.integers(1, 11))
        p = [int(x) for x in rng.integers(1, 6, L)]
        tb = [float(x) for x in rng.integers(0, 4, L)]
        a, b = float(rng.integers(0, 4)), float(rng.choice([0.0, 0.25, 0.5]))
        t, merged = _exhaustive_recurrence(p, tb, 0.0, a, b)
        assert t == op.brute_force(p, tb, 0.0, a, b)[0] == op.simulate(p, tb, 0.0, a, b, merged)
        pl = mg.mgwfbp_plan(np.array(p, dtype=np.uint64), np.array(tb), 0.0, a, b, 4, mg.MODE_OPTIMAL)
        assert sorted(pl.merged_layers()) == merged and pl.info()["t_iter_ms"] == t
    for L, a, b in ((300, 0.5, 1e-6), (300, 0.5, 1e-4), (300, 5.0, 1e-3), (257, 0.0, 1e-5), (400, 30.0, 0.0)):
        for _ in range(3):
            p = [int(x) for x in np.round(2 ** rng.uniform(6, 16, L))]
            tb = [float(x) for x in rng.uniform(0.1, 2, L)]
            tf = float(rng.uniform(0, 3))
            t, merged = _exhaustive_recurrence(p, tb, tf, a, b)
            pl = mg.mgwfbp_plan(np.array(p, dtype=np.uint64), np.array(tb), tf, a, b, 8, mg.MODE_OPTIMAL)
            assert sorted(pl.merged_layers()) == merged and pl.info()["t_iter_ms"] == t
