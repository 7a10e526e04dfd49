"""Event-driven iteration (Algorithm 2 on two HIP streams): results equal the oracle's, and the
measured timeline obeys the start rule of Eq. 7 / Condition 2 (ordering and causality only: how
fast the schedule runs is checked in test_zy_gpu_timing.py, after every parity test)."""
import numpy as np
import pytest
import torch

from oracle import datapath as od
from oracle import planner as op
from paper_1811_11141_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mg():
    assert torch.cuda.is_available()
    from paper_1811_11141_amd import binding
    return binding


def to_np(ts):
    return [t.detach().cpu().numpy().copy() for t in ts]


@pytest.mark.parametrize("seed,update", [(0, False), (1, True), (2, True)])
def test_iteration_results_and_timeline(mg, seed, update):
    w = wl.tiny_workload(seed)
    tb = w.tb_ms * 0.5                      # 0.05 .. 1 ms per layer keeps the test short
    pl = mg.mgwfbp_plan(w.p, tb, 0.0, 0.2, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    grads = wl.make_gradients(w, seed, "cuda")
    out = [torch.zeros_like(t) for t in grads[0]]
    wt, vt = wl.make_weights(w, seed, "cuda")
    g_np, w_np, v_np = [to_np(r) for r in grads], to_np(wt), to_np(vt)
    pl.bind(grads, out, wt, vt)
    s_comp, s_comm = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    tl = pl.run_iteration(s_comp, s_comm, update=update, lr=0.1, momentum=0.9)
    groups = pl.groups()
    # results
    if update:
        od.merged_gradient_path(g_np, groups, w_np, v_np, lr=0.1, mu=0.9)
        for l in range(w.L):
            assert np.array_equal(wt[l].cpu().numpy().view(np.uint32), w_np[l].view(np.uint32))
            assert np.array_equal(vt[l].cpu().numpy().view(np.uint32), v_np[l].view(np.uint32))
    exp = od.merged_gradient_path(g_np, groups)
    for l in range(w.L):
        assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32))
    # timeline: each stand-in ends at its layer's mu_b after time zero (Eq. 6).  Time zero is
    # the device clock read by the gate kernel just before it ends; the reported times count
    # from an event recorded after that kernel (a few microseconds later, box dependent) and are
    # taken with another clock (rates agree to a few parts in 10^4), so "never early" is checked
    # up to 20 us plus 0.1 % -- small against the 50 us .. 1 ms a stand-in lasts.
    def early(t):
        return 0.02 + 1e-3 * t
    ready, gs, gf = tl["group_ready_ms"], tl["group_start_ms"], tl["group_finish_ms"]
    mu_b = np.array(op.backward_finish(tb.tolist(), 0.0))
    mu_low = np.array([mu_b[grp[-1]] for grp in groups])      # mu_b of each group's lowest layer
    assert np.all(ready >= mu_low - early(mu_low))            # never early
    eps = 0.02
    for k, grp in enumerate(groups):
        assert gs[k] >= ready[k] - eps                        # gradients exist (Condition 2)
        if k:
            assert gs[k] >= gf[k - 1] - eps                   # channel free (Eq. 7)
        assert gf[k] >= gs[k]
    assert tl["t_iter_ms"] >= gf.max() - 1e-6                 # the iteration ends with its last group (Eq. 8)
    # the same iteration without per-group timestamps: same results, only t_iter comes back
    if not update:
        for t in out:
            t.zero_()
        light = pl.run_iteration(s_comp, s_comm, timeline=False)
        assert set(light) == {"t_iter_ms"}
        assert light["t_iter_ms"] >= mu_b.max() - early(mu_b.max())
        for l in range(w.L):
            assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32))


@pytest.mark.parametrize("n_streams,update", [(2, False), (3, True), (8, False)])
def test_iteration_over_several_communication_streams(mg, n_streams, update):
    """Groups enqueued round-robin over several communication streams: the values are the
    oracle's whatever the number of streams, every group still waits for its own gradients
    (Condition 2), and the iteration ends when the last group has (Eq. 8).  The serial channel of
    Eq. 7 is what this mode gives up, so group k is not required to wait for group k-1."""
    seed = 3
    w = wl.tiny_workload(seed, L=12)
    tb = w.tb_ms * 0.2
    pl = mg.mgwfbp_plan(w.p, tb, 0.0, 0.05, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    groups = pl.groups()
    assert len(groups) >= 3
    grads = wl.make_gradients(w, seed, "cuda")
    out = [torch.full_like(t, float("nan")) for t in grads[0]]
    wt, vt = wl.make_weights(w, seed, "cuda")
    g_np, w_np, v_np = [to_np(r) for r in grads], to_np(wt), to_np(vt)
    pl.bind(grads, out, wt, vt)
    s_comp = torch.cuda.Stream()
    comm = [torch.cuda.Stream() for _ in range(n_streams)]
    torch.cuda.synchronize()
    tl = pl.run_iteration(s_comp, comm, update=update, lr=0.1, momentum=0.9)
    exp = od.merged_gradient_path(g_np, groups, w_np if update else None, v_np if update else None, lr=0.1, mu=0.9)
    for l in range(w.L):
        assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32)), l
        if update:
            assert np.array_equal(wt[l].cpu().numpy().view(np.uint32), w_np[l].view(np.uint32))
            assert np.array_equal(vt[l].cpu().numpy().view(np.uint32), v_np[l].view(np.uint32))
    ready, gs, gf = tl["group_ready_ms"], tl["group_start_ms"], tl["group_finish_ms"]
    for k in range(len(groups)):
        assert gs[k] >= ready[k] - 0.02 and gf[k] >= gs[k]
        if k >= n_streams:                                    # same stream: still in order
            assert gs[k] >= gf[k - n_streams] - 0.02
    assert tl["t_iter_ms"] >= gf.max() - 1e-6
    # argument errors: no stream, the same stream twice, too many
    with pytest.raises(mg.MgwfbpError) as ei:
        pl.run_iteration(s_comp, [])
    assert ei.value.code == mg.EINVAL
    with pytest.raises(mg.MgwfbpError):
        pl.run_iteration(s_comp, [comm[0], comm[0]])
    with pytest.raises(mg.MgwfbpError):
        pl.run_iteration(s_comp, [torch.cuda.Stream() for _ in range(9)])


def test_iteration_needs_binding(mg):
    w = wl.custom_workload([100, 200], 2)
    pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, 0.5, 1e-6, 2, mg.MODE_WFBP)
    with pytest.raises(mg.MgwfbpError) as ei:
        pl.run_iteration(torch.cuda.Stream(), torch.cuda.Stream())
    assert ei.value.code == mg.ESTATE
    grads = wl.make_gradients(w, 1, "cuda")
    pl.bind(grads, [torch.empty_like(t) for t in grads[0]])
    with pytest.raises(mg.MgwfbpError):
        pl.run_iteration(torch.cuda.Stream(), torch.cuda.Stream(), update=True)     # no w, v
    with pytest.raises(mg.MgwfbpError):
        pl.run_iteration(torch.cuda.Stream(), torch.cuda.Stream(), tb_ms=[-1.0, 1.0])
    tl = pl.run_iteration(torch.cuda.Stream(), torch.cuda.Stream(), tb_ms=[0.05, 0.05])
    assert tl["t_iter_ms"] > 0.09


@pytest.mark.parametrize("update", [False, True])
def test_iteration_graph_replays(mg, update):
    """The iteration captured into a HIP graph: every replay, with fresh gradients copied in
    eagerly between replays, gives the oracle's values, and its device-clock t_iter respects
    Eq. 8's lower bound (the backward pass itself)."""
    seed = 5
    w = wl.tiny_workload(seed, L=10)
    tb = w.tb_ms * 0.3
    pl = mg.mgwfbp_plan(w.p, tb, 0.0, 0.1, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    groups = pl.groups()
    grads = wl.make_gradients(w, seed, "cuda")
    out = [torch.zeros_like(t) for t in grads[0]]
    wt, vt = wl.make_weights(w, seed, "cuda")
    w_np, v_np = to_np(wt), to_np(vt)
    pl.bind(grads, out, wt, vt)
    s_comp, s_comm, s_run = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    it = pl.capture_iteration(s_comp, s_comm, update=update, lr=0.1, momentum=0.9)
    torch.cuda.synchronize()
    # nothing ran during capture
    assert all(float(t.abs().sum()) == 0.0 for t in out)
    times = []
    for rep in range(4):
        fresh = wl.make_gradients(w, 700 + rep, "cuda")
        for g in range(w.n_workers):
            for l in range(w.L):
                grads[g][l].copy_(fresh[g][l])
        for t in out:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        times.append(it.replay(s_run))
        g_np = [to_np(r) for r in grads]
        if update:
            exp = od.merged_gradient_path(g_np, groups, w_np, v_np, lr=0.1, mu=0.9)
        else:
            exp = od.merged_gradient_path(g_np, groups)
        for l in range(w.L):
            assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32)), (rep, l)
            if update:
                assert np.array_equal(wt[l].cpu().numpy().view(np.uint32), w_np[l].view(np.uint32))
                assert np.array_equal(vt[l].cpu().numpy().view(np.uint32), v_np[l].view(np.uint32))
    # asynchronous replay
    assert it.replay(s_run, measure=False) is None
    torch.cuda.synchronize()
    if update:
        od.merged_gradient_path([to_np(r) for r in grads], groups, w_np, v_np, lr=0.1, mu=0.9)
        assert np.array_equal(wt[0].cpu().numpy().view(np.uint32), w_np[0].view(np.uint32))
    backward = float(tb.sum())
    for t in times:                         # Eq. 8: no iteration is shorter than its backward pass
        assert t >= backward - (0.02 + 1e-3 * backward), (t, backward)
    it.destroy()
    # streams used for the capture are ordinary streams again
    pl.pack_reduce_unpack(stream=s_comp)
    torch.cuda.synchronize()


def test_iteration_graph_argument_errors(mg):
    w = wl.custom_workload([100, 200], 2)
    pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, 0.5, 1e-6, 2, mg.MODE_WFBP)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    with pytest.raises(mg.MgwfbpError) as ei:
        pl.capture_iteration(s1, s2)
    assert ei.value.code == mg.ESTATE                      # not bound
    grads = wl.make_gradients(w, 1, "cuda")
    pl.bind(grads, [torch.empty_like(t) for t in grads[0]])
    with pytest.raises(mg.MgwfbpError) as ei:
        pl.capture_iteration(s1, s1)                       # fork and join need two streams
    assert ei.value.code == mg.EINVAL
    with pytest.raises(mg.MgwfbpError):
        pl.capture_iteration(s1, s2, update=True)          # no w, v
    it = pl.capture_iteration(s1, s2, tb_ms=[0.05, 0.05])
    assert it.replay(s1) >= 0.095
    # a new binding replaces the device tables the graph points into: the graph is stale
    pl.bind(grads, [torch.empty_like(t) for t in grads[0]])
    with pytest.raises(mg.MgwfbpError) as ei:
        it.replay(s1)
    assert ei.value.code == mg.ESTATE
    it2 = pl.capture_iteration(s1, s2, tb_ms=[0.05, 0.05])
    assert it2.replay(s1) >= 0.095
    pl.destroy()                      # takes its graphs with it
    assert not it2._h
    # through the C ABI alone, destroying the plan first leaves the iteration handle valid but stale
    raw = mg.raw()
    import ctypes as C
    pl2 = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, 0.5, 1e-6, 2, mg.MODE_WFBP)
    pl2.bind(grads, [torch.empty_like(t) for t in grads[0]])
    it3 = pl2.capture_iteration(s1, s2, tb_ms=[0.05, 0.05])
    handle, it3._h = it3._h, C.c_void_p(0)            # take the handle away from the wrapper
    pl2._graphs = []
    pl2.destroy()
    t = C.c_double()
    assert raw.mgwfbp_iteration_replay(handle, C.c_void_p(int(s1.cuda_stream)), C.byref(t)) == mg.ESTATE
    assert "destroyed" in mg.last_error()
    raw.mgwfbp_iteration_destroy(handle)
