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
    # from an event recorded after that kernel and are taken with another clock (rates agree to a
    # few parts in 10^4).  The event is stamped when the command processor gets to it: 2-6 us
    # after the gate's reading on a quiet box, 22 us on a busy one (every group of that run was
    # "early" by the same 22 us), so "never early" is checked up to 0.1 ms plus 0.1 % for the
    # event times -- a stand-in that did not wait would be early by its whole 0.5 .. 4 ms -- and
    # up to 20 us plus 0.1 % where both ends are read from the device clock.
    def early(t, skew=0.02):
        return skew + 1e-3 * t
    ready, gs, gf = tl["group_ready_ms"], tl["group_start_ms"], tl["group_finish_ms"]
    mu_b = np.array(op.backward_finish(tb.tolist(), 0.0))
    mu_low = np.array([mu_b[grp[-1]] for grp in groups])      # mu_b of each group's lowest layer
    assert np.all(ready >= mu_low - early(mu_low, 0.1))       # never early
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


# ---- Algorithm 2's communication side as one gated launch -------------------------------------

def streams_side_by_side(pl, tries=8):
    """(signalling, waiting) streams whose kernels the device runs at the same time.  The runtime
    serves its streams from four hardware queues; a pair that shares one cannot be used."""
    for _ in range(tries):
        a, b = torch.cuda.Stream(), torch.cuda.Stream()
        if pl.streams_side_by_side(a, b):
            return a, b
    pytest.fail(f"no pair of streams ran side by side in {tries} tries")


@pytest.mark.parametrize("name,update", [("tiny", False), ("tiny", True), ("googlenet", False), ("resnet50", True)])
def test_gated_iteration_equals_oracle(mg, name, update):
    """mgwfbp_run_iteration_gated: one launch walks the groups in arrival order and waits on the
    device for each group's arrival counter; values equal the oracle's, the iteration is not
    shorter than its backward pass (Eq. 8), and a second iteration (counters at 2) works too."""
    if name == "tiny":
        w = wl.tiny_workload(9, L=12)
        tb = w.tb_ms * 0.1
        pl = mg.mgwfbp_plan(w.p, tb, 0.0, 0.05, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    else:
        w = wl.cnn_workload(name)
        tb = w.tb_ms * (1.0 / w.tb_ms.sum())                   # a 1 ms backward pass
        pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    groups = pl.groups()
    grads = wl.make_gradients(w, 21, "cuda")
    out = [torch.full_like(t, float("nan")) for t in grads[0]]
    wt, vt = wl.make_weights(w, 21, "cuda")
    for t in vt:
        t.normal_(0, 1e-3)
    w0, v0 = [t.clone() for t in wt], [t.clone() for t in vt]
    pl.bind(grads, out, wt, vt)
    s_comp, s_comm = streams_side_by_side(pl)
    torch.cuda.synchronize()
    t_iter = pl.run_iteration_gated(s_comp, s_comm, tb_ms=tb, update=update, lr=0.1, momentum=0.9)
    backward = float(np.sum(tb))
    assert t_iter >= backward - (0.02 + 1e-3 * backward)
    assert not pl.gated_gave_up()

    def check(w_ref, v_ref):
        for l, n in enumerate(int(x) for x in w.p):
            avg = od.reduce([grads[g][l].cpu().numpy() for g in range(w.n_workers)])
            assert np.array_equal(out[l].cpu().numpy().view(np.uint32), avg.view(np.uint32)), l
            if update:
                ww, vv = w_ref[l].cpu().numpy(), v_ref[l].cpu().numpy()
                od.sgd(ww, vv, avg, 0.1, 0.9)
                assert np.array_equal(wt[l].cpu().numpy().view(np.uint32), ww.view(np.uint32)), l
                assert np.array_equal(vt[l].cpu().numpy().view(np.uint32), vv.view(np.uint32)), l
    check(w0, v0)
    # next iteration: fresh gradients, counters move on to 2
    w1, v1 = [t.clone() for t in wt], [t.clone() for t in vt]
    fresh = wl.make_gradients(w, 22, "cuda")
    for g in range(w.n_workers):
        for l in range(w.L):
            grads[g][l].copy_(fresh[g][l])
    for t in out:
        t.fill_(float("nan"))
    torch.cuda.synchronize()
    pl.run_iteration_gated(s_comp, s_comm, tb_ms=tb, update=update, lr=0.1, momentum=0.9)
    check(w1, v1)
    assert len(groups) >= 1


def test_gated_launch_waits_for_signals_in_any_order_and_gives_up_when_none_comes(mg):
    """The launch and the signals through the C ABI.  Signals come from another stream in reverse
    group order, each behind a short stand-in: every group still runs, after its own signal.  A
    launch whose groups are never signalled ends by itself after give_up_ms (a bounded wait that
    the host forces to fail: every workgroup still exits normally) and says so."""
    w = wl.custom_workload([70001, 5, 4096 * 3, 300, 9000, 64, 12289], 3, sigma=1e-2)
    merged = [7, 5, 4, 2]
    pl = mg.mgwfbp_plan_explicit(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, 3, merged)
    groups = pl.groups()
    grads = wl.make_gradients(w, 5, "cuda")
    out = [torch.full_like(t, float("nan")) for t in grads[0]]
    pl.bind(grads, out)
    s_sig, s_launch = streams_side_by_side(pl)
    torch.cuda.synchronize()
    # 1. never signalled: gives up after 20 ms, nothing is written
    pl.gated_launch(arrival=1, give_up_ms=20.0, stream=s_launch)
    torch.cuda.synchronize()
    assert pl.gated_gave_up()
    assert all(bool(torch.isnan(t).all()) for t in out)
    # 2. signalled in reverse order from another stream
    pl.gated_launch(arrival=1, give_up_ms=5000.0, stream=s_launch)
    with torch.cuda.stream(s_sig):
        for k in reversed(range(len(groups))):
            torch.cuda._sleep(200_000)                        # ~0.1 ms of device time between arrivals
            pl.gated_signal(k, 1, stream=s_sig)
    torch.cuda.synchronize()
    assert not pl.gated_gave_up()
    exp = od.merged_gradient_path([to_np(r) for r in grads], groups)
    for l in range(w.L):
        assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32)), l
    # 3. counters only grow: a launch for arrival 1 again runs at once, one for arrival 2 waits
    for t in out:
        t.fill_(float("nan"))
    pl.gated_launch(arrival=1, give_up_ms=5000.0, stream=s_launch)
    torch.cuda.synchronize()
    assert not pl.gated_gave_up() and all(bool(torch.isfinite(t).all()) for t in out)
    pl.gated_launch(arrival=2, give_up_ms=10.0, stream=s_launch)
    torch.cuda.synchronize()
    assert pl.gated_gave_up()
    with pytest.raises(mg.MgwfbpError):
        pl.gated_signal(len(groups), 1)                       # no such group
    with pytest.raises(mg.MgwfbpError):
        pl.run_iteration_gated(s_launch, s_launch)            # needs two streams


def test_streams_that_share_a_hardware_queue_are_refused(mg):
    """mgwfbp_streams_side_by_side: a stream does not run beside itself; among fresh pairs most run
    side by side; a pair that does not is refused by the gated iteration at once (MGWFBP_ESTATE,
    nothing run) instead of after give_up_ms."""
    import time
    w = wl.tiny_workload(9, L=12)
    pl = mg.mgwfbp_plan(w.p, w.tb_ms * 0.1, 0.0, 0.05, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    grads = wl.make_gradients(w, 3, "cuda")
    out = [torch.full_like(t, float("nan")) for t in grads[0]]
    pl.bind(grads, out)
    s = torch.cuda.Stream()
    assert not pl.streams_side_by_side(s, s)
    good, bad = [], []
    for _ in range(16):                                       # torch hands out 32 pooled streams in turn
        a, b = torch.cuda.Stream(), torch.cuda.Stream()
        (good if pl.streams_side_by_side(a, b) else bad).append((a, b))
    assert len(good) >= 8
    a, b = good[0]
    assert pl.streams_side_by_side(a, b)                      # remembered
    pl.run_iteration_gated(a, b, tb_ms=w.tb_ms * 0.1)
    assert all(bool(torch.isfinite(t).all()) for t in out)
    if bad:
        for t in out:
            t.fill_(float("nan"))
        a, b = bad[0]
        t0 = time.perf_counter()
        with pytest.raises(mg.MgwfbpError) as ei:
            pl.run_iteration_gated(a, b, tb_ms=w.tb_ms * 0.1, give_up_ms=5000.0)
        assert ei.value.code == mg.ESTATE
        assert time.perf_counter() - t0 < 1.0
        torch.cuda.synchronize()
        assert all(bool(torch.isnan(t).all()) for t in out)


@pytest.mark.parametrize("seed", range(16))
def test_gated_launch_random_shapes(mg, seed):
    """Random layer counts, sizes (tiny, around tile boundaries, mid-sized), worker counts, merge
    sets, gather thresholds, padded layouts and misaligned pointers through the gated launch:
    first with the groups signalled in a random order from a second stream, then as an update with
    every group already arrived; out[], w and v against the oracle, bit for bit."""
    rng = np.random.default_rng(7000 + seed)
    L = int(rng.integers(1, 33))
    sizes = []
    for kd in rng.integers(0, 4, size=L):
        if kd == 0:
            sizes.append(int(rng.integers(1, 600)))
        elif kd == 1:
            sizes.append(max(1, int(rng.integers(1, 6)) * int(rng.choice([512, 4096])) + int(rng.integers(-5, 6))))
        elif kd == 2:
            sizes.append(int(rng.integers(1, 40)) * 4)
        else:
            sizes.append(int(rng.integers(10_000, 200_000)))
    N = int(rng.choice([1, 2, 3, 4, 5, 8, 16, 17]))
    w = wl.custom_workload(sizes, N, sigma=1e-2)
    merged = [l for l in range(2, L + 1) if rng.random() < 0.5]
    groups = [[l - 1 for l in g] for g in op.groups_from_merged(L, merged)]
    pl = mg.mgwfbp_plan_explicit(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, N, merged)
    pl.set_option(mg.OPT_SMALL_ELEMS, int(rng.choice([0, 1, 64, 512, 1024])))
    pl.set_option(mg.OPT_PAD_ELEMS, int(rng.choice([0, 0, 4, 32])))
    pl.set_option(mg.OPT_GATED_WGS_PER_CU, int(rng.choice([-1, 1, 3, 15])))
    misalign = bool(rng.integers(0, 2))
    gen = torch.Generator(device="cuda").manual_seed(seed)

    def tensor(n, scale):
        k = int(rng.integers(0, 4)) if misalign else 0
        base = torch.empty(n + 4, dtype=torch.float32, device="cuda").normal_(0, scale, generator=gen)
        return base[k:k + n]

    grads = [[tensor(n, 1e-2) for n in sizes] for _ in range(N)]
    out = [tensor(n, 1.0) for n in sizes]
    wt = [tensor(n, 0.1) for n in sizes]
    vt = [tensor(n, 1e-3) for n in sizes]
    g_np, w_np, v_np = [to_np(r) for r in grads], to_np(wt), to_np(vt)
    for t in out:
        t.fill_(float("nan"))
    without_out = seed % 4 == 3                               # the update alone: out[] not bound
    pl.bind(grads, None if without_out else out, wt, vt)
    exp = od.merged_gradient_path(g_np, groups)
    s_sig, s_launch = streams_side_by_side(pl)
    torch.cuda.synchronize()
    if without_out:
        with pytest.raises(mg.MgwfbpError):
            pl.gated_launch(arrival=1, stream=s_launch)       # the reduction needs somewhere to write
        with torch.cuda.stream(s_sig):
            for k in rng.permutation(len(groups)):
                pl.gated_signal(int(k), 1, stream=s_sig)
    else:
        pl.gated_launch(arrival=1, give_up_ms=5000.0, stream=s_launch)
        with torch.cuda.stream(s_sig):
            for k in rng.permutation(len(groups)):
                pl.gated_signal(int(k), 1, stream=s_sig)
        torch.cuda.synchronize()
        assert not pl.gated_gave_up()
        for l in range(L):
            assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32)), (seed, l)
    pl.gated_launch(arrival=1, update=True, lr=0.3, momentum=0.7, give_up_ms=5000.0, stream=s_launch)
    torch.cuda.synchronize()
    assert not pl.gated_gave_up()
    if without_out:
        assert all(bool(torch.isnan(t).all()) for t in out)
    od.merged_gradient_path(g_np, groups, w_np, v_np, 0.3, 0.7)
    for l in range(L):
        assert np.array_equal(wt[l].cpu().numpy().view(np.uint32), w_np[l].view(np.uint32)), (seed, l)
        assert np.array_equal(vt[l].cpu().numpy().view(np.uint32), v_np[l].view(np.uint32)), (seed, l)


@pytest.mark.parametrize("update", [False, True])
def test_gated_launch_reads_what_the_producer_wrote_while_it_was_waiting(mg, update):
    """The pattern the gated launch exists for: it is already running (and waiting) when the
    gradients of a group are produced on another stream, and it must read those values, not what
    the tensors held when it started.  The tensors hold NaN until, group by group in a random
    order, a copy kernel on the signalling stream fills them and the group is signalled: a tile
    that ran before its signal, or read a line cached from before, would leave NaN behind."""
    rng = np.random.default_rng(99 + int(update))
    sizes = [70001, 5, 4096 * 3, 300, 9000, 64, 12289, 300000, 1024 * 7, 513]
    N = 4
    w = wl.custom_workload(sizes, N, sigma=1e-2)
    merged = [10, 8, 7, 4, 3]
    groups = [[l - 1 for l in g] for g in op.groups_from_merged(w.L, merged)]
    pl = mg.mgwfbp_plan_explicit(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, N, merged)
    fresh = wl.make_gradients(w, 31, "cuda")
    grads = [[torch.full_like(t, float("nan")) for t in rep] for rep in fresh]
    out = [torch.full_like(t, float("nan")) for t in fresh[0]]
    wt, vt = wl.make_weights(w, 31, "cuda")
    for t in vt:
        t.normal_(0, 1e-3)
    w_np, v_np = to_np(wt), to_np(vt)
    pl.bind(grads, out, wt, vt)
    s_sig, s_launch = streams_side_by_side(pl)
    for arrival in (1, 2):                                    # the second pass finds the first one's values in place
        for rep in grads:
            for t in rep:
                t.fill_(float("nan"))
        for t in out:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        pl.gated_launch(arrival=arrival, update=update, lr=0.1, momentum=0.9, give_up_ms=5000.0, stream=s_launch)
        with torch.cuda.stream(s_sig):
            for k in rng.permutation(len(groups)):
                torch.cuda._sleep(100_000)                    # the launch is waiting by now
                for l in groups[int(k)]:
                    for g in range(N):
                        grads[g][l].copy_(fresh[g][l])
                pl.gated_signal(int(k), arrival, stream=s_sig)
        torch.cuda.synchronize()
        assert not pl.gated_gave_up()
        exp = od.merged_gradient_path([to_np(r) for r in fresh], groups)
        for l in range(w.L):
            assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32)), (arrival, l)
        if update:
            od.merged_gradient_path([to_np(r) for r in fresh], groups, w_np, v_np, 0.1, 0.9)
            for l in range(w.L):
                assert np.array_equal(wt[l].cpu().numpy().view(np.uint32), w_np[l].view(np.uint32)), (arrival, l)
                assert np.array_equal(vt[l].cpu().numpy().view(np.uint32), v_np[l].view(np.uint32)), (arrival, l)
        fresh = wl.make_gradients(w, 32 + arrival, "cuda")     # other values for the next pass


@pytest.mark.parametrize("update", [False, True])
def test_gated_launch_leaves_room_for_producers_with_full_size_workgroups(mg, update):
    """The default grid of the gated launch leaves four workgroup slots per compute unit free: a
    producer whose workgroups have 256 lanes (an elementwise torch kernel per group, on the
    signalling stream) is placed and runs while the ResNet-50-sized launch waits, for the reduction
    and for the update form (with two slots free the update form starved it and gave up)."""
    w = wl.cnn_workload("resnet50")
    pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    grads = wl.make_gradients(w, 8, "cuda")
    out = [torch.empty_like(t) for t in grads[0]]
    wt, vt = wl.make_weights(w, 8, "cuda")
    pl.bind(grads, out, wt, vt)
    total, per_cu = pl.gated_workgroups(update)
    holds = 14 if update else 16
    assert 0 < per_cu <= holds - 4 and total <= per_cu * 256
    greedy = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    greedy.set_option(mg.OPT_GATED_WGS_PER_CU, 15)
    greedy.bind(grads, out, wt, vt)
    assert per_cu <= greedy.gated_workgroups(update)[1] <= holds - 2      # never fewer than two free
    greedy.destroy()
    s_sig, s_launch = streams_side_by_side(pl)
    scratch = torch.zeros(4096, 4096, device="cuda")
    with torch.cuda.stream(s_sig):
        scratch.add_(1.0)                                     # first use on this stream, before any waiting
    torch.cuda.synchronize()
    pl.gated_launch(arrival=1, update=update, lr=0.1, momentum=0.9, give_up_ms=2000.0, stream=s_launch)
    with torch.cuda.stream(s_sig):
        for k in range(pl.info()["n_groups"]):
            scratch.add_(1.0)
            pl.gated_signal(k, 1, stream=s_sig)
    torch.cuda.synchronize()
    assert not pl.gated_gave_up()
    assert float(scratch[0, 0]) == pl.info()["n_groups"] + 1


def test_gated_launch_confined_to_half_the_chip_lets_matrix_core_producers_run(mg):
    """mgwfbp_confined_stream_create + MGWFBP_OPT_GATED_CUS: the gated launch (update form) sits on
    the first 128 compute units only, so producers that need whole SIMDs -- an fp16 matrix-core
    GEMM per group on the signalling stream -- run on the rest of the chip while it waits (on the
    whole chip they are never placed and the launch gives up).  Results against the oracle; the
    fused pass on the confined stream, too."""
    w = wl.cnn_workload("googlenet")
    pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    pl.set_option(mg.OPT_GATED_CUS, 128)
    grads = wl.make_gradients(w, 12, "cuda")
    out = [torch.full_like(t, float("nan")) for t in grads[0]]
    wt, vt = wl.make_weights(w, 12, "cuda")
    for t in vt:
        t.normal_(0, 1e-3)
    w_np, v_np = to_np(wt), to_np(vt)
    pl.bind(grads, out, wt, vt)
    with pytest.raises(mg.MgwfbpError):
        mg.ConfinedStream(100)                                # whole 32-unit words only
    with pytest.raises(mg.MgwfbpError):
        mg.ConfinedStream(4096)                               # more than the device has
    cs = mg.ConfinedStream(128)
    try:
        total, per_cu = pl.gated_workgroups(True)
        assert 0 < total <= per_cu * 128
        for _ in range(8):
            s_sig = torch.cuda.Stream()
            if pl.streams_side_by_side(s_sig, cs.stream):
                break
        else:
            pytest.fail("no stream ran beside the confined one")
        a = torch.randn(2048, 2048, device="cuda").half()
        b = torch.randn(2048, 2048, device="cuda").half()
        with torch.cuda.stream(s_sig):
            ref = torch.mm(a, b)                              # first call on this stream, before any waiting
        torch.cuda.synchronize()
        groups = pl.groups()
        pl.gated_launch(arrival=1, update=True, lr=0.1, momentum=0.9, give_up_ms=2000.0, stream=cs.stream)
        with torch.cuda.stream(s_sig):
            for k in range(len(groups)):
                c = torch.mm(a, b)
                pl.gated_signal(k, 1, stream=s_sig)
        torch.cuda.synchronize()
        assert not pl.gated_gave_up()
        assert torch.equal(c, ref)
        g_np = [to_np(r) for r in grads]
        exp = od.merged_gradient_path(g_np, groups)
        od.merged_gradient_path(g_np, groups, w_np, v_np, 0.1, 0.9)
        for l in range(w.L):
            assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32)), l
            assert np.array_equal(wt[l].cpu().numpy().view(np.uint32), w_np[l].view(np.uint32)), l
            assert np.array_equal(vt[l].cpu().numpy().view(np.uint32), v_np[l].view(np.uint32)), l
        for t in out:
            t.fill_(float("nan"))
        pl.pack_reduce_unpack(stream=cs.stream)               # any launch may go to the confined stream
        torch.cuda.synchronize()
        for l in range(w.L):
            assert np.array_equal(out[l].cpu().numpy().view(np.uint32), exp[l].view(np.uint32)), l
    finally:
        torch.cuda.synchronize()
        cs.destroy()
