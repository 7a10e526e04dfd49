"""Speed and ranking claims, kept apart from the parity tests.

Everything here asserts how FAST something runs on the box, with a margin; none of it decides
whether a result is right.  The file name sorts after every parity test, so that under
`pytest -x` a noisy box can fail only these.  What each margin bounds, what a quiet MI355X machine
showed for it (18 iterations over three tiny nets, 6 graph captures, 3 calibrations), and why the
margin is larger: the GPU machines are shared hosts, and one host stall of ~0.1 ms between two
enqueued operations is enough to move any of these by that much.

  * a stand-in of the backward pass ends at most 0.2 ms after its deadline (measured 0-6 us;
    the stand-ins wait for absolute deadlines, so lateness does not add up over the layers);
  * t_iter is at most 0.02 ms after the last group's end event (measured 5-8 us: one more small
    kernel and the event record);
  * an iteration without per-group timestamps takes at most 0.2 ms longer than one with them
    (measured 2-11 us shorter);
  * a replayed iteration graph ends at most 0.2 ms after its backward pass and within 0.2 ms of
    the eager schedule (measured 8-11 us and 4-8 us);
  * the iteration with the communication side as one gated launch ends at most 0.2 ms after its
    backward pass (measured 5.7 us on the ResNet-50 and GoogLeNet sets; 15.5 us with a launch per
    group);
  * a single small message is done sooner after its arrival in the gated launch than with a launch
    of its own (4-5 us against 14-15 us), and the unmerged plan runs faster as one gated launch than
    as a launch per group (GoogLeNet sizes, 0.3 ms backward pass);
  * tuning may not make the pass more than 10 % slower (repeated timings of one launch shape
    scatter by 2-4 % between runs, the candidates differ from each other by 1-5 %);
  * ranking of the four plans under a 0.3 ms backward pass: no merging at least 2x the optimal
    plan (measured 6.9x), optimal within 1.25x of the better of single-group and Theorem 1's
    rule (measured 1.00x on GoogLeNet's sizes, where all three coincide; the margin allows for
    the 2-9 % by which the model misses communication-bound schedules), model within 30 % of
    the measurement for the no-merging plan (measured 1.7-2.3 %).
"""
import numpy as np
import pytest
import torch

from oracle import planner as op
from paper_1811_11141_amd import workloads as wl

pytestmark = [pytest.mark.gpu, pytest.mark.gpu_timing]


@pytest.fixture(scope="module")
def mg():
    assert torch.cuda.is_available()
    from paper_1811_11141_amd import binding
    return binding


@pytest.mark.parametrize("seed", [0, 1])
def test_iteration_timeline_is_tight(mg, seed):
    w = wl.tiny_workload(seed)
    tb = w.tb_ms * 0.5
    pl = mg.mgwfbp_plan(w.p, tb, 0.0, 0.2, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    grads = wl.make_gradients(w, seed, "cuda")
    pl.bind(grads, [torch.zeros_like(t) for t in grads[0]])
    s_comp, s_comm = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    tl = pl.run_iteration(s_comp, s_comm)
    groups = pl.groups()
    ready, gf = tl["group_ready_ms"], tl["group_finish_ms"]
    mu_b = np.array(op.backward_finish(tb.tolist(), 0.0))
    mu_low = np.array([mu_b[grp[-1]] for grp in groups])
    assert np.all(ready <= mu_low + 0.2)                      # absolute deadlines: gaps do not add up
    assert tl["t_iter_ms"] <= gf.max() + 0.02                 # one more event after the last group
    light = pl.run_iteration(s_comp, s_comm, timeline=False)
    assert light["t_iter_ms"] <= tl["t_iter_ms"] + 0.2
    # the reductions overlap the backward pass: every group but the last ends before it does
    assert np.all(gf[:-1] <= ready[-1] + 0.02) or len(groups) == 1


def test_iteration_graph_is_as_fast_as_the_eager_schedule(mg):
    seed = 5
    w = wl.tiny_workload(seed, L=10)
    tb = w.tb_ms * 0.3
    pl = mg.mgwfbp_plan(w.p, tb, 0.0, 0.1, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    grads = wl.make_gradients(w, seed, "cuda")
    pl.bind(grads, [torch.zeros_like(t) for t in grads[0]])
    s_comp, s_comm, s_run = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    it = pl.capture_iteration(s_comp, s_comm)
    torch.cuda.synchronize()
    times = [it.replay(s_run) for _ in range(4)]
    eager = pl.run_iteration(s_comp, s_comm, timeline=False)["t_iter_ms"]
    backward = float(tb.sum())
    for t in times:
        assert t <= backward + 0.2, (t, backward)
        assert abs(t - eager) < 0.2, (t, eager)
    it.destroy()


def test_gated_iteration_ends_right_after_its_backward_pass(mg):
    w = wl.cnn_workload("googlenet")
    tb = w.tb_ms * (1.0 / w.tb_ms.sum())                      # a 1 ms backward pass
    pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    grads = wl.make_gradients(w, 4, "cuda")
    pl.bind(grads, [torch.zeros_like(t) for t in grads[0]])
    for _ in range(8):
        s_comp, s_comm = torch.cuda.Stream(), torch.cuda.Stream()
        if pl.streams_side_by_side(s_comp, s_comm):
            break
    else:
        pytest.fail("no pair of streams ran side by side")
    pl.run_iteration_gated(s_comp, s_comm, tb_ms=tb)          # first use: code load
    t = min(pl.run_iteration_gated(s_comp, s_comm, tb_ms=tb) for _ in range(3))
    assert 1.0 - 0.02 <= t <= 1.0 + 0.2


@pytest.mark.parametrize("name", ["googlenet", "alexnet"])
def test_tune_is_not_slower(mg, name):
    w = wl.cnn_workload(name)
    pl = mg.mgwfbp_plan(w.p, w.tb_ms, 0.0, w.a_ms, w.b_ms_per_byte, w.n_workers, mg.MODE_OPTIMAL)
    grads = wl.make_gradients(w, wl.BASE_SEED + 3, "cuda")
    pl.bind(grads, [torch.empty_like(t) for t in grads[0]])
    stream = torch.cuda.Stream()

    def per_launch_us():
        best = 1e9
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for _ in range(10):
                pl.pack_reduce_unpack(stream=stream)
            e1.record(stream)
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 100.0)
        return best

    pl.pack_reduce_unpack(stream=stream)
    before = per_launch_us()
    res = pl.tune(stream)
    after = per_launch_us()
    assert after <= before * 1.10, (before, after, res)


def test_calibrated_schedule_ranks_plans_like_the_model(mg):
    """Fit (a, b) on this machine from the schedule itself, then run the four plans with a short
    backward pass: no merging must be the slowest by far, and the model must rank the optimal
    plan first, as measured."""
    from paper_1811_11141_amd import experiments as ex

    cal = ex.calibrate_in_schedule("googlenet", reps=3)
    assert 1e-3 < cal["a_ms"] < 0.2 and 0 < cal["b_ms_per_byte"] < 1e-7
    res = ex.schedule("googlenet", cal["a_ms"], cal["b_ms_per_byte"], backward_ms=0.3, reps=3)["plans"]
    assert res["optimal"]["predicted_t_iter_ms"] <= res["theorem1"]["predicted_t_iter_ms"] + 1e-12
    assert res["optimal"]["predicted_t_iter_ms"] <= res["wfbp"]["predicted_t_iter_ms"] + 1e-12
    assert res["wfbp"]["measured_t_iter_ms"] > 2.0 * res["optimal"]["measured_t_iter_ms"]
    assert res["optimal"]["measured_t_iter_ms"] <= 1.25 * min(res["single"]["measured_t_iter_ms"],
                                                              res["theorem1"]["measured_t_iter_ms"])
    # the model tracks the measurement for the communication-bound plan
    assert res["wfbp"]["measured_t_iter_ms"] == pytest.approx(res["wfbp"]["predicted_t_iter_ms"], rel=0.3)
    # as one gated launch the 59 unmerged groups cost no start-up each: faster than a launch per group
    assert res["wfbp"]["measured_t_iter_gated_launch_ms"] < res["wfbp"]["measured_t_iter_ms"]


def test_a_message_that_arrives_alone_is_done_sooner_in_the_gated_launch(mg):
    """Eq. 9 fitted to single messages after their arrival: the start-up term of the gated launch is
    below that of a launch per group (measured 4.6-7.5 us against 15-16.5 us for messages up to 2 MB)."""
    from paper_1811_11141_amd import experiments as ex

    c = ex.calibrate_arrival(reps=5, sizes=(1 << 10, 1 << 13, 1 << 16))
    small_launch = np.array(c["launch_per_group"]["after_arrival_ms"])
    small_gated = np.array(c["gated_launch"]["after_arrival_ms"])
    assert np.all(small_gated > 0) and np.all(small_launch > 0)
    assert np.median(small_gated) < np.median(small_launch)
