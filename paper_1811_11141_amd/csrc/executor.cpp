// Event-driven MG-WFBP iteration: Algorithm 2's two threads mapped onto two HIP streams.
//
// Algorithm 2 runs a computation thread (backward pass, pushing each finished layer into a
// queue) and a communication thread (popping layers into the layer buffer and all-reducing it
// whenever a layer that is not merged arrives).  On the GPU the queue becomes a HIP event per
// group: the backward stand-in of the group's lowest layer is followed by an event record on
// the compute stream, and the communication stream waits for that event before it runs the
// group's reduction.  The host enqueues everything up front and only waits at the end, so the
// start rule of Eq. 7 (a group starts when the channel is free and its gradients exist) is
// enforced by the hardware queues, not by host threads.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <new>
#include <string>
#include <vector>

#include "../../include/mgwfbp.h"
#include "plan.hpp"

using namespace mgwfbp;

namespace {

struct Events {
    std::vector<hipEvent_t> ev;
    ~Events()
    {
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    }
    int make(hipEvent_t *out, bool timed = true)
    {
        const hipError_t e =
            timed ? hipEventCreate(out) : hipEventCreateWithFlags(out, hipEventDisableTiming);
        if (e != hipSuccess) {
            set_error(std::string("hipEventCreate: ") + hipGetErrorString(e));
            return MGWFBP_EHIP;
        }
        ev.push_back(*out);
        return MGWFBP_OK;
    }
};

int hip_fail(const char *what, hipError_t e)
{
    set_error(std::string(what) + ": " + hipGetErrorString(e));
    return MGWFBP_EHIP;
}

}  // namespace

namespace {

int check_iteration_args(mgwfbp_plan_t *pl, const double *tb, int32_t update)
{
    if (!pl) {
        set_error("plan is NULL");
        return MGWFBP_EINVAL;
    }
    if (!pl->bound) {
        set_error("mgwfbp_bind has not been called");
        return MGWFBP_ESTATE;
    }
    if (update ? !pl->has_wv : !pl->has_out) {
        set_error(update ? "w[] and v[] are not bound" : "out[] is not bound");
        return MGWFBP_ESTATE;
    }
    for (int32_t l = 0; l < pl->L; ++l) {
        if (!(tb[l] >= 0.0) || tb[l] > 1.0e4) {
            set_error("tb_ms[" + std::to_string(l) + "] must be in [0, 10000] ms");
            return MGWFBP_EINVAL;
        }
    }
    return MGWFBP_OK;
}

// Enqueue one iteration: gate (publishes time zero in the plan's clock word 0) on `cs`, then per
// group a backward stand-in on `cs`, an event, and the group's reduction behind that event on
// communication stream k mod n; finally word 1 of the clock gets the device time at which the
// last group ended.  With one communication stream the groups follow each other as on the
// serial channel of Eq. 7; with more, consecutive groups go to different streams and may overlap
// (they touch disjoint tensors), each still waiting for its own gradients (Condition 2).
// g_start / g_finish may be NULL (no per-group timestamps).  `joins` holds one untimed event per
// communication stream beyond the first.
int enqueue_iteration(mgwfbp_plan_t *pl, const double *tb, bool update, float lr, float momentum,
                      hipStream_t cs, const std::vector<hipStream_t> &ms, double gate_ms, hipEvent_t base,
                      const std::vector<hipEvent_t> &g_ready, const std::vector<hipEvent_t> *g_start,
                      const std::vector<hipEvent_t> *g_finish, const std::vector<hipEvent_t> &joins)
{
    int rc;
    if ((rc = launch_spin(gate_ms, cs, pl->d_clock))) return rc;
    // no communication stream may start before the backward pass does
    hipError_t e = hipEventRecord(base, cs);
    if (e != hipSuccess) return hip_fail("hipEventRecord", e);
    for (hipStream_t m : ms)
        if ((e = hipStreamWaitEvent(m, base, 0)) != hipSuccess) return hip_fail("hipStreamWaitEvent", e);

    // Backward pass, highest layer first.  Only the moment a group's lowest layer finishes
    // matters to the communication side, so the layers of a group share one stand-in kernel
    // that ends when the backward pass has reached the end of the group's lowest layer.
    double elapsed_ms = 0.0;
    for (int32_t l = pl->L - 1; l >= 0; --l) {
        elapsed_ms += tb[l];
        if (pl->merged[l]) continue;  // layer l rides with layer l-1: nothing is sent yet
        // layer l is the lowest layer of its group: the group's gradients are complete
        const size_t k = static_cast<size_t>(pl->group_of_layer[l]);
        hipStream_t m = ms[k % ms.size()];
        if ((rc = launch_spin_until(elapsed_ms, pl->d_clock, cs))) return rc;
        if ((e = hipEventRecord(g_ready[k], cs)) != hipSuccess) return hip_fail("hipEventRecord", e);
        if ((e = hipStreamWaitEvent(m, g_ready[k], 0)) != hipSuccess)
            return hip_fail("hipStreamWaitEvent", e);
        if (g_start && (e = hipEventRecord((*g_start)[k], m)) != hipSuccess)
            return hip_fail("hipEventRecord", e);
        if ((rc = run_scope(pl, static_cast<int32_t>(k), update, lr, momentum, nullptr, 0, m))) return rc;
        if (g_finish && (e = hipEventRecord((*g_finish)[k], m)) != hipSuccess)
            return hip_fail("hipEventRecord", e);
    }
    // the first communication stream collects the others: its end is the end of the iteration (Eq. 8)
    for (size_t i = 1; i < ms.size(); ++i) {
        if ((e = hipEventRecord(joins[i - 1], ms[i])) != hipSuccess) return hip_fail("hipEventRecord", e);
        if ((e = hipStreamWaitEvent(ms[0], joins[i - 1], 0)) != hipSuccess) return hip_fail("hipStreamWaitEvent", e);
    }
    return launch_spin(0.0, ms[0], pl->d_clock + 1);
}

// The communication streams of a call: distinct handles, at least one, at most kMaxCommStreams.
constexpr int32_t kMaxCommStreams = 8;
int collect_streams(void *const *comm_streams, int32_t n, std::vector<hipStream_t> &out)
{
    if (!comm_streams || n < 1 || n > kMaxCommStreams) {
        set_error("need 1 to " + std::to_string(kMaxCommStreams) + " communication streams");
        return MGWFBP_EINVAL;
    }
    out.clear();
    for (int32_t i = 0; i < n; ++i) {
        hipStream_t s = static_cast<hipStream_t>(comm_streams[i]);
        for (hipStream_t t : out)
            if (t == s) {
                set_error("the communication streams must be different streams");
                return MGWFBP_EINVAL;
            }
        out.push_back(s);
    }
    return MGWFBP_OK;
}

// (clock word 1 - clock word 0) in milliseconds, after the streams have drained.
int read_t_iter(const mgwfbp_plan_t *pl, double *t_iter_ms)
{
    uint64_t words[2] = {0, 0};
    const hipError_t e = hipMemcpy(words, pl->d_clock, sizeof(words), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail("hipMemcpy of the clock words", e);
    *t_iter_ms = static_cast<double>(words[1] - words[0]) / static_cast<double>(wall_clock_khz());
    return MGWFBP_OK;
}

}  // namespace

namespace {
int run_iteration_impl(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr,
                       float momentum, void *compute_stream, void *const *comm_streams,
                       int32_t n_comm_streams, double *group_ready_ms, double *group_start_ms,
                       double *group_finish_ms, double *t_iter_ms)
{
    const double *tb = tb_ms ? tb_ms : (pl ? pl->tb.data() : nullptr);
    int rc = check_iteration_args(pl, tb, update);
    if (rc) return rc;
    const size_t G = pl->groups.size();
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    std::vector<hipStream_t> ms;
    if ((rc = collect_streams(comm_streams, n_comm_streams, ms))) return rc;

    // Per-group timestamps are taken only when the caller asks for them: a timed event record
    // costs a few microseconds of stream time, which is a large part of a short group's cost.
    const bool time_ready = group_ready_ms != nullptr;
    const bool time_comm = group_start_ms != nullptr || group_finish_ms != nullptr;
    Events pool;
    hipEvent_t base;
    std::vector<hipEvent_t> g_ready(G), g_start(time_comm ? G : 0), g_finish(time_comm ? G : 0);
    std::vector<hipEvent_t> joins(ms.size() - 1);
    rc = pool.make(&base);
    for (size_t k = 0; k < G && !rc; ++k) {
        rc = pool.make(&g_ready[k], time_ready);
        if (!rc && time_comm) rc = pool.make(&g_start[k]);
        if (!rc && time_comm) rc = pool.make(&g_finish[k]);
    }
    for (size_t i = 0; i < joins.size() && !rc; ++i) rc = pool.make(&joins[i], false);
    if (rc) return rc;

    // A zero-length stand-in first: the first launch of a kernel loads its code.  Then a gate:
    // the host needs tens of microseconds per group to enqueue kernels, event records and
    // waits, far more than a short group takes to run, so without a head start the measured
    // timeline would show the host's enqueue rate.  The gate keeps the compute stream busy
    // while everything behind it is being queued; time zero is the end of the gate, where the
    // gate publishes the device clock.  Every stand-in then waits for an absolute deadline
    // (time zero + the backward time accumulated so far), so launch gaps between stand-ins do
    // not stretch the backward pass.
    if ((rc = launch_spin(0.0, cs))) return rc;
    rc = enqueue_iteration(pl, tb, update != 0, lr, momentum, cs, ms, 1.0 + 0.06 * static_cast<double>(G),
                           base, g_ready, time_comm ? &g_start : nullptr, time_comm ? &g_finish : nullptr, joins);
    // whatever was enqueued must drain before the events are destroyed or read
    const hipError_t e1 = hipStreamSynchronize(cs);
    hipError_t e2 = hipSuccess;
    for (hipStream_t m : ms) {
        const hipError_t em = hipStreamSynchronize(m);
        if (e2 == hipSuccess) e2 = em;
    }
    if (rc) return rc;
    if (e1 != hipSuccess) return hip_fail("hipStreamSynchronize(compute)", e1);
    if (e2 != hipSuccess) return hip_fail("hipStreamSynchronize(comm)", e2);

    auto since_base = [&](hipEvent_t ev, double *out) -> int {
        float t = 0.0f;
        const hipError_t er = hipEventElapsedTime(&t, base, ev);
        if (er != hipSuccess) return hip_fail("hipEventElapsedTime", er);
        *out = static_cast<double>(t);
        return MGWFBP_OK;
    };
    for (size_t k = 0; k < G; ++k) {
        double t;
        if (time_ready) {
            if ((rc = since_base(g_ready[k], &t))) return rc;
            group_ready_ms[k] = t;
        }
        if (time_comm) {
            if ((rc = since_base(g_start[k], &t))) return rc;
            if (group_start_ms) group_start_ms[k] = t;
            if ((rc = since_base(g_finish[k], &t))) return rc;
            if (group_finish_ms) group_finish_ms[k] = t;
        }
    }
    if (t_iter_ms) return read_t_iter(pl, t_iter_ms);
    return MGWFBP_OK;
}
}  // namespace

extern "C" int mgwfbp_run_iteration(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr,
                                    float momentum, void *compute_stream, void *comm_stream,
                                    double *group_ready_ms, double *group_start_ms,
                                    double *group_finish_ms, double *t_iter_ms)
{
    return guarded([&]() -> int {
        void *const one[1] = {comm_stream};
        return run_iteration_impl(pl, tb_ms, update, lr, momentum, compute_stream, one, 1,
                                  group_ready_ms, group_start_ms, group_finish_ms, t_iter_ms);
    });
}

extern "C" int mgwfbp_run_iteration_streams(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr,
                                            float momentum, void *compute_stream, void *const *comm_streams,
                                            int32_t n_comm_streams, double *group_ready_ms,
                                            double *group_start_ms, double *group_finish_ms, double *t_iter_ms)
{
    return guarded([&]() -> int {
        return run_iteration_impl(pl, tb_ms, update, lr, momentum, compute_stream, comm_streams, n_comm_streams,
                                  group_ready_ms, group_start_ms, group_finish_ms, t_iter_ms);
    });
}

// ---- the iteration with the communication side as ONE gated launch ------------------------------

namespace {
int run_iteration_gated_impl(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr, float momentum,
                             void *compute_stream, void *comm_stream, double give_up_ms, double *t_iter_ms)
{
    const double *tb = tb_ms ? tb_ms : (pl ? pl->tb.data() : nullptr);
    int rc = check_iteration_args(pl, tb, update);
    if (rc) return rc;
    if (!(give_up_ms > 0.0) || give_up_ms > 6.0e4) {
        set_error("give_up_ms must be in (0, 60000]");
        return MGWFBP_EINVAL;
    }
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    hipStream_t ms = static_cast<hipStream_t>(comm_stream);
    if (cs == ms) {
        // one stream would put the launch that waits in front of the kernels it waits for
        set_error("the gated iteration needs two different streams");
        return MGWFBP_EINVAL;
    }
    // the launch that waits must not sit in front of the kernels it waits for: two streams that the
    // runtime serves from one hardware queue would do just that, and the launch would give up
    bool apart = false;
    if ((rc = streams_side_by_side(pl, compute_stream, comm_stream, apart))) return rc;
    if (!apart) {
        set_error("the device does not run these two streams' kernels at the same time (they share a "
                  "hardware queue): the gated iteration needs a pair that mgwfbp_streams_side_by_side accepts");
        return MGWFBP_ESTATE;
    }
    Events pool;
    hipEvent_t base;
    if ((rc = pool.make(&base, false))) return rc;
    const uint32_t epoch = ++pl->gated_epoch;
    const uint64_t max_polls = 1 + static_cast<uint64_t>(give_up_ms * 1000.0);  // a poll sleeps about a microsecond

    // same shape as enqueue_iteration: a gate publishes time zero, the stand-ins wait for absolute
    // deadlines; but instead of an event per group the compute stream bumps the group's arrival
    // counter, and the communication stream holds a single launch that is already running
    hipError_t e = hipSuccess;
    if ((rc = launch_spin(0.0, cs))) return rc;
    rc = launch_spin(0.3, cs, pl->d_clock);
    if (!rc && (e = hipEventRecord(base, cs)) != hipSuccess) rc = hip_fail("hipEventRecord", e);
    if (!rc && (e = hipStreamWaitEvent(ms, base, 0)) != hipSuccess) rc = hip_fail("hipStreamWaitEvent", e);
    if (!rc) rc = launch_fused_gated(*pl, update != 0, lr, momentum, pl->d_ready, epoch, pl->d_gave_up, max_polls, ms);
    if (!rc) rc = launch_spin(0.0, ms, pl->d_clock + 1);
    double elapsed_ms = 0.0;
    for (int32_t l = pl->L - 1; l >= 0 && !rc; --l) {
        elapsed_ms += tb[l];
        if (pl->merged[l]) continue;
        const size_t k = static_cast<size_t>(pl->group_of_layer[l]);
        // the stand-in for the group's lowest layer bumps the counter itself, at its end
        rc = launch_spin_until(elapsed_ms, pl->d_clock, cs, pl->d_ready + k, epoch);
    }
    const hipError_t e1 = hipStreamSynchronize(cs);
    const hipError_t e2 = hipStreamSynchronize(ms);
    if (rc) return rc;
    if (e1 != hipSuccess) return hip_fail("hipStreamSynchronize(compute)", e1);
    if (e2 != hipSuccess) return hip_fail("hipStreamSynchronize(comm)", e2);
    uint32_t gave_up = 0;
    if ((e = hipMemcpy(&gave_up, pl->d_gave_up, sizeof(gave_up), hipMemcpyDeviceToHost)) != hipSuccess)
        return hip_fail("hipMemcpy of the give-up word", e);
    if (gave_up) {
        set_error("the gated launch gave up waiting for a group's gradients (give_up_ms too short?)");
        return MGWFBP_ESTATE;
    }
    if (t_iter_ms) return read_t_iter(pl, t_iter_ms);
    return MGWFBP_OK;
}
}  // namespace

extern "C" int mgwfbp_run_iteration_gated(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr,
                                          float momentum, void *compute_stream, void *comm_stream,
                                          double give_up_ms, double *t_iter_ms)
{
    return guarded([&]() -> int {
        return run_iteration_gated_impl(pl, tb_ms, update, lr, momentum, compute_stream, comm_stream, give_up_ms,
                                        t_iter_ms);
    });
}

// ---- the same iteration as a HIP graph -------------------------------------------------------

struct mgwfbp_iteration_s {
    mgwfbp_plan_t *plan = nullptr;
    uint64_t binding_generation = 0;  // of the plan at capture: the graph holds table addresses
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

extern "C" void mgwfbp_iteration_destroy(mgwfbp_iteration_t *it);

namespace {
int iteration_capture_impl(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr,
                           float momentum, void *compute_stream, void *comm_stream,
                           mgwfbp_iteration_t **out)
{
    if (!out) {
        set_error("out is NULL");
        return MGWFBP_EINVAL;
    }
    *out = nullptr;
    const double *tb = tb_ms ? tb_ms : (pl ? pl->tb.data() : nullptr);
    int rc = check_iteration_args(pl, tb, update);
    if (rc) return rc;
    if (update && (!std::isfinite(lr) || !std::isfinite(momentum))) {
        set_error("lr and momentum must be finite");
        return MGWFBP_EINVAL;
    }
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    hipStream_t ms = static_cast<hipStream_t>(comm_stream);
    if (!cs || !ms || cs == ms) {
        set_error("capture needs two different non-default streams");
        return MGWFBP_EINVAL;
    }
    const size_t G = pl->groups.size();
    Events pool;  // the graph keeps the dependencies, not the events: they go when this call ends
    hipEvent_t base, done;
    std::vector<hipEvent_t> g_ready(G);
    rc = pool.make(&base, false);
    if (!rc) rc = pool.make(&done, false);
    for (size_t k = 0; k < G && !rc; ++k) rc = pool.make(&g_ready[k], false);
    if (rc) return rc;
    // A kernel's first use makes the runtime load and look up its code, which may allocate, and
    // capture forbids that.  So before capturing: one eager launch of the stand-in (it touches
    // no memory of the caller's), and for every group a look-up of the very kernel its launch
    // will pick, without launching it -- running a group here would write out[], w[] and v[].
    if ((rc = launch_spin(0.0, cs))) return rc;
    hipError_t e = hipStreamSynchronize(cs);
    if (e != hipSuccess) return hip_fail("hipStreamSynchronize", e);
    for (size_t k = 0; k < pl->groups.size(); ++k)
        if ((rc = resolve_scope_kernel(pl, static_cast<int32_t>(k), update != 0))) return rc;

    mgwfbp_iteration_t *it = new (std::nothrow) mgwfbp_iteration_t();
    if (!it) {
        set_error("out of host memory");
        return MGWFBP_ENOMEM;
    }
    it->plan = pl;
    it->binding_generation = pl->binding_generation;
    pl->iterations.push_back(it);  // so that destroying the plan first can be told apart
    if ((e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal)) != hipSuccess) {
        mgwfbp_iteration_destroy(it);
        return hip_fail("hipStreamBeginCapture", e);
    }
    // A short gate only: replaying a graph needs no head start for the host, but time zero still
    // has to be published by a kernel that precedes every stand-in.
    rc = enqueue_iteration(pl, tb, update != 0, lr, momentum, cs, std::vector<hipStream_t>{ms}, 0.05, base, g_ready,
                           nullptr, nullptr, std::vector<hipEvent_t>());
    // join the communication stream back into the capturing stream (also on failure, so that
    // the capture can end and both streams stay usable)
    hipError_t ej = hipEventRecord(done, ms);
    if (ej == hipSuccess) ej = hipStreamWaitEvent(cs, done, 0);
    e = hipStreamEndCapture(cs, &it->graph);
    if (rc == MGWFBP_OK && ej != hipSuccess) rc = hip_fail("joining the captured streams", ej);
    if (rc == MGWFBP_OK && e != hipSuccess) rc = hip_fail("hipStreamEndCapture", e);
    if (rc == MGWFBP_OK && (e = hipGraphInstantiate(&it->exec, it->graph, nullptr, nullptr, 0)) != hipSuccess)
        rc = hip_fail("hipGraphInstantiate", e);
    if (rc) {
        mgwfbp_iteration_destroy(it);
        return rc;
    }
    *out = it;
    return MGWFBP_OK;
}
}  // namespace

extern "C" int mgwfbp_iteration_capture(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr,
                                        float momentum, void *compute_stream, void *comm_stream,
                                        mgwfbp_iteration_t **out)
{
    return guarded([&]() -> int {
        return iteration_capture_impl(pl, tb_ms, update, lr, momentum, compute_stream, comm_stream, out);
    });
}

extern "C" int mgwfbp_iteration_replay(mgwfbp_iteration_t *it, void *hip_stream, double *t_iter_ms)
{
    return guarded([&]() -> int {
        if (!it || !it->exec) {
            set_error("iteration handle is NULL");
            return MGWFBP_EINVAL;
        }
        if (!it->plan) {
            set_error("the plan of this iteration has been destroyed");
            return MGWFBP_ESTATE;
        }
        if (!it->plan->bound || it->plan->binding_generation != it->binding_generation) {
            set_error("the plan was re-bound after the capture: capture the iteration again");
            return MGWFBP_ESTATE;
        }
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        hipError_t e = hipGraphLaunch(it->exec, s);
        if (e != hipSuccess) return hip_fail("hipGraphLaunch", e);
        if (!t_iter_ms) return MGWFBP_OK;
        if ((e = hipStreamSynchronize(s)) != hipSuccess) return hip_fail("hipStreamSynchronize", e);
        return read_t_iter(it->plan, t_iter_ms);
    });
}

namespace mgwfbp {
// The plan is going away: its iteration handles stay valid objects but can no longer replay.
void detach_iterations(mgwfbp_plan_t *pl)
{
    for (mgwfbp_iteration_s *it : pl->iterations) it->plan = nullptr;
    pl->iterations.clear();
}
}  // namespace mgwfbp

extern "C" void mgwfbp_iteration_destroy(mgwfbp_iteration_t *it)
{
    if (!it) return;
    if (it->plan) {
        std::vector<mgwfbp_iteration_s *> &v = it->plan->iterations;
        for (size_t i = 0; i < v.size(); ++i)
            if (v[i] == it) {
                v.erase(v.begin() + static_cast<std::ptrdiff_t>(i));
                break;
            }
    }
    if (it->exec) (void)hipGraphExecDestroy(it->exec);
    if (it->graph) (void)hipGraphDestroy(it->graph);
    delete it;
}
