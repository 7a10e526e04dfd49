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
        const hipError_t e = timed ? hipEventCreate(out) : hipEventCreateWithFlags(out, hipEventDisableTiming);
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

extern "C" int mgwfbp_run_iteration(mgwfbp_plan_t *pl, const double *tb_ms, int32_t update, float lr,
                                    float momentum, void *compute_stream, void *comm_stream,
                                    double *group_ready_ms, double *group_start_ms,
                                    double *group_finish_ms, double *t_iter_ms)
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
    const int32_t L = pl->L;
    const size_t G = pl->groups.size();
    const double *tb = tb_ms ? tb_ms : pl->tb.data();
    for (int32_t l = 0; l < L; ++l) {
        if (!(tb[l] >= 0.0) || tb[l] > 1.0e4) {
            set_error("tb_ms[" + std::to_string(l) + "] must be in [0, 10000] ms");
            return MGWFBP_EINVAL;
        }
    }
    hipStream_t cs = static_cast<hipStream_t>(compute_stream);
    hipStream_t ms = static_cast<hipStream_t>(comm_stream);

    // Per-group timestamps are taken only when the caller asks for them: a timed event record
    // costs a few microseconds of stream time, which is a large part of a short group's cost.
    const bool time_ready = group_ready_ms != nullptr;
    const bool time_comm = group_start_ms != nullptr || group_finish_ms != nullptr;
    Events pool;
    hipEvent_t base, done;
    std::vector<hipEvent_t> g_ready(G), g_start(time_comm ? G : 0), g_finish(time_comm ? G : 0);
    int rc = pool.make(&base);
    if (!rc) rc = pool.make(&done);
    for (size_t k = 0; k < G && !rc; ++k) {
        rc = pool.make(&g_ready[k], time_ready);
        if (!rc && time_comm) rc = pool.make(&g_start[k]);
        if (!rc && time_comm) rc = pool.make(&g_finish[k]);
    }
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
    if ((rc = launch_spin(1.0 + 0.06 * static_cast<double>(G), cs, pl->d_clock))) return rc;
    // the communication stream must not start before the backward pass does
    hipError_t e = hipEventRecord(base, cs);
    if (e != hipSuccess) return hip_fail("hipEventRecord", e);
    if ((e = hipStreamWaitEvent(ms, base, 0)) != hipSuccess) return hip_fail("hipStreamWaitEvent", e);

    // Backward pass, highest layer first.  Only the moment a group's lowest layer finishes
    // matters to the communication side, so the layers of a group share one stand-in kernel
    // that ends when the backward pass has reached the end of the group's lowest layer.
    double elapsed_ms = 0.0;
    for (int32_t l = L - 1; l >= 0; --l) {
        elapsed_ms += tb[l];
        if (pl->merged[l]) continue;  // layer l rides with layer l-1: nothing is sent yet
        // layer l is the lowest layer of its group: the group's gradients are complete
        const size_t k = static_cast<size_t>(pl->group_of_layer[l]);
        if ((rc = launch_spin_until(elapsed_ms, pl->d_clock, cs))) break;
        if ((e = hipEventRecord(g_ready[k], cs)) != hipSuccess) {
            rc = hip_fail("hipEventRecord", e);
            break;
        }
        if ((e = hipStreamWaitEvent(ms, g_ready[k], 0)) != hipSuccess) {
            rc = hip_fail("hipStreamWaitEvent", e);
            break;
        }
        if (time_comm && (e = hipEventRecord(g_start[k], ms)) != hipSuccess) {
            rc = hip_fail("hipEventRecord", e);
            break;
        }
        if ((rc = run_scope(pl, static_cast<int32_t>(k), update != 0, lr, momentum, nullptr, 0, ms)))
            break;
        if (time_comm && (e = hipEventRecord(g_finish[k], ms)) != hipSuccess) {
            rc = hip_fail("hipEventRecord", e);
            break;
        }
    }
    // groups run in order on the communication stream: its end is the end of the iteration (Eq. 8)
    if (!rc && (e = hipEventRecord(done, ms)) != hipSuccess) rc = hip_fail("hipEventRecord", e);
    // whatever was enqueued must drain before the events are destroyed or read
    const hipError_t e1 = hipStreamSynchronize(cs);
    const hipError_t e2 = hipStreamSynchronize(ms);
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
    double total = 0.0;
    if ((rc = since_base(done, &total))) return rc;
    if (t_iter_ms) *t_iter_ms = total;
    return MGWFBP_OK;
}
