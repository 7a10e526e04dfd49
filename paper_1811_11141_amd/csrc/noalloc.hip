// mgwfbp_pack_reduce_unpack_static: the materialised pack -> reduce -> unpack path with its
// workspace in a file-scope device array instead of caller memory, for callers that cannot
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// The array's name is a host-side stand-in, not a device address.  Its address on a device is
// asked from the runtime once per device (at mgwfbp_bind, with that device current, or at the
// first call on a device that was never bound on) and kept; every use of the memory from host
// code goes through that pointer.  Each device holds its own copy of the array from the moment
// the library's code is loaded there until the process ends.
#include <hip/hip_runtime.h>

#include <atomic>
#include <string>

#include "../../include/mgwfbp.h"
#include "plan.hpp"

namespace {

constexpr size_t kScratchBytes = size_t(64) << 20;  // MGWFBP_STATIC_WORKSPACE_BYTES
static_assert(kScratchBytes == MGWFBP_STATIC_WORKSPACE_BYTES, "header and array disagree");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of the array on the current device; resolves it on first use.
int scratch_on_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        mgwfbp::set_error(e != hipSuccess ? std::string("hipGetDevice: ") + hipGetErrorString(e)
                                          : "device index beyond the static workspace table");
        return MGWFBP_EHIP;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            mgwfbp::set_error(std::string("hipGetSymbolAddress of the static workspace: ") + hipGetErrorString(e));
            return MGWFBP_EHIP;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return MGWFBP_OK;
}

}  // namespace

namespace mgwfbp {

int prepare_static_workspace()
{
    void *p = nullptr;
    return scratch_on_current_device(&p);
}

}  // namespace mgwfbp

extern "C" int mgwfbp_pack_reduce_unpack_static(mgwfbp_plan_t *pl, int32_t group, void *hip_stream)
{
    return mgwfbp::guarded([&]() -> int {
        if (pl && !pl->bound) {
            mgwfbp::set_error("mgwfbp_bind has not been called");
            return MGWFBP_ESTATE;
        }
        size_t need = 0;
        int rc = mgwfbp_workspace_bytes(pl, group, &need);
        if (rc) return rc;
        if (need > kScratchBytes) {
            mgwfbp::set_error("the static workspace holds " + std::to_string(kScratchBytes) + " bytes, this call needs " +
                              std::to_string(need) + ": use mgwfbp_pack_reduce_unpack with a workspace of your own");
            return MGWFBP_EINVAL;
        }
        // the plan's own checks (bound, out[] present, current device) come before the address:
        // a bound plan has resolved it at mgwfbp_bind, so no runtime query happens here
        void *ws = nullptr;
        if ((rc = scratch_on_current_device(&ws))) return rc;
        return mgwfbp::run_scope(pl, group, false, 0.0f, 0.0f, ws, kScratchBytes, hip_stream);
    });
}
