// Stand-ins for the kernel launchers, so that the host sources of the library (api, planner,
// tables, executor) link into a host-only test binary without any device code.  No test that
// uses them reaches a launch: every launch path is refused earlier (plan not bound).
#include "../../paper_1811_11141_amd/csrc/plan.hpp"

namespace mgwfbp {
int launch_fused(const mgwfbp_plan_t &, const LaunchScope &, bool, float, float, void *, float *) { return MGWFBP_EHIP; }
int launch_pack(const mgwfbp_plan_t &, const LaunchScope &, float *, uint64_t, void *) { return MGWFBP_EHIP; }
int launch_reduce(const mgwfbp_plan_t &, const LaunchScope &, float *, uint64_t, void *) { return MGWFBP_EHIP; }
int launch_unpack(const mgwfbp_plan_t &, const LaunchScope &, const float *, bool, float, float, void *) { return MGWFBP_EHIP; }
int launch_spin(double, void *, uint64_t *) { return MGWFBP_EHIP; }
int launch_spin_until(double, uint64_t *, void *, uint32_t *, uint32_t) { return MGWFBP_EHIP; }
int wall_clock_khz() { return 100000; }
int prepare_static_workspace() { return MGWFBP_EHIP; }
int launch_fused_gated(const mgwfbp_plan_t &, bool, float, float, const uint32_t *, uint32_t, uint32_t *, uint64_t, void *) { return MGWFBP_EHIP; }
int launch_signal(uint32_t *, uint32_t, void *) { return MGWFBP_EHIP; }
uint32_t gated_grid(const mgwfbp_plan_t &, bool) { return 0; }
int gated_resident_per_cu(bool, bool, int *) { return MGWFBP_EHIP; }
int launch_await(const uint32_t *, uint32_t, uint32_t *, uint64_t, void *) { return MGWFBP_EHIP; }
}  // namespace mgwfbp
