// Internal data structures of libmgwfbp: the host-side plan and the device tables the
// kernels walk.  Not part of the public ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "../../include/mgwfbp.h"

namespace mgwfbp {

// One layer's gradient inside the plan.  Segments are stored in communication order:
// group 0 first, and inside a group the highest layer first (the order Algorithm 2's
// layer buffer receives them).
struct SegDev {
    uint64_t n;          // elements p_l
    uint64_t plan_off;   // offset in plan-wide merged coordinates (groups laid end to end)
    uint64_t group_off;  // offset inside its own group's merged buffer
    uint32_t layer;      // 0-based layer index
    uint32_t group;
    uint32_t flags;      // SEG_* bits
    uint32_t pad;
};
static_assert(sizeof(SegDev) == 40, "SegDev layout");

enum : uint32_t {
    SEG_SRC_ALIGNED = 1u,  // all N gradient pointers of the layer are 16-byte aligned
    SEG_OUT_ALIGNED = 2u,  // out pointer (if bound) is 16-byte aligned
    SEG_WV_ALIGNED = 4u,   // w and v pointers (if bound) are 16-byte aligned
};

// Unit of work of one workgroup.
//   nseg == 1 : "direct" tile, elements [start, start+n) of segment `seg`
//   nseg  > 1 : "gather" tile, plan-wide merged coordinates [start, start+n), covering the
//               whole of segments seg .. seg+nseg-1 (all of them short)
struct TileDev {
    uint64_t start;
    uint32_t seg;
    uint32_t nseg;
    uint32_t n;
    uint32_t pad;
};
static_assert(sizeof(TileDev) == 24, "TileDev layout");

constexpr uint32_t kMaxGatherSegs = 256;  // segments one gather tile may span
// arrival-ordered list: groups of up to kGatedSmallGroupElems elements are cut into kGatedShortTile pieces
constexpr uint32_t kGatedShortTile = 512;
constexpr uint64_t kGatedSmallGroupElems = 64u * 1024u;

struct DeviceTables {
    const SegDev *segs = nullptr;
    const TileDev *tiles = nullptr;
    const float *const *src = nullptr;  // [n_segs * N], segment-major
    float *const *out = nullptr;        // [n_segs] or null
    float *const *w = nullptr;          // [n_segs] or null
    float *const *v = nullptr;          // [n_segs] or null
};

struct Options {
    uint32_t tile_elems = 4096;
    uint32_t small_elems = 64;
    int nontemporal = 1;
    int pace = -1;  // -1: chosen per launch from its size and N
    uint32_t pad_elems = 0;  // 0: merged buffers hold exactly sum p; 4 .. 32: every layer starts on a multiple
    int long_tiles = -1;  // tile length of the whole-plan fused reduce pass: -1 by rule, 0 = tile_elems,
                          // 1 = 8192, or 5120 / 6144 / 7168 / 8192 elements
    int update_wgs_per_cu = -1;  // update kernel: -1 by rule, 0 uncapped, 8..11 forced
    int gated_wgs_per_cu = -1;   // gated launch: -1 = all but the reserve, or 1..15
    int gated_cus = 0;           // gated launch: compute units its stream may use (0 = all of the device)
};

struct GroupInfo {
    std::vector<int32_t> layers;  // arrival order (highest first)
    uint64_t elems = 0;
    uint64_t plan_off = 0;
    uint32_t seg_begin = 0, seg_end = 0;
    uint32_t tile_begin = 0, tile_end = 0;
    uint32_t tile_elems = 0;  // tile length of the group's own list (<= the plan's tile_elems)
    uint32_t gated_tile_elems = 0;  // and of its part of the arrival-ordered list
    double start_ms = 0, finish_ms = 0;
};

}  // namespace mgwfbp

struct mgwfbp_plan_s {
    int32_t L = 0, N = 0;
    std::vector<uint64_t> p;
    std::vector<double> tb;
    double tf = 0, a = 0, b = 0;
    std::vector<uint8_t> merged;  // merged[l] != 0: layer l rides with layer l-1
    std::vector<double> mu_b;
    std::vector<int32_t> group_of_layer;
    std::vector<uint64_t> off_in_group;
    std::vector<mgwfbp::GroupInfo> groups;
    double t_iter = 0, t_iter_wfbp = 0;
    uint64_t total_elems = 0;

    mgwfbp::Options opt;

    // binding
    bool bound = false, has_out = false, has_wv = false;
    int device = -1;
    uint32_t all_tile_begin = 0, all_tile_count = 0;  // whole-plan ordering of the tiles
    // third list: the whole plan cut into longer tiles, for the fused reduce pass when that fills
    // the chip's batches of workgroups better (0 tiles = not built)
    uint32_t long_tile_begin = 0, long_tile_count = 0, long_tile_elems = 0;
    // fourth list: the whole plan group after group in communication order (inside a group slow
    // tiles first), in tiles of its own length (gated_tile_elems; small groups 512), for the
    // single gated launch that walks the groups in the order their gradients arrive
    uint32_t ordered_tile_begin = 0, ordered_tile_count = 0;
    uint32_t gated_tile_elems = 4096;  // full-tile length of that list: 1024 or 4096
    std::vector<const float *> host_src;  // host copies of the bound pointers (alias checks)
    std::vector<float *> host_out;
    bool long_by_default = false;  // the rule (or the option) says to use it
    // launch shape of the whole-plan fused reduce pass found by mgwfbp_tune (valid = false: rules)
    struct Tuned {
        bool valid = false;
        bool use_long = false;
        int pace = 0;
        uint32_t occupancy_lds = 0;  // dynamic LDS bytes requested only to cap workgroups per CU
    } tuned;
    std::vector<mgwfbp::SegDev> segs;
    std::vector<mgwfbp::TileDev> tiles;
    void *d_blob = nullptr;  // one device allocation holding every table
    int n_cus = 256;  // compute units of the device the plan is bound on (MI355X until bound)
    uint32_t lds_per_cu = 160u * 1024u;  // LDS bytes per compute unit of that device
    uint64_t binding_generation = 0;  // bumped whenever the device tables are released or replaced
    std::vector<struct mgwfbp_iteration_s *> iterations;  // graphs captured from this plan and still alive
    // two words at the end of d_blob: device clock at the start and at the end of an iteration
    uint64_t *d_clock = nullptr;
    // behind them, for the gated launch: one arrival counter per group and the give-up word
    uint32_t *d_ready = nullptr, *d_gave_up = nullptr;
    // workgroups of the gated kernel a compute unit holds: [reduce, update][1024-, 4096-element tiles]
    int gated_resident_per_cu[2][2] = {{0, 0}, {0, 0}};
    uint32_t gated_epoch = 0;  // arrival number the executor used last
    // and two words for the handshake that shows whether two streams' kernels run at the same time
    uint32_t *d_handshake = nullptr;
    uint32_t handshake_epoch = 0;
    std::vector<std::pair<void *, void *>> side_by_side;  // (signalling, waiting) stream pairs that passed it
    mgwfbp::DeviceTables dt;
};

namespace mgwfbp {

void set_error(const std::string &msg);

// Runs f and turns any C++ exception into a status code: nothing may propagate through the C ABI.
template <class F>
int guarded(F f) noexcept
{
    try {
        return f();
    } catch (const std::bad_alloc &) {
        try {
            set_error("out of host memory");
        } catch (...) {
        }
        return MGWFBP_ENOMEM;
    } catch (...) {
        try {
            set_error("unexpected C++ exception");
        } catch (...) {
        }
        return MGWFBP_EHIP;
    }
}

// planner.cpp
double simulate(const mgwfbp_plan_t &pl, const std::vector<uint8_t> &merged,
                std::vector<double> *group_start, std::vector<double> *group_finish);
void plan_optimal(const mgwfbp_plan_t &pl, std::vector<uint8_t> &merged);
void plan_paper_greedy(const mgwfbp_plan_t &pl, std::vector<uint8_t> &merged);
void finish_plan(mgwfbp_plan_t &pl);

// api.cpp
int run_scope(mgwfbp_plan_t *pl, int32_t group, bool step, float lr, float mu, void *ws,
              size_t bytes, void *stream);
// Makes the runtime look up the kernel run_scope would launch for the fused form of `group`,
// without launching it.
int resolve_scope_kernel(mgwfbp_plan_t *pl, int32_t group, bool step);

// executor.cpp
void detach_iterations(mgwfbp_plan_t *pl);

// noalloc.hip: resolves the device address of the library's static workspace on the current
// device (once per device; mgwfbp_bind calls it so that later calls need no runtime query)
int prepare_static_workspace();

// tables.cpp
void build_tables(mgwfbp_plan_t &pl, const float *const *grads, float *const *out,
                  float *const *w, float *const *v, std::vector<const float *> &src_tbl,
                  std::vector<float *> &out_tbl, std::vector<float *> &w_tbl,
                  std::vector<float *> &v_tbl);

// Tile lengths the fused reduce pass can run on its fast path (8, 10, 12, 14, 16 pieces per lane)
// and the rule that picks one for a launch.  tables.cpp
constexpr int kTileChoices = 5;
constexpr uint32_t kTileChoice[kTileChoices] = {4096, 5120, 6144, 7168, 8192};
// Workgroups of the fused reduce kernel one compute unit holds at once (from its register use;
// a test checks the table against the compiled code).
int fused_workgroups_per_cu(int n_workers, uint32_t tile_elems);
// Predicted efficiency (0..1] of a launch of `workgroups` when `resident` fit the chip at once.
double launch_fill_efficiency(uint64_t workgroups, uint64_t resident, int n_cus);
// Index into kTileChoice of the best tile length for the given workgroup counts per choice.
int best_tile_choice(int n_workers, int n_cus, const uint64_t (&workgroups)[kTileChoices]);

// Unused dynamic LDS (bytes) that makes the update kernel's launch of `workgroups` fill the chip
// best by lowering the workgroups per compute unit; 0 = none.  forced_per_cu: -1 = by the rule,
// 0 = none, 8..11 = that many.  tables.cpp
uint32_t update_occupancy_lds(int n_workers, int n_cus, uint32_t lds_per_cu, uint64_t workgroups,
                              int forced_per_cu);

// kernels.hip
struct LaunchScope {
    uint32_t tile_begin, n_tiles;
    uint64_t elems;       // elements in scope (one group or the whole plan)
    uint64_t base_off;    // plan_off of the scope's first element
    uint32_t tile_elems;  // length of the full tiles in this scope's list
    int pace;                // >= 0: use this pause instead of the rule
    uint32_t occupancy_lds;  // unused dynamic LDS bytes, to cap the workgroups per CU (0 = no cap)
    bool resolve_only;       // look the kernel up in the runtime instead of launching it
};
int launch_fused(const mgwfbp_plan_t &pl, const LaunchScope &sc, bool step, float lr, float mu,
                 void *stream, float *merged_out = nullptr);
int launch_pack(const mgwfbp_plan_t &pl, const LaunchScope &sc, float *ws, uint64_t epad,
                void *stream);
int launch_reduce(const mgwfbp_plan_t &pl, const LaunchScope &sc, float *ws, uint64_t epad,
                  void *stream);
int launch_unpack(const mgwfbp_plan_t &pl, const LaunchScope &sc, const float *reduced, bool step,
                  float lr, float mu, void *stream);
// One launch over the whole plan in arrival order; a tile runs once its group's counter has
// reached `epoch` (or the launch gives up after max_polls polls of ~1 us and says so in *ctl).
// ctl: the plan's give-up word; a small kernel in front of the launch clears it.
int launch_fused_gated(const mgwfbp_plan_t &pl, bool step, float lr, float mu, const uint32_t *ready,
                       uint32_t epoch, uint32_t *ctl, uint64_t max_polls, void *stream);
// How many workgroups of the gated kernel (update form or not, 4096- or 1024-element tiles) one
// compute unit of the current device holds.
int gated_resident_per_cu(bool step, bool long_tiles, int *per_cu);
// Workgroups the gated launch would use now (0: the device holds too few, or nothing to do).
uint32_t gated_grid(const mgwfbp_plan_t &pl, bool step);
// Sets *counter = epoch (device scope, release) behind the work already in the stream.
int launch_signal(uint32_t *counter, uint32_t epoch, void *stream);
// One wave polls *word until it equals `value` (then *result = 1) or max_polls polls of ~1 us have
// passed (then *result = 2).
int launch_await(const uint32_t *word, uint32_t value, uint32_t *result, uint64_t max_polls, void *stream);
// Do kernels of stream_a run while a kernel of stream_b is still running?  Streams that the runtime
// serves from one hardware queue do not.  Pairs that passed are remembered in the plan.
int streams_side_by_side(mgwfbp_plan_t *pl, void *stream_a, void *stream_b, bool &yes);
// Timed stand-ins for the backward pass: wait `ms`, optionally publishing the device clock at the
// end; or wait until `deadline_ms` after the published clock value and then, if `arrive` is given,
// set *arrive = epoch as the gated launch's signal.
int launch_spin(double ms, void *stream, uint64_t *publish_clock = nullptr);
int launch_spin_until(double deadline_ms, uint64_t *clock, void *stream, uint32_t *arrive = nullptr,
                      uint32_t epoch = 0);
int wall_clock_khz();  // ticks per millisecond of the device clock the stand-ins read

}  // namespace mgwfbp
