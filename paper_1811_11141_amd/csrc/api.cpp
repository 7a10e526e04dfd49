// extern "C" entry points of libmgwfbp: argument checking, plan life cycle, table upload and
// the translation of (group, workspace) into kernel launches.  See include/mgwfbp.h for the
// contract of every call.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "../../include/mgwfbp.h"
#include "plan.hpp"

namespace mgwfbp {

namespace {
thread_local std::string g_error;
}

void set_error(const std::string &msg) { g_error = msg; }

namespace {

int fail(int code, const std::string &msg)
{
    set_error(msg);
    return code;
}

bool good_time(double x) { return std::isfinite(x) && x >= 0.0; }

// Checks the model description and fills the parts of a plan that do not depend on the merge
// decision.  Exceptions (allocation failure) propagate to the guarded() wrapper of the caller.
int make_plan(int32_t L, const uint64_t *p, const double *tb, double tf, double a, double b,
              int32_t N, std::unique_ptr<mgwfbp_plan_t> &out)
{
    if (L < 1 || L > (1 << 20)) return fail(MGWFBP_EINVAL, "L must be in [1, 2^20]");
    if (N < 1 || N > 1024) return fail(MGWFBP_EINVAL, "N must be in [1, 1024]");
    if (!p || !tb) return fail(MGWFBP_EINVAL, "p_elems or tb_ms is NULL");
    if (!good_time(tf) || !good_time(a) || !good_time(b))
        return fail(MGWFBP_EINVAL, "tf_ms, a_ms and b_ms_per_byte must be finite and >= 0");
    // 2^40 elements (4 TiB of fp32) in total keeps every byte count below, times N + 1 <= 1025
    // workspace copies, far inside 64 bits
    const uint64_t kMaxTotal = 1ull << 40;
    uint64_t total = 0;
    for (int32_t l = 0; l < L; ++l) {
        if (p[l] == 0) return fail(MGWFBP_EINVAL, "p_elems[" + std::to_string(l) + "] is 0");
        if (p[l] > kMaxTotal || (total += p[l]) > kMaxTotal)
            return fail(MGWFBP_EINVAL, "p_elems[0.." + std::to_string(l) + "] exceed 2^40 elements in total");
        if (!good_time(tb[l]))
            return fail(MGWFBP_EINVAL, "tb_ms[" + std::to_string(l) + "] must be finite and >= 0");
    }
    std::unique_ptr<mgwfbp_plan_t> pl(new mgwfbp_plan_t());
    pl->L = L;
    pl->N = N;
    pl->p.assign(p, p + L);
    pl->tb.assign(tb, tb + L);
    pl->tf = tf;
    pl->a = a;
    pl->b = b;
    // mu_b(l) = tau_b(l) + t_b(l) with tau_b from Eq. 6: accumulate from the top layer down
    pl->mu_b.assign(L, 0.0);
    double t = tf;
    for (int32_t l = L - 1; l >= 0; --l) {
        t = t + tb[l];
        pl->mu_b[l] = t;
    }
    pl->merged.assign(L, 0);
    // 8 float4 per lane and worker in the fused kernel
    pl->opt.tile_elems = 4096;
    out = std::move(pl);
    return MGWFBP_OK;
}

void release_device(mgwfbp_plan_t *pl)
{
    if (pl->d_blob) {
        int cur = -1;
        const bool sw = hipGetDevice(&cur) == hipSuccess && cur != pl->device && pl->device >= 0;
        if (sw) (void)hipSetDevice(pl->device);
        (void)hipFree(pl->d_blob);
        if (sw) (void)hipSetDevice(cur);
    }
    pl->d_blob = nullptr;
    pl->d_clock = nullptr;
    pl->d_ready = pl->d_gave_up = pl->d_handshake = nullptr;
    pl->side_by_side.clear();
    pl->dt = DeviceTables();
    pl->bound = false;
    ++pl->binding_generation;  // graphs captured against the old tables must not run again
}

// long_ok: the caller's kernel has the double-length fast path (the fused pass without update)
int scope_of(const mgwfbp_plan_t *pl, int32_t group, LaunchScope &sc, bool long_ok = false)
{
    if (group < -1 || group >= static_cast<int32_t>(pl->groups.size()))
        return fail(MGWFBP_EINVAL, "group " + std::to_string(group) + " out of range");
    sc.pace = -1;
    sc.occupancy_lds = 0;
    sc.resolve_only = false;
    if (group < 0) {
        sc.tile_begin = pl->all_tile_begin;
        sc.n_tiles = pl->all_tile_count;
        sc.elems = pl->total_elems;
        sc.base_off = 0;
        sc.tile_elems = pl->opt.tile_elems;
        const bool use_long = pl->tuned.valid ? pl->tuned.use_long : pl->long_by_default;
        if (long_ok && pl->long_tile_count && use_long) {
            sc.tile_begin = pl->long_tile_begin;
            sc.n_tiles = pl->long_tile_count;
            sc.tile_elems = pl->long_tile_elems;
        }
        if (long_ok && pl->tuned.valid) {
            sc.pace = pl->tuned.pace;
            sc.occupancy_lds = pl->tuned.occupancy_lds;
        }
    } else {
        const GroupInfo &g = pl->groups[group];
        sc.tile_begin = g.tile_begin;
        sc.n_tiles = g.tile_end - g.tile_begin;
        sc.elems = g.elems;
        sc.base_off = g.plan_off;
        sc.tile_elems = g.tile_elems;
    }
    return MGWFBP_OK;
}

uint64_t padded(uint64_t elems) { return (elems + 63) & ~uint64_t(63); }

int check_ws(const mgwfbp_plan_t *pl, const LaunchScope &sc, void *ws, size_t bytes)
{
    if (!ws) return fail(MGWFBP_EINVAL, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(ws) & 255u)
        return fail(MGWFBP_EINVAL, "workspace must be 256-byte aligned");
    const size_t need = static_cast<size_t>(pl->N + 1) * padded(sc.elems) * sizeof(float);
    if (bytes < need)
        return fail(MGWFBP_EINVAL, "workspace too small: need " + std::to_string(need) + " bytes");
    return MGWFBP_OK;
}

int check_bound(const mgwfbp_plan_t *pl, bool need_out, bool need_wv)
{
    if (!pl) return fail(MGWFBP_EINVAL, "plan is NULL");
    if (!pl->bound) return fail(MGWFBP_ESTATE, "mgwfbp_bind has not been called");
    if (need_out && !pl->has_out) return fail(MGWFBP_ESTATE, "out[] is not bound");
    if (need_wv && !pl->has_wv) return fail(MGWFBP_ESTATE, "w[] and v[] are not bound");
    // the tables live in the memory of the device that was current at mgwfbp_bind
    int cur = -1;
    if (hipGetDevice(&cur) == hipSuccess && cur != pl->device)
        return fail(MGWFBP_ESTATE, "plan is bound on device " + std::to_string(pl->device) +
                                       " but the current device is " + std::to_string(cur));
    return MGWFBP_OK;
}

}  // namespace

int run_scope(mgwfbp_plan_t *pl, int32_t group, bool step, float lr, float mu, void *ws,
              size_t bytes, void *stream)
{
    int rc = check_bound(pl, !step, step);
    if (rc) return rc;
    if (step && (!std::isfinite(lr) || !std::isfinite(mu)))
        return fail(MGWFBP_EINVAL, "lr and momentum must be finite");
    LaunchScope sc{};
    if ((rc = scope_of(pl, group, sc, !ws && !step))) return rc;
    if (!ws) {
        if (bytes != 0) return fail(MGWFBP_EINVAL, "workspace is NULL but workspace_bytes != 0");
        return launch_fused(*pl, sc, step, lr, mu, stream);
    }
    if ((rc = check_ws(pl, sc, ws, bytes))) return rc;
    float *w = static_cast<float *>(ws);
    const uint64_t epad = padded(sc.elems);
    if ((rc = launch_pack(*pl, sc, w, epad, stream))) return rc;
    if ((rc = launch_reduce(*pl, sc, w, epad, stream))) return rc;
    return launch_unpack(*pl, sc, w + static_cast<uint64_t>(pl->N) * epad, step, lr, mu, stream);
}

int resolve_scope_kernel(mgwfbp_plan_t *pl, int32_t group, bool step)
{
    int rc = check_bound(pl, !step, step);
    if (rc) return rc;
    LaunchScope sc{};
    if ((rc = scope_of(pl, group, sc, !step))) return rc;
    sc.resolve_only = true;
    return launch_fused(*pl, sc, step, 0.0f, 0.0f, nullptr);
}

}  // namespace mgwfbp

using namespace mgwfbp;

namespace {
int bind_impl(mgwfbp_plan_t *pl, const float *const *grads, float *const *out, float *const *w,
                float *const *v)
{
    if (!pl) return fail(MGWFBP_EINVAL, "plan is NULL");
    if (!grads) return fail(MGWFBP_EINVAL, "grads is NULL");
    if ((w == nullptr) != (v == nullptr)) return fail(MGWFBP_EINVAL, "w and v must be given together");
    const int32_t L = pl->L, N = pl->N;
    for (int64_t i = 0; i < static_cast<int64_t>(N) * L; ++i) {
        if (!grads[i]) return fail(MGWFBP_EINVAL, "grads[" + std::to_string(i) + "] is NULL");
        if (reinterpret_cast<uintptr_t>(grads[i]) & 3u)
            return fail(MGWFBP_EINVAL, "grads[" + std::to_string(i) + "] is not 4-byte aligned");
    }
    for (int32_t l = 0; l < L; ++l) {
        if (out && (!out[l] || (reinterpret_cast<uintptr_t>(out[l]) & 3u)))
            return fail(MGWFBP_EINVAL, "out[" + std::to_string(l) + "] is NULL or misaligned");
        if (w && (!w[l] || !v[l] || ((reinterpret_cast<uintptr_t>(w[l]) | reinterpret_cast<uintptr_t>(v[l])) & 3u)))
            return fail(MGWFBP_EINVAL, "w/v[" + std::to_string(l) + "] is NULL or misaligned");
    }
    release_device(pl);
    pl->tuned = mgwfbp_plan_s::Tuned();
    // the device that owns the tables; its size enters the choice of tile lengths
    if (hipGetDevice(&pl->device) != hipSuccess) return fail(MGWFBP_EHIP, "hipGetDevice failed: no usable HIP device");
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, pl->device) == hipSuccess && cus > 0)
        pl->n_cus = cus;
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, pl->device) == hipSuccess && lds > 0)
        pl->lds_per_cu = static_cast<uint32_t>(lds);

    std::vector<const float *> src_tbl;
    std::vector<float *> out_tbl, w_tbl, v_tbl;
    try {
        build_tables(*pl, grads, out, w, v, src_tbl, out_tbl, w_tbl, v_tbl);
    } catch (const std::bad_alloc &) {
        return fail(MGWFBP_ENOMEM, "out of host memory");
    }

    // one device allocation: [segs][tiles][src][out][w][v][clock word], each part 256-byte aligned
    auto up = [](size_t x) { return (x + 255) & ~size_t(255); };
    const size_t b_seg = up(pl->segs.size() * sizeof(SegDev));
    const size_t b_tile = up(pl->tiles.size() * sizeof(TileDev));
    const size_t b_src = up(src_tbl.size() * sizeof(void *));
    const size_t b_ptr = up(pl->segs.size() * sizeof(void *));
    const size_t b_flags = up((pl->groups.size() + 3) * sizeof(uint32_t));
    const size_t total = b_seg + b_tile + b_src + 3 * b_ptr + 256 + b_flags;
    std::vector<char> host(total, 0);
    size_t o = 0;
    std::memcpy(host.data() + o, pl->segs.data(), pl->segs.size() * sizeof(SegDev));
    const size_t o_seg = o; o += b_seg;
    std::memcpy(host.data() + o, pl->tiles.data(), pl->tiles.size() * sizeof(TileDev));
    const size_t o_tile = o; o += b_tile;
    std::memcpy(host.data() + o, src_tbl.data(), src_tbl.size() * sizeof(void *));
    const size_t o_src = o; o += b_src;
    const size_t o_out = o; o += b_ptr;
    const size_t o_w = o; o += b_ptr;
    const size_t o_v = o; o += b_ptr;
    const size_t o_clock = o; o += 256;
    const size_t o_flags = o;
    // [arrival counters][give-up word][two handshake words]
    if (out) std::memcpy(host.data() + o_out, out_tbl.data(), out_tbl.size() * sizeof(void *));
    if (w) {
        std::memcpy(host.data() + o_w, w_tbl.data(), w_tbl.size() * sizeof(void *));
        std::memcpy(host.data() + o_v, v_tbl.data(), v_tbl.size() * sizeof(void *));
    }

    hipError_t e = hipSuccess;
    e = hipMalloc(&pl->d_blob, total);
    if (e != hipSuccess) {
        pl->d_blob = nullptr;
        return fail(e == hipErrorOutOfMemory ? MGWFBP_ENOMEM : MGWFBP_EHIP,
                    std::string("hipMalloc of the plan tables: ") + hipGetErrorString(e));
    }
    e = hipMemcpy(pl->d_blob, host.data(), total, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        release_device(pl);
        return fail(MGWFBP_EHIP, std::string("hipMemcpy of the plan tables: ") + hipGetErrorString(e));
    }
    char *d = static_cast<char *>(pl->d_blob);
    pl->dt.segs = reinterpret_cast<const SegDev *>(d + o_seg);
    pl->dt.tiles = reinterpret_cast<const TileDev *>(d + o_tile);
    pl->dt.src = reinterpret_cast<const float *const *>(d + o_src);
    pl->dt.out = out ? reinterpret_cast<float *const *>(d + o_out) : nullptr;
    pl->dt.w = w ? reinterpret_cast<float *const *>(d + o_w) : nullptr;
    pl->dt.v = w ? reinterpret_cast<float *const *>(d + o_v) : nullptr;
    pl->d_clock = reinterpret_cast<uint64_t *>(d + o_clock);
    pl->d_ready = reinterpret_cast<uint32_t *>(d + o_flags);
    pl->d_gave_up = pl->d_ready + pl->groups.size();
    pl->d_handshake = pl->d_gave_up + 1;
    pl->gated_epoch = 0;
    pl->handshake_epoch = 0;
    pl->side_by_side.clear();
    pl->host_src = src_tbl;
    pl->host_out = out_tbl;
    pl->has_out = out != nullptr;
    pl->has_wv = w != nullptr;
    pl->bound = true;
    for (int step = 0; step < 2; ++step)
        for (int lng = 0; lng < 2; ++lng)
            if (int rc = gated_resident_per_cu(step != 0, lng != 0, &pl->gated_resident_per_cu[step][lng])) {
                release_device(pl);
                return rc;
            }
    // set-up is the place for runtime queries: find this device's copy of the static workspace
    // now, so that mgwfbp_pack_reduce_unpack_static never has to ask
    if (int rc = prepare_static_workspace()) {
        release_device(pl);
        return rc;
    }
    return MGWFBP_OK;
}
}  // namespace

namespace {
int tune_impl(mgwfbp_plan_t *pl, void *hip_stream, int32_t *chosen, double *chosen_ms)
{
    int rc = check_bound(pl, true, false);
    if (rc) return rc;
    {
        std::vector<const float *> srcs(pl->host_src);
        std::sort(srcs.begin(), srcs.end());
        for (const float *o : pl->host_out)
            if (std::binary_search(srcs.begin(), srcs.end(), o))
                return fail(MGWFBP_EINVAL,
                            "mgwfbp_tune repeats the pass: out[] must not alias a gradient tensor");
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return fail(MGWFBP_EHIP, "hipEventCreate failed");
    }
    // candidate launch shapes: (longer-tile list, pause, unused LDS bytes that cap the workgroups
    // per CU at 11 / 10 instead of 16 or 14).  Index 0 is what the rules alone would do.
    struct Cand { int use_long; int pace; uint32_t lds; };
    std::vector<Cand> cands;
    cands.push_back({-1, -1, 0});
    for (int use_long = 0; use_long <= (pl->long_tile_count ? 1 : 0); ++use_long) {
        for (int pace : {1, 4, 8, 12}) cands.push_back({use_long, pace, 0});
        for (int pace : {2, 4}) cands.push_back({use_long, pace, 11000});
        cands.push_back({use_long, 2, 12500});
    }
    const mgwfbp_plan_s::Tuned before = pl->tuned;
    // launches timed per candidate: enough of them that the timed stretch is about 2 ms (4 to 32),
    // so that short launches are not chosen on noise; sized from two launches under the rules
    int reps = 4;
    {
        pl->tuned = mgwfbp_plan_s::Tuned();
        hipError_t pe = hipSuccess;
        rc = run_scope(pl, -1, false, 0.0f, 0.0f, nullptr, 0, hip_stream);
        if (!rc && (pe = hipEventRecord(e0, s)) == hipSuccess) {
            for (int i = 0; i < 2 && !rc; ++i) rc = run_scope(pl, -1, false, 0.0f, 0.0f, nullptr, 0, hip_stream);
            float ms = 0.0f;
            if (!rc && (pe = hipEventRecord(e1, s)) == hipSuccess && (pe = hipEventSynchronize(e1)) == hipSuccess &&
                (pe = hipEventElapsedTime(&ms, e0, e1)) == hipSuccess && ms > 0.0f) {
                const double want = 2.0 / (static_cast<double>(ms) / 2.0);
                reps = want < 4.0 ? 4 : want > 32.0 ? 32 : static_cast<int>(want);
            }
        }
        if (rc || pe != hipSuccess) {
            pl->tuned = before;
            (void)hipStreamSynchronize(s);
            (void)hipEventDestroy(e0);
            (void)hipEventDestroy(e1);
            return rc ? rc : fail(MGWFBP_EHIP, std::string("timing the pass: ") + hipGetErrorString(pe));
        }
    }
    int best = 0;
    double best_ms = 0.0;
    hipError_t e = hipSuccess;
    for (size_t c = 0; c < cands.size() && !rc && e == hipSuccess; ++c) {
        if (cands[c].use_long < 0) {
            pl->tuned = mgwfbp_plan_s::Tuned();
        } else {
            pl->tuned.valid = true;
            pl->tuned.use_long = cands[c].use_long != 0;
            pl->tuned.pace = cands[c].pace;
            pl->tuned.occupancy_lds = cands[c].lds;
        }
        for (int i = 0; i < 2 && !rc; ++i) rc = run_scope(pl, -1, false, 0.0f, 0.0f, nullptr, 0, hip_stream);
        if (rc) break;
        if ((e = hipEventRecord(e0, s)) != hipSuccess) break;
        for (int i = 0; i < reps && !rc; ++i)
            rc = run_scope(pl, -1, false, 0.0f, 0.0f, nullptr, 0, hip_stream);
        if (rc) break;
        if ((e = hipEventRecord(e1, s)) != hipSuccess) break;
        if ((e = hipEventSynchronize(e1)) != hipSuccess) break;
        float ms = 0.0f;
        if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) break;
        const double per = static_cast<double>(ms) / reps;
        // a candidate must beat the rules by more than the noise of the timed stretch to replace them
        if (c == 0 || per < best_ms * (best == 0 ? 0.99 : 1.0)) {
            best = static_cast<int>(c);
            best_ms = per;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc || e != hipSuccess) {
        pl->tuned = before;
        (void)hipStreamSynchronize(s);
        return rc ? rc : fail(MGWFBP_EHIP, std::string("timing a candidate: ") + hipGetErrorString(e));
    }
    if (best == 0) {
        pl->tuned = mgwfbp_plan_s::Tuned();
    } else {
        pl->tuned.valid = true;
        pl->tuned.use_long = cands[best].use_long != 0;
        pl->tuned.pace = cands[best].pace;
        pl->tuned.occupancy_lds = cands[best].lds;
    }
    if (chosen) *chosen = best;
    if (chosen_ms) *chosen_ms = best_ms;
    return MGWFBP_OK;
}
}  // namespace

namespace {
int scaling_curve_impl(int32_t L, const uint64_t *p_elems, const double *tb_ms, double tf_ms,
                         int32_t algorithm, double alpha_ms, double beta, double gamma,
                         int32_t n_points, const int32_t *n_workers, int32_t mode,
                         double *t_iter_ms, double *speedup)
{
    if (n_points < 0 || (n_points > 0 && !n_workers)) return fail(MGWFBP_EINVAL, "bad n_points / n_workers");
    for (int32_t i = 0; i < n_points; ++i) {
        double a = 0, b = 0;
        int rc = mgwfbp_table2_cost(algorithm, n_workers[i], alpha_ms, beta, gamma, &a, &b);
        if (rc) return rc;
        mgwfbp_plan_t *pl = nullptr;
        if ((rc = mgwfbp_plan(L, p_elems, tb_ms, tf_ms, a, b, n_workers[i], mode, &pl))) return rc;
        const double t = pl->t_iter;
        double compute = tf_ms;  // t_f + t_b of one worker
        for (int32_t l = 0; l < L; ++l) compute += tb_ms[l];
        mgwfbp_plan_destroy(pl);
        if (t_iter_ms) t_iter_ms[i] = t;
        if (speedup) speedup[i] = t > 0 ? static_cast<double>(n_workers[i]) * compute / t : 0.0;
    }
    return MGWFBP_OK;
}
}  // namespace

extern "C" {

int mgwfbp_plan(int32_t L, const uint64_t *p_elems, const double *tb_ms, double tf_ms,
                double a_ms, double b_ms_per_byte, int32_t N, int32_t mode, mgwfbp_plan_t **out)
{
    if (!out) return guarded([]() -> int { return fail(MGWFBP_EINVAL, "out is NULL"); });
    *out = nullptr;
    return guarded([&]() -> int {
        if (mode < MGWFBP_MODE_OPTIMAL || mode > MGWFBP_MODE_SINGLE) return fail(MGWFBP_EINVAL, "unknown mode");
        std::unique_ptr<mgwfbp_plan_t> pl;
        int rc = make_plan(L, p_elems, tb_ms, tf_ms, a_ms, b_ms_per_byte, N, pl);
        if (rc) return rc;
        switch (mode) {
        case MGWFBP_MODE_OPTIMAL: plan_optimal(*pl, pl->merged); break;
        case MGWFBP_MODE_PAPER_GREEDY: plan_paper_greedy(*pl, pl->merged); break;
        case MGWFBP_MODE_WFBP: pl->merged.assign(L, 0); break;
        case MGWFBP_MODE_SINGLE:
            pl->merged.assign(L, 1);
            pl->merged[0] = 0;
            break;
        }
        finish_plan(*pl);
        *out = pl.release();
        return MGWFBP_OK;
    });
}

int mgwfbp_plan_explicit(int32_t L, const uint64_t *p_elems, const double *tb_ms, double tf_ms,
                         double a_ms, double b_ms_per_byte, int32_t N, const uint8_t *merged,
                         mgwfbp_plan_t **out)
{
    if (!out) return guarded([]() -> int { return fail(MGWFBP_EINVAL, "out is NULL"); });
    *out = nullptr;
    return guarded([&]() -> int {
        if (!merged) return fail(MGWFBP_EINVAL, "merged is NULL");
        std::unique_ptr<mgwfbp_plan_t> pl;
        int rc = make_plan(L, p_elems, tb_ms, tf_ms, a_ms, b_ms_per_byte, N, pl);
        if (rc) return rc;
        if (merged[0])
            return fail(MGWFBP_EINVAL, "merged[0] must be 0: the lowest layer has nothing below it");
        for (int32_t l = 0; l < L; ++l) pl->merged[l] = merged[l] ? 1 : 0;
        finish_plan(*pl);
        *out = pl.release();
        return MGWFBP_OK;
    });
}

int mgwfbp_plan_info(const mgwfbp_plan_t *pl, int32_t *n_groups, int32_t *group_of_layer,
                     uint64_t *offset_in_group, uint64_t *group_elems, double *t_iter_ms,
                     double *t_iter_wfbp_ms)
{
    return guarded([&]() -> int {
        if (!pl) return fail(MGWFBP_EINVAL, "plan is NULL");
        if (n_groups) *n_groups = static_cast<int32_t>(pl->groups.size());
        if (group_of_layer) std::memcpy(group_of_layer, pl->group_of_layer.data(), sizeof(int32_t) * pl->L);
        if (offset_in_group) std::memcpy(offset_in_group, pl->off_in_group.data(), sizeof(uint64_t) * pl->L);
        if (group_elems)
            for (size_t k = 0; k < pl->groups.size(); ++k) group_elems[k] = pl->groups[k].elems;
        if (t_iter_ms) *t_iter_ms = pl->t_iter;
        if (t_iter_wfbp_ms) *t_iter_wfbp_ms = pl->t_iter_wfbp;
        return MGWFBP_OK;
    });
}

int mgwfbp_plan_timeline(const mgwfbp_plan_t *pl, double *mu_b, double *group_start,
                         double *group_finish)
{
    return guarded([&]() -> int {
        if (!pl) return fail(MGWFBP_EINVAL, "plan is NULL");
        if (mu_b) std::memcpy(mu_b, pl->mu_b.data(), sizeof(double) * pl->L);
        for (size_t k = 0; k < pl->groups.size(); ++k) {
            if (group_start) group_start[k] = pl->groups[k].start_ms;
            if (group_finish) group_finish[k] = pl->groups[k].finish_ms;
        }
        return MGWFBP_OK;
    });
}

int mgwfbp_plan_set_option(mgwfbp_plan_t *pl, int32_t key, int64_t value)
{
    return guarded([&]() -> int {
        if (!pl) return fail(MGWFBP_EINVAL, "plan is NULL");
        if (pl->bound) return fail(MGWFBP_ESTATE, "options must be set before mgwfbp_bind");
        switch (key) {
        case MGWFBP_OPT_TILE_ELEMS:
            // upper bound: the longest tile the fused reduce pass has a fast path for
            if (value < 1024 || value > 8192 || (value % 1024) != 0)
                return fail(MGWFBP_EINVAL, "tile_elems must be a multiple of 1024 in [1024, 8192]");
            pl->opt.tile_elems = static_cast<uint32_t>(value);
            return MGWFBP_OK;
        case MGWFBP_OPT_SMALL_ELEMS:
            if (value < 0 || value > 8192) return fail(MGWFBP_EINVAL, "small_elems must be in [0, 8192]");
            pl->opt.small_elems = static_cast<uint32_t>(value);
            return MGWFBP_OK;
        case MGWFBP_OPT_NONTEMPORAL:
            if (value != 0 && value != 1) return fail(MGWFBP_EINVAL, "nontemporal must be 0 or 1");
            pl->opt.nontemporal = static_cast<int>(value);
            return MGWFBP_OK;
        case MGWFBP_OPT_PACE:
            if (value < -1 || value > 16) return fail(MGWFBP_EINVAL, "pace must be in [-1, 16]");
            pl->opt.pace = static_cast<int>(value);
            return MGWFBP_OK;
        case MGWFBP_OPT_PAD_ELEMS:
            if (value != 0 && value != 4 && value != 8 && value != 16 && value != 32)
                return fail(MGWFBP_EINVAL, "pad_elems must be 0, 4, 8, 16 or 32");
            pl->opt.pad_elems = static_cast<uint32_t>(value);
            finish_plan(*pl);  // offsets and group sizes follow the layout
            return MGWFBP_OK;
        case MGWFBP_OPT_LONG_TILES:
            if (!(value >= -1 && value <= 1) && value != 5120 && value != 6144 && value != 7168 && value != 8192)
                return fail(MGWFBP_EINVAL, "long_tiles must be -1, 0, 1, 5120, 6144, 7168 or 8192");
            pl->opt.long_tiles = static_cast<int>(value);
            return MGWFBP_OK;
        case MGWFBP_OPT_UPDATE_WGS_PER_CU:
            if (value != -1 && value != 0 && !(value >= 8 && value <= 11))
                return fail(MGWFBP_EINVAL, "update_wgs_per_cu must be -1, 0, 8, 9, 10 or 11");
            pl->opt.update_wgs_per_cu = static_cast<int>(value);
            return MGWFBP_OK;
        case MGWFBP_OPT_GATED_WGS_PER_CU:
            if (value != -1 && !(value >= 1 && value <= 15))
                return fail(MGWFBP_EINVAL, "gated_wgs_per_cu must be -1 or 1 .. 15");
            pl->opt.gated_wgs_per_cu = static_cast<int>(value);
            return MGWFBP_OK;
        case MGWFBP_OPT_GATED_CUS:
            if (value < 0 || value > 65536) return fail(MGWFBP_EINVAL, "gated_cus must be 0 (all) or a number of compute units");
            pl->opt.gated_cus = static_cast<int>(value);
            return MGWFBP_OK;
        default: return fail(MGWFBP_EINVAL, "unknown option key");
        }
    });
}

int mgwfbp_plan_layout(const mgwfbp_plan_t *pl, uint64_t *n_segments, uint64_t *segments,
                       size_t segments_cap, uint64_t *n_tiles, uint64_t *tiles, size_t tiles_cap)
{
    return guarded([&]() -> int {
        if (!pl) return fail(MGWFBP_EINVAL, "plan is NULL");
        // the tables are built on a copy, from placeholder pointers that are only inspected for
        // their alignment and never dereferenced; the copy owns no device memory
        mgwfbp_plan_t tmp = *pl;
        tmp.d_blob = nullptr;
        tmp.d_clock = nullptr;
        tmp.bound = false;
        const size_t L = static_cast<size_t>(pl->L), N = static_cast<size_t>(pl->N);
        float *const fake = reinterpret_cast<float *>(uintptr_t(1) << 20);
        std::vector<const float *> g(N * L, fake);
        std::vector<float *> o(L, fake);
        std::vector<const float *> src_tbl;
        std::vector<float *> out_tbl, w_tbl, v_tbl;
        build_tables(tmp, g.data(), o.data(), o.data(), o.data(), src_tbl, out_tbl, w_tbl, v_tbl);
        if (n_segments) *n_segments = tmp.segs.size();
        if (n_tiles) *n_tiles = tmp.tiles.size();
        if (segments) {
            if (segments_cap < tmp.segs.size()) return fail(MGWFBP_EINVAL, "segments array too small");
            for (size_t i = 0; i < tmp.segs.size(); ++i) {
                const SegDev &sd = tmp.segs[i];
                uint64_t *r = segments + MGWFBP_LAYOUT_SEGMENT_COLS * i;
                r[0] = sd.layer; r[1] = sd.n; r[2] = sd.plan_off; r[3] = sd.group;
            }
        }
        if (tiles) {
            if (tiles_cap < tmp.tiles.size()) return fail(MGWFBP_EINVAL, "tiles array too small");
            for (size_t i = 0; i < tmp.tiles.size(); ++i) {
                const TileDev &t = tmp.tiles[i];
                uint64_t *r = tiles + MGWFBP_LAYOUT_TILE_COLS * i;
                r[0] = t.seg; r[1] = t.nseg; r[2] = t.start; r[3] = t.n; r[6] = t.pad;
                r[4] = i >= tmp.all_tile_begin ? 1 : 0;
                r[5] = tmp.opt.tile_elems;
                if (tmp.long_tile_count && i >= tmp.long_tile_begin) {
                    r[4] = tmp.long_by_default ? 2 : 3;
                    r[5] = tmp.long_tile_elems;
                }
                if (i >= tmp.ordered_tile_begin) {
                    r[4] = 4;
                    r[5] = tmp.groups[tmp.segs[t.seg].group].gated_tile_elems;
                }
            }
            // the per-group lists carry their own (possibly halved) tile length
            for (const GroupInfo &g : tmp.groups)
                for (size_t i = g.tile_begin; i < g.tile_end; ++i)
                    tiles[MGWFBP_LAYOUT_TILE_COLS * i + 5] = g.tile_elems;
        }
        return MGWFBP_OK;
    });
}

int mgwfbp_bind(mgwfbp_plan_t *pl, const float *const *grads, float *const *out, float *const *w,
                float *const *v)
{
    return guarded([&]() -> int { return bind_impl(pl, grads, out, w, v); });
}

int mgwfbp_workspace_bytes(const mgwfbp_plan_t *pl, int32_t group, size_t *bytes)
{
    return guarded([&]() -> int {
        if (!pl || !bytes) return fail(MGWFBP_EINVAL, "plan or bytes is NULL");
        uint64_t elems;
        if (group == -1) elems = pl->total_elems;
        else if (group >= 0 && group < static_cast<int32_t>(pl->groups.size())) elems = pl->groups[group].elems;
        else return fail(MGWFBP_EINVAL, "group out of range");
        *bytes = static_cast<size_t>(pl->N + 1) * padded(elems) * sizeof(float);
        return MGWFBP_OK;
    });
}

int mgwfbp_pack_reduce_unpack(mgwfbp_plan_t *pl, int32_t group, void *workspace,
                              size_t workspace_bytes, void *hip_stream)
{
    return guarded([&]() -> int {
        return run_scope(pl, group, false, 0.0f, 0.0f, workspace, workspace_bytes, hip_stream);
    });
}

int mgwfbp_step(mgwfbp_plan_t *pl, int32_t group, float lr, float momentum, void *workspace,
                size_t workspace_bytes, void *hip_stream)
{
    return guarded([&]() -> int {
        return run_scope(pl, group, true, lr, momentum, workspace, workspace_bytes, hip_stream);
    });
}

int mgwfbp_pack(mgwfbp_plan_t *pl, int32_t group, void *workspace, size_t workspace_bytes,
                void *hip_stream)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, false, false);
        if (rc) return rc;
        LaunchScope sc{};
        if ((rc = scope_of(pl, group, sc))) return rc;
        if ((rc = check_ws(pl, sc, workspace, workspace_bytes))) return rc;
        return launch_pack(*pl, sc, static_cast<float *>(workspace), padded(sc.elems), hip_stream);
    });
}

int mgwfbp_reduce(mgwfbp_plan_t *pl, int32_t group, void *workspace, size_t workspace_bytes,
                  void *hip_stream)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, false, false);
        if (rc) return rc;
        LaunchScope sc{};
        if ((rc = scope_of(pl, group, sc))) return rc;
        if ((rc = check_ws(pl, sc, workspace, workspace_bytes))) return rc;
        return launch_reduce(*pl, sc, static_cast<float *>(workspace), padded(sc.elems), hip_stream);
    });
}

int mgwfbp_unpack(mgwfbp_plan_t *pl, int32_t group, void *workspace, size_t workspace_bytes,
                  void *hip_stream)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, true, false);
        if (rc) return rc;
        LaunchScope sc{};
        if ((rc = scope_of(pl, group, sc))) return rc;
        if ((rc = check_ws(pl, sc, workspace, workspace_bytes))) return rc;
        const float *reduced = static_cast<float *>(workspace) + static_cast<uint64_t>(pl->N) * padded(sc.elems);
        return launch_unpack(*pl, sc, reduced, false, 0.0f, 0.0f, hip_stream);
    });
}

int mgwfbp_tune(mgwfbp_plan_t *pl, void *hip_stream, int32_t *chosen, double *chosen_ms)
{
    return guarded([&]() -> int { return tune_impl(pl, hip_stream, chosen, chosen_ms); });
}

namespace {
int check_merged(const LaunchScope &sc, void *merged, size_t bytes)
{
    if (!merged) return fail(MGWFBP_EINVAL, "merged is NULL");
    if (reinterpret_cast<uintptr_t>(merged) & 255u)
        return fail(MGWFBP_EINVAL, "merged must be 256-byte aligned");
    if (bytes < sc.elems * sizeof(float))
        return fail(MGWFBP_EINVAL, "merged buffer too small: need " +
                                       std::to_string(sc.elems * sizeof(float)) + " bytes");
    return MGWFBP_OK;
}
}  // namespace

int mgwfbp_pack_reduce(mgwfbp_plan_t *pl, int32_t group, void *merged, size_t merged_bytes,
                       void *hip_stream)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, false, false);
        if (rc) return rc;
        LaunchScope sc{};
        if ((rc = scope_of(pl, group, sc, true))) return rc;
        if ((rc = check_merged(sc, merged, merged_bytes))) return rc;
        return launch_fused(*pl, sc, false, 0.0f, 0.0f, hip_stream, static_cast<float *>(merged));
    });
}

int mgwfbp_unpack_update(mgwfbp_plan_t *pl, int32_t group, const void *merged, size_t merged_bytes,
                         int32_t update, float lr, float momentum, void *hip_stream)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, !update, update != 0);
        if (rc) return rc;
        if (update && (!std::isfinite(lr) || !std::isfinite(momentum)))
            return fail(MGWFBP_EINVAL, "lr and momentum must be finite");
        LaunchScope sc{};
        if ((rc = scope_of(pl, group, sc))) return rc;
        if ((rc = check_merged(sc, const_cast<void *>(merged), merged_bytes))) return rc;
        return launch_unpack(*pl, sc, static_cast<const float *>(merged), update != 0, lr, momentum, hip_stream);
    });
}

}  // extern "C"

namespace mgwfbp {
int streams_side_by_side(mgwfbp_plan_t *pl, void *stream_a, void *stream_b, bool &yes)
{
    yes = false;
    if (stream_a == stream_b) return MGWFBP_OK;
    for (const auto &pr : pl->side_by_side)
        if (pr.first == stream_a && pr.second == stream_b) {
            yes = true;
            return MGWFBP_OK;
        }
    // a kernel on stream_b waits (for at most 2 ms) for a word that a kernel put into stream_a
    // AFTER it writes; it sees the word only if the device runs the two streams' kernels at once
    const uint32_t value = ++pl->handshake_epoch;
    int rc = launch_signal(pl->d_handshake + 1, 0u, stream_b);
    if (!rc) rc = launch_await(pl->d_handshake, value, pl->d_handshake + 1, 2000, stream_b);
    if (!rc) rc = launch_signal(pl->d_handshake, value, stream_a);
    const hipError_t e1 = hipStreamSynchronize(static_cast<hipStream_t>(stream_a));
    const hipError_t e2 = hipStreamSynchronize(static_cast<hipStream_t>(stream_b));
    if (rc) return rc;
    if (e1 != hipSuccess || e2 != hipSuccess) {
        set_error(std::string("hipStreamSynchronize in the stream handshake: ") +
                  hipGetErrorString(e1 != hipSuccess ? e1 : e2));
        return MGWFBP_EHIP;
    }
    uint32_t seen = 0;
    const hipError_t e = hipMemcpy(&seen, pl->d_handshake + 1, sizeof(seen), hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        set_error(std::string("hipMemcpy of the handshake word: ") + hipGetErrorString(e));
        return MGWFBP_EHIP;
    }
    yes = seen == 1u;
    if (yes) pl->side_by_side.emplace_back(stream_a, stream_b);
    return MGWFBP_OK;
}
}  // namespace mgwfbp

extern "C" {

int mgwfbp_gated_launch(mgwfbp_plan_t *pl, int32_t update, float lr, float momentum, uint32_t arrival,
                        double give_up_ms, void *hip_stream)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, !update, update != 0);
        if (rc) return rc;
        if (update && (!std::isfinite(lr) || !std::isfinite(momentum)))
            return fail(MGWFBP_EINVAL, "lr and momentum must be finite");
        if (!(give_up_ms > 0.0) || give_up_ms > 6.0e4) return fail(MGWFBP_EINVAL, "give_up_ms must be in (0, 60000]");
        return launch_fused_gated(*pl, update != 0, lr, momentum, pl->d_ready, arrival, pl->d_gave_up,
                                  1 + static_cast<uint64_t>(give_up_ms * 1000.0), hip_stream);
    });
}

int mgwfbp_streams_side_by_side(mgwfbp_plan_t *pl, void *stream_a, void *stream_b, int32_t *side_by_side)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, false, false);
        if (rc) return rc;
        if (!side_by_side) return fail(MGWFBP_EINVAL, "side_by_side is NULL");
        bool yes = false;
        if ((rc = streams_side_by_side(pl, stream_a, stream_b, yes))) return rc;
        *side_by_side = yes ? 1 : 0;
        return MGWFBP_OK;
    });
}

int mgwfbp_confined_stream_create(uint32_t n_compute_units, void **hip_stream)
{
    return guarded([&]() -> int {
        if (!hip_stream) return fail(MGWFBP_EINVAL, "hip_stream is NULL");
        *hip_stream = nullptr;
        int dev = 0, cus = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return fail(MGWFBP_EHIP, std::string("device query: ") + hipGetErrorString(e));
        if (n_compute_units == 0 || n_compute_units % 32 != 0 || static_cast<int>(n_compute_units) >= cus)
            return fail(MGWFBP_EINVAL, "n_compute_units must be a multiple of 32 below the device's " +
                                           std::to_string(cus) + " compute units");
        // one bit per compute unit, whole 32-bit words: the first n_compute_units of the device
        std::vector<uint32_t> mask(static_cast<size_t>((cus + 31) / 32), 0u);
        for (uint32_t i = 0; i < n_compute_units / 32; ++i) mask[i] = 0xffffffffu;
        hipStream_t s = nullptr;
        e = hipExtStreamCreateWithCUMask(&s, static_cast<uint32_t>(mask.size()), mask.data());
        if (e != hipSuccess) return fail(MGWFBP_EHIP, std::string("hipExtStreamCreateWithCUMask: ") + hipGetErrorString(e));
        *hip_stream = s;
        return MGWFBP_OK;
    });
}

int mgwfbp_confined_stream_destroy(void *hip_stream)
{
    return guarded([&]() -> int {
        if (!hip_stream) return MGWFBP_OK;
        const hipError_t e = hipStreamDestroy(static_cast<hipStream_t>(hip_stream));
        if (e != hipSuccess) return fail(MGWFBP_EHIP, std::string("hipStreamDestroy: ") + hipGetErrorString(e));
        return MGWFBP_OK;
    });
}

int mgwfbp_gated_workgroups(mgwfbp_plan_t *pl, int32_t update, uint32_t *workgroups, uint32_t *per_compute_unit)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, false, false);
        if (rc) return rc;
        if (!workgroups && !per_compute_unit) return fail(MGWFBP_EINVAL, "both outputs are NULL");
        const uint32_t g = gated_grid(*pl, update != 0);
        uint32_t cus = static_cast<uint32_t>(pl->n_cus > 0 ? pl->n_cus : 256);
        if (pl->opt.gated_cus > 0) cus = std::min(cus, static_cast<uint32_t>(pl->opt.gated_cus));
        if (workgroups) *workgroups = g;
        if (per_compute_unit) *per_compute_unit = (g + cus - 1) / cus;
        return MGWFBP_OK;
    });
}

int mgwfbp_gated_signal(mgwfbp_plan_t *pl, int32_t group, uint32_t arrival, void *hip_stream)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, false, false);
        if (rc) return rc;
        if (group < 0 || group >= static_cast<int32_t>(pl->groups.size()))
            return fail(MGWFBP_EINVAL, "group " + std::to_string(group) + " out of range");
        return launch_signal(pl->d_ready + group, arrival, hip_stream);
    });
}

int mgwfbp_gated_gave_up(mgwfbp_plan_t *pl, int32_t *gave_up)
{
    return guarded([&]() -> int {
        int rc = check_bound(pl, false, false);
        if (rc) return rc;
        if (!gave_up) return fail(MGWFBP_EINVAL, "gave_up is NULL");
        uint32_t word = 0;
        const hipError_t e = hipMemcpy(&word, pl->d_gave_up, sizeof(word), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail(MGWFBP_EHIP, std::string("hipMemcpy of the give-up word: ") + hipGetErrorString(e));
        *gave_up = word != 0;
        return MGWFBP_OK;
    });
}

int mgwfbp_fit_cost(int32_t n, const double *bytes, const double *ms, double *a_ms,
                    double *b_ms_per_byte)
{
    return guarded([&]() -> int {
        if (!bytes || !ms || !a_ms || !b_ms_per_byte) return fail(MGWFBP_EINVAL, "NULL argument");
        if (n < 2) return fail(MGWFBP_EINVAL, "need at least two measurements");
        double sx = 0, sy = 0;
        for (int32_t i = 0; i < n; ++i) {
            if (!std::isfinite(bytes[i]) || !std::isfinite(ms[i]) || bytes[i] < 0)
                return fail(MGWFBP_EINVAL, "measurements must be finite, sizes >= 0");
            sx += bytes[i];
            sy += ms[i];
        }
        const double mx = sx / n, my = sy / n;
        double sxx = 0, sxy = 0, sxx0 = 0, sxy0 = 0;
        for (int32_t i = 0; i < n; ++i) {
            sxx += (bytes[i] - mx) * (bytes[i] - mx);
            sxy += (bytes[i] - mx) * (ms[i] - my);
            sxx0 += bytes[i] * bytes[i];
            sxy0 += bytes[i] * ms[i];
        }
        if (!(sxx > 0)) return fail(MGWFBP_EINVAL, "need at least two distinct message sizes");
        double b = sxy / sxx;
        double a = my - b * mx;
        if (a < 0) {  // refit through the origin
            a = 0;
            b = sxy0 / sxx0;
        }
        if (b < 0) b = 0;
        *a_ms = a;
        *b_ms_per_byte = b;
        return MGWFBP_OK;
    });
}

int mgwfbp_table2_cost(int32_t algorithm, int32_t N, double alpha, double beta, double gamma,
                       double *a_ms, double *b_ms_per_byte)
{
    return guarded([&]() -> int {
        if (!a_ms || !b_ms_per_byte) return fail(MGWFBP_EINVAL, "NULL argument");
        if (N < 1) return fail(MGWFBP_EINVAL, "N must be >= 1");
        if (!good_time(alpha) || !good_time(beta) || !good_time(gamma))
            return fail(MGWFBP_EINVAL, "alpha, beta, gamma must be finite and >= 0");
        const double n = static_cast<double>(N), lg = std::log2(n);
        switch (algorithm) {
        case 0: *a_ms = 2 * alpha * lg; *b_ms_per_byte = (2 * beta + gamma) * lg; break;
        case 1: *a_ms = alpha * lg; *b_ms_per_byte = (beta + gamma) * lg; break;
        case 2: *a_ms = 2 * alpha * lg; *b_ms_per_byte = 2 * beta - (2 * beta + gamma) / n + gamma; break;
        case 3: *a_ms = 2 * (n - 1) * alpha; *b_ms_per_byte = 2 * (n - 1) / n * beta + (n - 1) / n * gamma; break;
        default: return fail(MGWFBP_EINVAL, "algorithm must be 0..3");
        }
        return MGWFBP_OK;
    });
}

int mgwfbp_scaling_curve(int32_t L, const uint64_t *p_elems, const double *tb_ms, double tf_ms,
                         int32_t algorithm, double alpha_ms, double beta, double gamma,
                         int32_t n_points, const int32_t *n_workers, int32_t mode,
                         double *t_iter_ms, double *speedup)
{
    return guarded([&]() -> int {
        return scaling_curve_impl(L, p_elems, tb_ms, tf_ms, algorithm, alpha_ms, beta, gamma, n_points,
                                  n_workers, mode, t_iter_ms, speedup);
    });
}

void mgwfbp_plan_destroy(mgwfbp_plan_t *pl)
{
    if (!pl) return;
    detach_iterations(pl);
    release_device(pl);
    delete pl;
}

const char *mgwfbp_last_error(void) { return g_error.c_str(); }

}  // extern "C"
