// Builds the flat tables the kernels walk: one segment per layer in communication order
// (the order Algorithm 2's layer buffer is filled), and the tile list that cuts the plan
// into equal pieces of work for the workgroups.
#include "plan.hpp"

#include <algorithm>
#include <cmath>

namespace mgwfbp {

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

// The fused reduce kernel needs 38-61 VGPRs up to 14 pieces per lane (8 waves per SIMD, 16
// workgroups of two waves per compute unit) and 69 with 16 pieces (7 waves, 14 workgroups); with
// 16 workers it holds 93 SGPRs, which also allows 7 waves only.
int fused_workgroups_per_cu(int n_workers, uint32_t tile_elems)
{
    return (n_workers >= 16 || tile_elems >= 8192) ? 14 : 16;
}

// A workgroup lives for as long as its chain of N * (pieces per lane) dependent loads, tens of
// microseconds, and the workgroups of a launch start in batches of `resident`.  Measured on
// MI355X (single tensors of 3 k to 34 k tiles, N = 8 and 16, five tile lengths; start and end
// times of every workgroup recorded with the device clock):
//   * full batches run at the same rate whatever their number;
//   * a last batch filled to at least ~65 % costs its share; one filled less costs as much as a
//     65 % one, because a workgroup running on a nearly empty chip is bound by latency (a few
//     stragglers cost most of a batch; a launch of exactly k batches still has them, since the
//     first workgroups start before the rest and finish out of step);
//   * a launch that fits the chip at once streams best with 11-13 workgroups per compute unit
//     (5600-6600 waves in flight); up to 95 % of the slots it loses ~3 %, beyond that ~6 %, and
//     below 11 per unit there is too little in flight.
double launch_fill_efficiency(uint64_t workgroups, uint64_t resident, int n_cus)
{
    if (workgroups == 0 || resident == 0) return 1.0;
    const double w = static_cast<double>(workgroups), s = static_cast<double>(resident);
    if (w <= s) {
        const double lo = 11.0 * n_cus, hi = 13.0 * n_cus;
        if (w < lo) return 0.5 + 0.5 * w / lo;
        if (w <= hi) return 1.0;
        return w <= 0.95 * s ? 0.97 : 0.94;
    }
    const double x = w / s, k = std::floor(x), f = x - k;
    return x / (k + std::max(f, 0.65));
}

int best_tile_choice(int n_workers, int n_cus, const uint64_t (&workgroups)[kTileChoices])
{
    int best = 0;
    double best_eff = 0.0;
    for (int c = 0; c < kTileChoices; ++c) {
        // a launch of fewer than 8 workgroups per compute unit is too short to stream: not a candidate
        if (c > 0 && workgroups[c] < 8ull * static_cast<uint64_t>(n_cus)) break;
        const uint64_t resident = static_cast<uint64_t>(fused_workgroups_per_cu(n_workers, kTileChoice[c])) * n_cus;
        const double eff = launch_fill_efficiency(workgroups[c], resident, n_cus);
        // a longer tile must promise at least 2 % to replace a shorter one
        if (c == 0 || eff > best_eff + 0.02) {
            best = c;
            best_eff = eff;
        }
    }
    return best;
}

// The update kernel (k_fused with the SGD-momentum step) on 4096-element tiles.  It holds 14
// workgroups per compute unit (68 VGPRs: 7 waves per SIMD; 12 for N = 16, whose 105 SGPRs
// allow 6 -- a test recomputes both from the compiled kernels, and both are where the steps
// of the measured staircase fall), its fast path exists for this tile length only, and size
// sweeps (3 k to 20 k workgroups, N = 8 and 16) show the same staircase as
// the reduce pass: a launch that just overflows a batch of resident workgroups pays for most of
// another batch -- here 0.3 of one plus 0.7 of its share -- so the efficiency swings between 64 %
// and 80 % of peak with the size of the net.  What can be chosen per launch without another tile
// list is the batch itself: unused dynamic LDS lowers the workgroups a compute unit holds
// (11 000 / 12 500 / 14 000 / 16 000 bytes give 11 / 10 / 9 / 8 on gfx950's 160 KiB; checked by
// where the dips of the sweeps fall), which moves the steps of the staircase.  With fewer
// workgroups per unit the well-filled launch itself gets a little slower (peak column, measured).
// Returns the LDS bytes to request; 0 = leave the launch alone.
uint32_t update_occupancy_lds(int n_workers, int n_cus, uint32_t lds_per_cu, uint64_t workgroups,
                              int forced_per_cu)
{
    // The byte counts below are measured ones for this LDS size.  Asking the runtime's occupancy
    // calculator for them instead was tried: the counts it named for 10 and for 9 workgroups per
    // unit ran at identical speed, and the rule built on them chose worse shapes than none (a
    // tensor of 5002 tiles: 201 us against 181 us uncapped and 170 us at a true 11 per unit).
    if (lds_per_cu != 160u * 1024u) return 0;
    if (forced_per_cu == 0) return 0;
    if (forced_per_cu > 0) {
        switch (forced_per_cu) {
        case 11: return 11000;
        case 10: return 12500;
        case 9: return 14000;
        case 8: return 16000;
        default: return 0;
        }
    }
    if (n_workers != 1 && n_workers != 2 && n_workers != 4 && n_workers != 8 && n_workers != 16) return 0;
    // short launches (under 8 workgroups per compute unit) run the deeper-pipelined kernel
    if (n_cus <= 0 || workgroups < 8ull * static_cast<uint64_t>(n_cus)) return 0;
    struct Choice { int per_cu; uint32_t lds; double peak; };
    const Choice choices[] = {{n_workers >= 16 ? 12 : 14, 0, 1.0}, {11, 11000, 1.0}, {10, 12500, 0.985},
                              {9, 14000, 0.955}, {8, 16000, 0.915}};
    uint32_t best_lds = 0;
    double best = 0.0;
    for (const Choice &c : choices) {
        if (c.lds != 0 && c.per_cu >= choices[0].per_cu) continue;
        const double x = static_cast<double>(workgroups) / (static_cast<double>(c.per_cu) * n_cus);
        const double k = std::floor(x), f = x - k;
        double fill;
        if (k < 1.0) fill = std::min(1.0, x / 0.8);
        else fill = x / (k + (f > 0.0 ? 0.3 + 0.7 * f : 0.0));
        const double eff = c.peak * fill;
        // a cap must promise 2 % over the uncapped launch
        if (c.lds == 0 || eff > best + (best_lds == 0 ? 0.02 : 0.0)) {
            best = eff;
            best_lds = c.lds;
        }
    }
    return best_lds;
}

void build_tables(mgwfbp_plan_t &pl, const float *const *grads, float *const *out,
                  float *const *w, float *const *v, std::vector<const float *> &src_tbl,
                  std::vector<float *> &out_tbl, std::vector<float *> &w_tbl,
                  std::vector<float *> &v_tbl)
{
    const int32_t L = pl.L, N = pl.N;
    const uint32_t tile = pl.opt.tile_elems;
    const uint32_t small = std::min(pl.opt.small_elems, tile);
    // elements one gather tile may hold: a few per lane, since each costs a table search;
    // small <= tile, so no tile of any kind exceeds tile_elems
    const uint32_t gather_cap = std::max<uint32_t>(std::min<uint32_t>(tile, 1024), small);
    std::vector<TileDev> all_slow, all_full, ordered;
    // the longer tile lengths the fused reduce pass may use instead (only next to 4096)
    const bool longer_ok = tile == 4096 && pl.opt.long_tiles != 0;
    std::vector<TileDev> alt_slow[kTileChoices], alt_full[kTileChoices];

    pl.segs.clear();
    pl.tiles.clear();
    src_tbl.clear();
    out_tbl.clear();
    w_tbl.clear();
    v_tbl.clear();

    // Tile length of the arrival-ordered list (the gated launch), whatever tile_elems says: its
    // workgroups stay and walk several tiles each, so the length only sets how finely the work is
    // dealt and how long a tile that is alone on the chip takes (a full tile is a chain of N * U
    // loads, each waited for).  A plan that the launch covers in about two passes of 4096-element
    // tiles is cut into 1024-element tiles (GoogLeNet's sizes against 4096: 99 -> 81 us with every
    // group arrived, ResNet-50's update 237 -> 225 us, its reduction 145 -> 148 us; a 4 MB message
    // that arrives alone is done after 13 us instead of 22 us with 2048); a long plan keeps 4096
    // (VGG-16, N = 16: 1556 us against 1666 us with 2048, every tile pays its table loads and its
    // store drain).  One length per plan: the tiles are dealt by count, and a mix of lengths leaves
    // the workgroups with unequal shares (AlexNet's sizes with two of four groups in 1024-element
    // tiles: 339 -> 361 us).
    {
        uint64_t total = 0;
        for (const GroupInfo &g : pl.groups) total += g.elems;
        const uint64_t two_passes = 2ull * 14ull * static_cast<uint64_t>(pl.n_cus > 0 ? pl.n_cus : 256);
        pl.gated_tile_elems = (total + 4095) / 4096 <= two_passes ? 1024u : 4096u;
    }
    const uint64_t short_launch = 8ull * static_cast<uint64_t>(pl.n_cus > 0 ? pl.n_cus : 256);  // workgroups
    for (size_t k = 0; k < pl.groups.size(); ++k) {
        GroupInfo &g = pl.groups[k];
        g.seg_begin = static_cast<uint32_t>(pl.segs.size());
        for (int32_t l : g.layers) {
            SegDev s{};
            s.n = pl.p[l];
            s.group_off = pl.off_in_group[l];
            s.plan_off = g.plan_off + s.group_off;
            s.layer = static_cast<uint32_t>(l);
            s.group = static_cast<uint32_t>(k);
            bool src_al = true;
            for (int32_t r = 0; r < N; ++r) {
                const float *ptr = grads[static_cast<size_t>(r) * L + l];
                src_al = src_al && aligned16(ptr);
                src_tbl.push_back(ptr);
            }
            if (src_al) s.flags |= SEG_SRC_ALIGNED;
            if (out) {
                out_tbl.push_back(out[l]);
                if (aligned16(out[l])) s.flags |= SEG_OUT_ALIGNED;
            } else {
                s.flags |= SEG_OUT_ALIGNED;
            }
            if (w) {
                w_tbl.push_back(w[l]);
                v_tbl.push_back(v[l]);
                if (aligned16(w[l]) && aligned16(v[l])) s.flags |= SEG_WV_ALIGNED;
            } else {
                s.flags |= SEG_WV_ALIGNED;
            }
            pl.segs.push_back(s);
        }
        g.seg_end = static_cast<uint32_t>(pl.segs.size());

        // Tiles of this group.  Long layers are cut into direct tiles; a run of short
        // layers shares gather tiles so that tiny tensors cost no workgroup each.  Gather
        // tiles and ragged tails run the general (slower) code path, so they are listed first:
        // workgroups are dispatched in order and the slow ones then overlap with the bulk.
        const uint64_t pad = pl.opt.pad_elems > 1 ? pl.opt.pad_elems : 1;
        auto padded_len = [pad](uint64_t n) { return (n + pad - 1) / pad * pad; };
        auto cut = [&](uint32_t tile_len, std::vector<TileDev> &slow, std::vector<TileDev> &full) {
            uint32_t s = g.seg_begin;
            while (s < g.seg_end) {
                const SegDev &sd = pl.segs[s];
                if (sd.n >= small) {
                    for (uint64_t st = 0; st < sd.n; st += tile_len) {
                        TileDev t{};
                        t.start = st;
                        t.seg = s;
                        t.nseg = 1;
                        t.n = static_cast<uint32_t>(std::min<uint64_t>(tile_len, sd.n - st));
                        // the last piece also owns the padding that follows the layer
                        if (st + t.n == sd.n) t.pad = static_cast<uint32_t>(padded_len(sd.n) - sd.n);
                        (t.n == tile_len ? full : slow).push_back(t);
                    }
                    ++s;
                    continue;
                }
                TileDev t{};
                t.start = sd.plan_off;
                t.seg = s;
                uint64_t n = 0;
                uint32_t cnt = 0;
                // n counts the run in the merged order, padding between the layers included
                while (s < g.seg_end && pl.segs[s].n < small && cnt < kMaxGatherSegs &&
                       (cnt == 0 || n + padded_len(pl.segs[s].n) <= gather_cap)) {
                    n += padded_len(pl.segs[s].n);
                    ++cnt;
                    ++s;
                }
                t.nseg = cnt;
                t.n = static_cast<uint32_t>(n);
                if (cnt == 1) {  // a lone short layer is an ordinary direct tile
                    t.start = 0;
                    t.n = static_cast<uint32_t>(sd.n);
                    t.pad = static_cast<uint32_t>(padded_len(sd.n) - sd.n);
                }
                // (a lone layer of exactly one tile length runs the fast code like any full tile)
                (t.nseg == 1 && t.n == tile_len ? full : slow).push_back(t);
            }
        };
        // A launch of this group alone is short: below about 8 workgroups per compute unit (half
        // the chip's wave slots) it cannot fill the chip and every wave's chain of dependent loads
        // decides its duration, so the group's own list uses shorter tiles (more workgroups,
        // shorter chains) while the whole-plan list keeps the long tiles that stream best.
        g.tile_elems = tile;
        while (g.tile_elems >= 2048 && (g.tile_elems / 2) % 1024 == 0 && g.tile_elems > tile / 4 &&
               (g.elems + g.tile_elems - 1) / g.tile_elems < short_launch)
            g.tile_elems /= 2;
        std::vector<TileDev> slow, full;
        cut(g.tile_elems, slow, full);
        g.tile_begin = static_cast<uint32_t>(pl.tiles.size());
        pl.tiles.insert(pl.tiles.end(), slow.begin(), slow.end());
        pl.tiles.insert(pl.tiles.end(), full.begin(), full.end());
        g.tile_end = static_cast<uint32_t>(pl.tiles.size());
        cut(tile, all_slow, all_full);
        {
            // In the gated launch a small group is usually alone on the chip when it arrives, and a
            // full tile is then a chain of N * 8 loads, each waited for (35 us for N = 8).  Cut into
            // 512-element pieces the group runs the general code instead: one 128-bit access per
            // lane and worker, four in flight.
            g.gated_tile_elems = g.elems <= kGatedSmallGroupElems ? kGatedShortTile : pl.gated_tile_elems;
            std::vector<TileDev> os, of;
            cut(g.gated_tile_elems, os, of);
            ordered.insert(ordered.end(), os.begin(), os.end());
            ordered.insert(ordered.end(), of.begin(), of.end());
        }
        if (longer_ok)
            for (int c = 1; c < kTileChoices; ++c) cut(kTileChoice[c], alt_slow[c], alt_full[c]);
    }
    // A second copy of the tile list for whole-plan launches: every slow tile of every group
    // first, then the full tiles.
    pl.all_tile_begin = static_cast<uint32_t>(pl.tiles.size());
    pl.tiles.insert(pl.tiles.end(), all_slow.begin(), all_slow.end());
    pl.tiles.insert(pl.tiles.end(), all_full.begin(), all_full.end());
    pl.all_tile_count = static_cast<uint32_t>(all_slow.size() + all_full.size());
    // A third copy in longer tiles for the fused reduce pass, whose fast path exists for 8 to 16
    // pieces per lane: the length that fills the batches of workgroups best (see
    // launch_fill_efficiency), or the one the option names.  It is the default for whole-plan
    // reduce launches when the rule prefers it to the 4096-element list; otherwise it is only
    // kept, when long enough, for mgwfbp_tune to try.
    pl.long_tile_begin = static_cast<uint32_t>(pl.tiles.size());
    pl.long_tile_count = 0;
    pl.long_tile_elems = 0;
    pl.long_by_default = false;
    if (longer_ok) {
        uint64_t counts[kTileChoices];
        counts[0] = pl.all_tile_count;
        for (int c = 1; c < kTileChoices; ++c) counts[c] = alt_slow[c].size() + alt_full[c].size();
        int pick = 0;
        if (pl.opt.long_tiles == -1) {
            pick = best_tile_choice(pl.N, pl.n_cus, counts);
            pl.long_by_default = pick != 0;
            if (pick == 0) {  // nothing beats 4096: keep the best of the others for the tuner
                double best_eff = 0.0;
                for (int c = 1; c < kTileChoices && counts[c] >= short_launch; ++c) {
                    const uint64_t res = static_cast<uint64_t>(fused_workgroups_per_cu(pl.N, kTileChoice[c])) * pl.n_cus;
                    const double eff = launch_fill_efficiency(counts[c], res, pl.n_cus);
                    if (eff > best_eff) {
                        best_eff = eff;
                        pick = c;
                    }
                }
            }
        } else {
            const uint32_t want = pl.opt.long_tiles == 1 ? 8192u : static_cast<uint32_t>(pl.opt.long_tiles);
            for (int c = 1; c < kTileChoices; ++c)
                if (kTileChoice[c] == want) pick = c;
            pl.long_by_default = pick != 0;
        }
        if (pick != 0) {
            pl.tiles.insert(pl.tiles.end(), alt_slow[pick].begin(), alt_slow[pick].end());
            pl.tiles.insert(pl.tiles.end(), alt_full[pick].begin(), alt_full[pick].end());
            pl.long_tile_count = static_cast<uint32_t>(counts[pick]);
            pl.long_tile_elems = kTileChoice[pick];
        }
    }
    // A fourth copy in arrival order, for the gated launch.
    pl.ordered_tile_begin = static_cast<uint32_t>(pl.tiles.size());
    pl.ordered_tile_count = static_cast<uint32_t>(ordered.size());
    pl.tiles.insert(pl.tiles.end(), ordered.begin(), ordered.end());
}

}  // namespace mgwfbp
