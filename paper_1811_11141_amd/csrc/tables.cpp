// Builds the flat tables the kernels walk: one segment per layer in communication order
// (the order Algorithm 2's layer buffer is filled), and the tile list that cuts the plan
// into equal pieces of work for the workgroups.
#include "plan.hpp"

#include <algorithm>

namespace mgwfbp {

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

void build_tables(mgwfbp_plan_t &pl, const float *const *grads, float *const *out,
                  float *const *w, float *const *v, std::vector<const float *> &src_tbl,
                  std::vector<float *> &out_tbl, std::vector<float *> &w_tbl,
                  std::vector<float *> &v_tbl)
{
    const int32_t L = pl.L, N = pl.N;
    const uint32_t tile = pl.opt.tile_elems;
    const uint32_t small = std::min(pl.opt.small_elems, tile);
    // elements one gather tile may hold: a few per lane, since each costs a table search;
    // small <= tile, so no tile of any kind exceeds tile_elems (the LDS staging size)
    const uint32_t gather_cap = std::max<uint32_t>(std::min<uint32_t>(tile, 1024), small);
    std::vector<TileDev> all_slow, all_full, long_slow, long_full;
    // double-length tiles exist for 16 pieces per lane only (8192 elements)
    const uint32_t long_tile = tile == 4096 && pl.opt.long_tiles != 0 ? 8192u : 0u;

    pl.segs.clear();
    pl.tiles.clear();
    src_tbl.clear();
    out_tbl.clear();
    w_tbl.clear();
    v_tbl.clear();
    pl.all_needs_lds = false;

    for (size_t k = 0; k < pl.groups.size(); ++k) {
        GroupInfo &g = pl.groups[k];
        g.seg_begin = static_cast<uint32_t>(pl.segs.size());
        g.needs_lds = false;
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
            // A copy between the tensor and a merged buffer is a plain 128-bit copy only when
            // both sides agree on 16-byte alignment, for the group-relative and the
            // plan-relative merged layout alike.
            const uint32_t all = SEG_SRC_ALIGNED | SEG_OUT_ALIGNED | SEG_WV_ALIGNED;
            if ((s.flags & all) != all || (s.group_off & 3) || (s.plan_off & 3))
                g.needs_lds = true;
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
                } else {
                    g.needs_lds = true;
                }
                // (a lone layer of exactly one tile length runs the fast code like any full tile)
                (t.nseg == 1 && t.n == tile_len ? full : slow).push_back(t);
            }
        };
        // A launch of this group alone is short: below about 2048 workgroups it cannot fill the
        // chip and every wave's chain of dependent loads decides its duration, so the group's
        // own list uses shorter tiles (more workgroups, shorter chains) while the whole-plan
        // list keeps the long tiles that stream best.
        g.tile_elems = tile;
        while (g.tile_elems >= 2048 && (g.tile_elems / 2) % 1024 == 0 && g.tile_elems > tile / 4 &&
               (g.elems + g.tile_elems - 1) / g.tile_elems < 2048)
            g.tile_elems /= 2;
        std::vector<TileDev> slow, full;
        cut(g.tile_elems, slow, full);
        g.tile_begin = static_cast<uint32_t>(pl.tiles.size());
        pl.tiles.insert(pl.tiles.end(), slow.begin(), slow.end());
        pl.tiles.insert(pl.tiles.end(), full.begin(), full.end());
        g.tile_end = static_cast<uint32_t>(pl.tiles.size());
        cut(tile, all_slow, all_full);
        if (long_tile) cut(long_tile, long_slow, long_full);
        pl.all_needs_lds = pl.all_needs_lds || g.needs_lds;
    }
    // A second copy of the tile list for whole-plan launches: every slow tile of every group
    // first, then the full tiles.
    pl.all_tile_begin = static_cast<uint32_t>(pl.tiles.size());
    pl.tiles.insert(pl.tiles.end(), all_slow.begin(), all_slow.end());
    pl.tiles.insert(pl.tiles.end(), all_full.begin(), all_full.end());
    pl.all_tile_count = static_cast<uint32_t>(all_slow.size() + all_full.size());
    // A third copy in double-length tiles.  A workgroup lives for as long as its chain of
    // N * (pieces per lane) dependent loads, tens of microseconds, so a launch of a few
    // batches of workgroups ends with a partly filled batch that costs almost a full one.  When
    // the double-length tiles put the whole launch on the chip at once (7 waves per SIMD fit:
    // 3584 workgroups) and the ordinary tiles do not (more than 4096), the fused reduce pass
    // uses this list; it is not long enough to keep the chip busy below 2048 workgroups.
    pl.long_tile_begin = static_cast<uint32_t>(pl.tiles.size());
    pl.long_tile_count = 0;
    pl.long_tile_elems = long_tile;
    const size_t n_long = long_slow.size() + long_full.size();
    const bool by_rule = pl.all_tile_count > 4096 && n_long <= 3584 && n_long >= 2048;
    pl.long_by_default = long_tile && (pl.opt.long_tiles == 1 || by_rule);
    // kept also when the rule says no but the launch would be long enough: mgwfbp_tune may pick it
    if (long_tile && (pl.opt.long_tiles == 1 || n_long >= 2048)) {
        pl.tiles.insert(pl.tiles.end(), long_slow.begin(), long_slow.end());
        pl.tiles.insert(pl.tiles.end(), long_full.begin(), long_full.end());
        pl.long_tile_count = static_cast<uint32_t>(n_long);
    }
}

}  // namespace mgwfbp
