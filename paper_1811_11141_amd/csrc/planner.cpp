// Host-side merge planner: the timeline model of Section II-C (Eq. 6-8) with the all-reduce
// cost of Eq. 9, merged layers obeying Conditions 1-3 (Eq. 14-16), and two ways of choosing
// the merged-gradient set M of Eq. 22: an exact dynamic program over contiguous groups, and
// the rule of Theorem 1 as Algorithm 1 applies it.
//
// Index convention: vectors are 0-based, element l is the paper's layer l+1.  The backward
// pass runs from index L-1 down to 0.
#include "plan.hpp"

#include <algorithm>
#include <limits>

namespace mgwfbp {

namespace {

constexpr uint64_t kBytesPerParam = 4;  // fp32 gradients (Section V)

inline double t_ar(const mgwfbp_plan_t &pl, uint64_t bytes)
{
    return pl.a + pl.b * static_cast<double>(bytes);  // Eq. 9
}

}  // namespace

// Iteration time of Eq. 8 for a given M.  Going down the layers, parameters pile up
// (Condition 3) until a layer that is not merged sends them; its message starts when the
// previous message is done and its own gradients are ready (Eq. 7, Condition 2).
double simulate(const mgwfbp_plan_t &pl, const std::vector<uint8_t> &merged,
                std::vector<double> *group_start, std::vector<double> *group_finish)
{
    double channel_free = 0.0;
    uint64_t pending = 0;
    if (group_start) group_start->clear();
    if (group_finish) group_finish->clear();
    for (int32_t l = pl.L - 1; l >= 0; --l) {
        pending += kBytesPerParam * pl.p[l];
        if (merged[l]) continue;
        const double start = std::max(channel_free, pl.mu_b[l]);
        channel_free = start + t_ar(pl, pending);
        pending = 0;
        if (group_start) group_start->push_back(start);
        if (group_finish) group_finish->push_back(channel_free);
    }
    return channel_free;
}

// Exact minimum of Eq. 19-23.  best[k] is the earliest moment the channel can be free after
// everything from layer k upwards has been sent, given that a message ends at layer k.  A
// message covering layers k..j starts at max(best[j+1], mu_b[k]) and that start is monotone
// in best[j+1], so the optimal prefix is also the optimal prefix of the whole plan.
// O(L^2) time at worst, the cost the paper quotes for Algorithm 1.  Growing the message upwards
// makes it longer (bytes only grow) while its start can never drop below mu_b[k], so the search
// for layer k stops as soon as a message that starts at mu_b[k] could no longer beat the best
// one found: with compute-bound stretches in the net that is after a few layers, which keeps
// nets of a million layers plannable.  The bound is evaluated with the same expression as the
// candidates (floating-point addition is monotone), so the result is the unpruned one.
void plan_optimal(const mgwfbp_plan_t &pl, std::vector<uint8_t> &merged)
{
    const int32_t L = pl.L;
    std::vector<double> best(L + 1, 0.0);
    std::vector<int32_t> top(L, 0);  // highest layer of the message whose lowest layer is k
    for (int32_t k = L - 1; k >= 0; --k) {
        double best_t = std::numeric_limits<double>::infinity();
        int32_t best_j = k;
        uint64_t bytes = 0;
        for (int32_t j = k; j < L; ++j) {
            bytes += kBytesPerParam * pl.p[j];
            const double cost = t_ar(pl, bytes);
            if (!(pl.mu_b[k] + cost < best_t)) break;  // no longer message can be strictly better
            const double t = std::max(best[j + 1], pl.mu_b[k]) + cost;
            if (t < best_t) {  // strict: on a tie keep the smaller group
                best_t = t;
                best_j = j;
            }
        }
        best[k] = best_t;
        top[k] = best_j;
    }
    merged.assign(L, 0);
    int32_t k = 0;
    while (k < L) {
        const int32_t j = top[k];
        for (int32_t l = k + 1; l <= j; ++l) merged[l] = 1;
        k = j + 1;
    }
}

// Theorem 1 / Algorithm 1: going down from the top, layer l (paper numbering, l >= 2) is
// merged into l-1 when tau_b(l-2) - tau_c(l) < a.  tau_b(l-2) is the moment layer l-1 ends
// its backward pass; tau_c(l), with every layer above either sent or merged into l, is the
// later of the channel becoming free and layer l's gradients being ready.  Recomputing all
// tau_c after a merge (the listing's CalculateCommStart) changes only that one value, so
// one downward sweep suffices.
void plan_paper_greedy(const mgwfbp_plan_t &pl, std::vector<uint8_t> &merged)
{
    const int32_t L = pl.L;
    merged.assign(L, 0);
    double channel_free = 0.0;  // tau_c + t_c of the last message sent
    uint64_t pending = 0;
    for (int32_t l = L - 1; l >= 1; --l) {
        pending += kBytesPerParam * pl.p[l];
        const double tau_c = std::max(channel_free, pl.mu_b[l]);
        if (pl.mu_b[l - 1] - tau_c < pl.a) {
            merged[l] = 1;
        } else {
            channel_free = tau_c + t_ar(pl, pending);
            pending = 0;
        }
    }
}

// Fill in everything derived from `merged`: groups, offsets, predicted times.
void finish_plan(mgwfbp_plan_t &pl)
{
    const int32_t L = pl.L;
    pl.group_of_layer.assign(L, 0);
    pl.off_in_group.assign(L, 0);
    pl.groups.clear();
    GroupInfo cur;
    uint64_t plan_off = 0;
    for (int32_t l = L - 1; l >= 0; --l) {
        pl.group_of_layer[l] = static_cast<int32_t>(pl.groups.size());
        pl.off_in_group[l] = cur.elems;
        cur.layers.push_back(l);
        cur.elems += pl.p[l];
        // optional: every layer starts on a multiple of pad_elems in the merged order
        if (pl.opt.pad_elems > 1)
            cur.elems = (cur.elems + pl.opt.pad_elems - 1) / pl.opt.pad_elems * pl.opt.pad_elems;
        if (!pl.merged[l]) {
            cur.plan_off = plan_off;
            plan_off += cur.elems;
            pl.groups.push_back(cur);
            cur = GroupInfo();
        }
    }
    pl.total_elems = plan_off;
    std::vector<double> gs, gf;
    pl.t_iter = simulate(pl, pl.merged, &gs, &gf);
    for (size_t k = 0; k < pl.groups.size(); ++k) {
        pl.groups[k].start_ms = gs[k];
        pl.groups[k].finish_ms = gf[k];
    }
    std::vector<uint8_t> none(L, 0);
    pl.t_iter_wfbp = simulate(pl, none, nullptr, nullptr);
}

}  // namespace mgwfbp
