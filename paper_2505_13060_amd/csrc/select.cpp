// Host side of libampsens: the epilogue of Sec. 2.2 (mean sensitivity, loss MSE per layer and
// per group) and the exact solution of the selection problem eq. (ip) of Sec. 2.1, a
// multiple-choice knapsack: one format combination per sequential sub-graph, maximum total
// gain, total loss MSE within the budget.
//
// Solver: groups are first reduced to their non-dominated choices; the search then walks the
// groups in order keeping a list of partial configurations (total mse, total gain) from which
// it drops (i) every partial that another one dominates and (ii) every partial whose upper
// bound -- its gain plus the LP relaxation of the remaining groups under the remaining
// budget, evaluated on the groups' upper convex hulls -- cannot reach the best complete
// configuration found so far.  The best complete configuration known is kept tight by completing
// every kept partial greedily along the hulls (the LP walk without its fractional last edge), so
// the gap between bound and incumbent is one hull edge and few partials survive.  Both rules keep
// at least one optimal configuration, so the result is exact.
#include "../../include/ampsens.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

namespace {

struct Choice {
    double d, g;
    int32_t idx;
};

struct Segment {            // one edge of a group's upper convex hull
    double dd, dg;          // increments, dd > 0, dg > 0
};

// LP relaxation of the groups not yet decided, as a concave piecewise-linear function of the
// budget: start from every such group's cheapest choice, then take hull edges in order of
// decreasing slope.  All hull edges are sorted by slope once; a segment tree over that order holds
// the increments of the edges whose group is still undecided, so that "walk the edges until the
// budget is used up" is one descent of the tree and dropping an edge is one leaf-to-root update.
// Inner nodes are always recomputed from their children, so removed edges leave no rounding residue.
struct Relaxation {
    std::vector<Segment> edges;          // sorted by decreasing slope
    std::vector<int32_t> group;          // owner of each edge
    std::vector<double> td, tg;          // segment tree over dd and dg of live edges: node p has children
                                         // 2p and 2p + 1, leaf of edge i is leaves + i
    size_t leaves = 1;                   // a power of two >= edges.size()
    double base_d = 0, base_g = 0;       // cheapest choices of the undecided groups

    void build() {
        const size_t n = edges.size();
        leaves = 1;
        while (leaves < n) leaves *= 2;
        td.assign(2 * leaves, 0.0);
        tg.assign(2 * leaves, 0.0);
        for (size_t i = 0; i < n; ++i)
            if (live[i]) { td[leaves + i] = edges[i].dd; tg[leaves + i] = edges[i].dg; }
        for (size_t p = leaves - 1; p >= 1; --p) { td[p] = td[2 * p] + td[2 * p + 1]; tg[p] = tg[2 * p] + tg[2 * p + 1]; }
    }
    void remove(size_t i) {
        live[i] = 0;
        size_t p = leaves + i;
        td[p] = 0.0;
        tg[p] = 0.0;
        for (p >>= 1; p >= 1; p >>= 1) { td[p] = td[2 * p] + td[2 * p + 1]; tg[p] = tg[2 * p] + tg[2 * p + 1]; }
    }
    // Greedy walk over the live edges, in order, while they fit into `room` (>= 0): the longest
    // prefix whose increments fit.  Returns the gain of the whole edges taken; *frac receives the
    // gain of the fraction of the next live edge that still fits.
    double walk(double room, double* frac) const {
        if (frac) *frac = 0.0;
        if (edges.empty()) return 0.0;
        if (td[1] <= room) return tg[1];                       // everything fits
        size_t p = 1;
        double used = 0, g = 0;
        while (p < leaves) {
            const size_t l = 2 * p;
            if (used + td[l] <= room) { used += td[l]; g += tg[l]; p = l + 1; }   // the left half fits: go on in the right
            else p = l;
        }
        // p is the leaf of the first edge that does not fit (removed edges weigh nothing and always fit)
        if (used + td[p] <= room) { used += td[p]; g += tg[p]; }
        else if (frac) *frac = tg[p] * ((room - used) / td[p]);
        return g;
    }
    // Index of the first live edge that the greedy walk cannot take whole, edges.size() if all fit.
    size_t first_unfit(double room) const {
        if (edges.empty() || td[1] <= room) return edges.size();
        size_t p = 1;
        double used = 0;
        while (p < leaves) {
            const size_t l = 2 * p;
            if (used + td[l] <= room) { used += td[l]; p = l + 1; }
            else p = l;
        }
        return used + td[p] <= room ? edges.size() : p - leaves;
    }
    std::vector<char> live;
    // upper bound: -inf when even the cheapest choices do not fit
    double bound(double budget) const {
        const double room = budget - base_d;
        if (room < 0) return -std::numeric_limits<double>::infinity();
        double frac;
        const double g = walk(room, &frac);
        return base_g + g + frac;
    }
    // The same walk without the fractional last edge.  Edges are taken in order of decreasing slope
    // and the slopes along one group's hull decrease, so the edges taken from a group are a prefix of
    // its hull: this is the gain of a real configuration that fits.
    double integral(double budget) const {
        const double room = budget - base_d;
        if (room < 0) return -std::numeric_limits<double>::infinity();
        return base_g + walk(room, nullptr);
    }
};

struct State {
    double d, g;
    int32_t parent, pick;   // index into the previous stage's list; position in the reduced group
};

}  // namespace

extern "C" {

double amp_alpha(int mantissa_bits) { return std::ldexp(1.0, -2 * mantissa_bits) / 12.0; }

amp_status_t amp_layer_loss_mse(const float* sums, int R, const amp_fp8_format_t* fmts, int n_fmts,
                                double* s_layer, double* d_model, double* d_measured) {
    if (n_fmts < 1 || n_fmts > AMP_MAX_FORMATS) return AMP_ERR_BAD_FORMAT;
    if (!fmts) return AMP_ERR_INVALID_ARG;
    for (int f = 0; f < n_fmts; ++f)
        if (fmts[f] != AMP_FP8_E4M3 && fmts[f] != AMP_FP8_E5M2) return AMP_ERR_BAD_FORMAT;
    if (R < 1 || !sums || !s_layer) return AMP_ERR_INVALID_ARG;
    double s = 0.0;
    for (int r = 0; r < R; ++r) {
        const float* p = sums + (size_t)r * n_fmts * 4;       // A is repeated per format; use f = 0
        s += (double)p[1] + (double)p[3];
    }
    s /= (double)R;
    *s_layer = s;
    for (int f = 0; f < n_fmts; ++f) {
        if (d_model) d_model[f] = s * amp_alpha(fmts[f] == AMP_FP8_E4M3 ? 3 : 2);
        if (d_measured) {
            double e = 0.0;
            for (int r = 0; r < R; ++r) {
                const float* p = sums + ((size_t)r * n_fmts + f) * 4;
                e += (double)p[0] + (double)p[2];
            }
            d_measured[f] = e / (double)R;
        }
    }
    return AMP_OK;
}

double amp_loss_second_moment(const double* losses, int n) {
    if (n < 1 || !losses) return std::numeric_limits<double>::quiet_NaN();
    double s = 0.0;
    for (int r = 0; r < n; ++r) s += losses[r] * losses[r];
    return s / (double)n;
}

double amp_mse_budget(double tau, double mean_g2) { return tau * tau * mean_g2; }

amp_status_t amp_group_tables(int n_layers, int F, const double* layer_mse, const double* layer_gain,
                              double* d, double* c) {
    if (n_layers < 0 || F < 1 || !d || !c) return AMP_ERR_INVALID_ARG;
    if (n_layers > 0 && (!layer_mse || !layer_gain)) return AMP_ERR_INVALID_ARG;
    int64_t ncol = 1;
    for (int l = 0; l < n_layers; ++l) {
        ncol *= F;
        if (ncol > ((int64_t)1 << 24)) return AMP_ERR_TOO_LARGE;
    }
    for (int64_t p = 0; p < ncol; ++p) {
        int64_t q = p;
        double dm = 0.0, cg = 0.0;
        for (int l = 0; l < n_layers; ++l) {
            const int f = (int)(q % F);
            q /= F;
            dm += layer_mse[(size_t)l * F + f];
            cg += layer_gain[(size_t)l * F + f];
        }
        d[p] = dm;
        c[p] = cg;
    }
    return AMP_OK;
}

amp_status_t amp_select_subgraphs(int J, const int32_t* n_choices, const double* gain,
                                  const double* mse, double mse_budget, int32_t* choice,
                                  double* total_gain, double* total_mse) {
    if (J < 0) return AMP_ERR_INVALID_ARG;
    if (J > 0 && (!n_choices || !gain || !mse || !choice)) return AMP_ERR_INVALID_ARG;
    if (std::isnan(mse_budget)) return AMP_ERR_INVALID_ARG;
    size_t total = 0;
    for (int j = 0; j < J; ++j) {
        if (n_choices[j] < 1) return AMP_ERR_INVALID_ARG;
        total += (size_t)n_choices[j];
    }
    for (size_t i = 0; i < total; ++i)
        if (!std::isfinite(gain[i]) || !std::isfinite(mse[i]) || mse[i] < 0) return AMP_ERR_INVALID_ARG;

    // 1. Non-dominated choices of every group, by increasing mse (and then increasing gain).
    std::vector<std::vector<Choice>> groups(J);
    size_t off = 0;
    for (int j = 0; j < J; ++j) {
        std::vector<Choice> all(n_choices[j]);
        for (int32_t p = 0; p < n_choices[j]; ++p) all[p] = Choice{mse[off + p], gain[off + p], p};
        std::sort(all.begin(), all.end(), [](const Choice& a, const Choice& b) {
            if (a.d != b.d) return a.d < b.d;
            if (a.g != b.g) return a.g > b.g;
            return a.idx < b.idx;
        });
        double best = -std::numeric_limits<double>::infinity();
        for (const Choice& ch : all)
            if (ch.g > best) { groups[j].push_back(ch); best = ch.g; }
        off += (size_t)n_choices[j];
    }

    // 2. LP relaxation over all groups; groups leave it as the search decides them.
    Relaxation rest;
    {
        struct Tagged { Segment s; int32_t j; int32_t k; };
        std::vector<Tagged> all;
        for (int j = 0; j < J; ++j) {
            // upper convex hull of the (d, g) points, which are sorted by d with increasing g
            std::vector<Choice> h;
            for (const Choice& ch : groups[j]) {
                while (h.size() >= 2) {
                    const Choice& a = h[h.size() - 2];
                    const Choice& b = h[h.size() - 1];
                    // drop b when it lies on or below the chord a -> ch
                    if ((b.g - a.g) * (ch.d - a.d) <= (ch.g - a.g) * (b.d - a.d)) h.pop_back();
                    else break;
                }
                h.push_back(ch);
            }
            for (size_t k = 1; k < h.size(); ++k)
                all.push_back(Tagged{Segment{h[k].d - h[k - 1].d, h[k].g - h[k - 1].g}, j, (int32_t)k});
            rest.base_d += groups[j].front().d;
            rest.base_g += groups[j].front().g;
        }
        // decreasing slope; among equal slopes a group's edges keep their hull order
        std::stable_sort(all.begin(), all.end(), [](const Tagged& a, const Tagged& b) {
            const double l = a.s.dg * b.s.dd, r = b.s.dg * a.s.dd;
            if (l != r) return l > r;
            if (a.j != b.j) return a.j < b.j;
            return a.k < b.k;
        });
        for (const Tagged& t : all) { rest.edges.push_back(t.s); rest.group.push_back(t.j); }
        rest.live.assign(rest.edges.size(), 1);
        rest.build();
    }
    std::vector<std::vector<size_t>> edges_of(J);
    for (size_t i = 0; i < rest.group.size(); ++i) edges_of[rest.group[i]].push_back(i);
    // Order in which the search decides the groups (any order is exact).  The LP optimum takes all hull
    // edges steeper than the slope of the edge at which the budget runs out; a group whose edges are all
    // far from that slope has one choice that survives the bound, a group with an edge near it has
    // several.  Deciding the clear-cut groups first keeps the list of partial configurations short
    // until the last stages.
    std::vector<int32_t> order(J);
    for (int j = 0; j < J; ++j) order[j] = j;
    {
        double base = 0.0;
        for (int j = 0; j < J; ++j) base += groups[j].front().d;
        rest.base_d = base;
        const size_t brk = mse_budget >= base ? rest.first_unfit(mse_budget - base) : rest.edges.size();
        if (brk < rest.edges.size()) {
            const double lam = std::log(rest.edges[brk].dg / rest.edges[brk].dd);
            std::vector<double> clear(J, std::numeric_limits<double>::infinity());
            for (int j = 0; j < J; ++j)
                for (size_t i : edges_of[j]) {
                    const double dist = std::fabs(std::log(rest.edges[i].dg / rest.edges[i].dd) - lam);
                    if (dist < clear[j]) clear[j] = dist;
                }
            std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return clear[a] > clear[b]; });
        }
    }
    // cheapest choices of the groups decided at stages t..J-1
    std::vector<double> suffix_d(J + 1, 0.0), suffix_g(J + 1, 0.0);
    for (int t = J - 1; t >= 0; --t) {
        suffix_d[t] = suffix_d[t + 1] + groups[order[t]].front().d;
        suffix_g[t] = suffix_g[t + 1] + groups[order[t]].front().g;
    }
    rest.base_d = suffix_d[0];
    rest.base_g = suffix_g[0];
    if (J == 0) {
        if (mse_budget < 0) return AMP_ERR_INFEASIBLE;
        if (total_gain) *total_gain = 0.0;
        if (total_mse) *total_mse = 0.0;
        return AMP_OK;
    }
    if (rest.base_d > mse_budget) return AMP_ERR_INFEASIBLE;

    // 3. Stage-wise search with dominance and bound pruning.
    const double ninf = -std::numeric_limits<double>::infinity();
    double incumbent = rest.integral(mse_budget);   // greedy configuration along the hulls: fits
    auto slack = [](double v) { return 1e-12 * (std::fabs(v) + 1.0); };
    std::vector<std::vector<State>> stages(J + 1);
    stages[0].push_back(State{0.0, 0.0, -1, -1});
    std::vector<State> cand;
    for (int t = 0; t < J; ++t) {
        const int j = order[t];
        cand.clear();
        // group j is decided in this stage: take it out of the relaxation
        for (size_t i : edges_of[j]) rest.remove(i);
        rest.base_d = suffix_d[t + 1];
        rest.base_g = suffix_g[t + 1];
        for (int32_t s = 0; s < (int32_t)stages[t].size(); ++s) {
            const State& st = stages[t][s];
            for (int32_t p = 0; p < (int32_t)groups[j].size(); ++p) {
                const double d = st.d + groups[j][p].d;
                if (d + rest.base_d > mse_budget) break;         // choices are sorted by mse
                const double g = st.g + groups[j][p].g;
                cand.push_back(State{d, g, s, p});
            }
        }
        std::sort(cand.begin(), cand.end(), [](const State& a, const State& b) {
            if (a.d != b.d) return a.d < b.d;
            if (a.g != b.g) return a.g > b.g;
            if (a.parent != b.parent) return a.parent < b.parent;
            return a.pick < b.pick;
        });
        double best = ninf;
        std::vector<State>& next = stages[t + 1];
        for (const State& c : cand) {
            if (!(c.g > best)) continue;                          // dominated
            best = c.g;
            const double room = mse_budget - c.d;
            const double ub = c.g + rest.bound(room);
            if (ub < incumbent - slack(incumbent)) continue;      // cannot reach the incumbent
            const double lb = c.g + rest.integral(room);          // a configuration that completes c
            if (lb > incumbent) incumbent = lb;
            next.push_back(c);
        }
        if (next.empty()) return AMP_ERR_INFEASIBLE;              // cannot happen once base fits
    }

    // 4. Best final state: largest gain, then smallest mse (list is sorted by mse, gains increase).
    const std::vector<State>& last = stages[J];
    int32_t bi = 0;
    for (int32_t s = 1; s < (int32_t)last.size(); ++s)
        if (last[s].g > last[bi].g) bi = s;
    if (total_gain) *total_gain = last[bi].g;
    if (total_mse) *total_mse = last[bi].d;
    int32_t s = bi;
    for (int t = J; t >= 1; --t) {
        choice[order[t - 1]] = groups[order[t - 1]][stages[t][s].pick].idx;
        s = stages[t][s].parent;
    }
    return AMP_OK;
}

}  // extern "C"
