// Host side of libampsens, second part: partition of a model graph into sequential sub-graphs
// (Appendix B of the paper), the per-layer gain formulas of Sec. 2.3.2 / 2.3.3, and the two
// baseline strategies of Sec. 3.1 (Prefix, Random) that respect the same loss-MSE budget.
//
// Partition.  The paper's groups are the single-entry / single-exit regions of the computation
// DAG: walking from the start vertex, a group closes at the first vertex through which every
// path to the sink passes.  Those vertices are exactly the dominators of the sink, so this
// implementation builds the dominator tree of the DAG (immediate dominator = nearest common
// ancestor of all predecessors, taken in topological order), reads the sink's dominator chain,
// and assigns every other vertex to the interval of the chain it falls in; the closing vertex
// belongs to the group it closes.  Non-quantisable vertices are then dropped and empty groups
// removed, as in the last steps of the paper's Algorithm 2.
#include "../../include/ampsens.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

extern "C" {

amp_status_t amp_partition_sequential(int n_vertices, int n_edges, const int32_t* edge_src,
                                      const int32_t* edge_dst, const uint8_t* quantizable,
                                      int32_t* group_of, int32_t* n_groups) {
    if (n_vertices < 1 || n_edges < 0 || !group_of || !n_groups) return AMP_ERR_INVALID_ARG;
    if (n_edges > 0 && (!edge_src || !edge_dst)) return AMP_ERR_INVALID_ARG;
    const int n = n_vertices;
    std::vector<std::vector<int>> succ(n), pred(n);
    for (int e = 0; e < n_edges; ++e) {
        const int a = edge_src[e], b = edge_dst[e];
        if (a < 0 || a >= n || b < 0 || b >= n || a == b) return AMP_ERR_INVALID_ARG;
        succ[a].push_back(b);
        pred[b].push_back(a);
    }
    // single source (vertex without predecessors) and single sink, acyclic
    int start = -1, sink = -1;
    for (int v = 0; v < n; ++v) {
        if (pred[v].empty()) { if (start >= 0) return AMP_ERR_INVALID_ARG; start = v; }
        if (succ[v].empty()) { if (sink >= 0) return AMP_ERR_INVALID_ARG; sink = v; }
    }
    if (start < 0 || sink < 0) return AMP_ERR_INVALID_ARG;
    std::vector<int> indeg(n), topo;
    for (int v = 0; v < n; ++v) indeg[v] = (int)pred[v].size();
    topo.push_back(start);
    for (size_t h = 0; h < topo.size(); ++h)
        for (int w : succ[topo[h]])
            if (--indeg[w] == 0) topo.push_back(w);
    if ((int)topo.size() != n) return AMP_ERR_INVALID_ARG;          // cycle
    std::vector<int> order(n);                                       // topological index
    for (int i = 0; i < n; ++i) order[topo[i]] = i;

    // dominator tree of a DAG
    std::vector<int> idom(n, -1), depth(n, 0);
    auto nca = [&](int a, int b) {
        while (a != b) {
            if (depth[a] < depth[b]) std::swap(a, b);
            a = idom[a];
        }
        return a;
    };
    idom[start] = start;
    for (int i = 1; i < n; ++i) {
        const int v = topo[i];
        int d = pred[v][0];
        for (size_t k = 1; k < pred[v].size(); ++k) d = nca(d, pred[v][k]);
        idom[v] = d;
        depth[v] = depth[d] + 1;
    }
    // chain of vertices every start -> sink path passes through, in execution order
    std::vector<int> chain;
    for (int v = sink; v != start; v = idom[v]) chain.push_back(v);
    std::reverse(chain.begin(), chain.end());                        // excludes the start vertex
    std::vector<int> chain_pos(n, -1);
    for (size_t k = 0; k < chain.size(); ++k) chain_pos[chain[k]] = (int)k;

    // A vertex that is not on the chain belongs to the interval closed by the first chain vertex
    // that comes after it: the chain vertex following its nearest dominating chain vertex.
    std::vector<int> interval(n, -1);
    for (int i = 0; i < n; ++i) {
        const int v = topo[i];
        if (v == start) continue;
        if (chain_pos[v] >= 0) { interval[v] = chain_pos[v]; continue; }
        int d = idom[v];
        while (d != start && chain_pos[d] < 0) d = idom[d];
        interval[v] = (d == start) ? 0 : chain_pos[d] + 1;
    }
    // drop non-quantisable vertices, renumber non-empty groups
    std::vector<int> remap(chain.size(), -1);
    std::vector<char> used(chain.size(), 0);
    for (int v = 0; v < n; ++v)
        if (v != start && (!quantizable || quantizable[v])) used[interval[v]] = 1;
    int g = 0;
    for (size_t k = 0; k < chain.size(); ++k)
        if (used[k]) remap[k] = g++;
    for (int v = 0; v < n; ++v)
        group_of[v] = (v != start && (!quantizable || quantizable[v])) ? remap[interval[v]] : -1;
    *n_groups = g;
    return AMP_OK;
}

double amp_time_gain_macs(int is_bgemm, double N, double C, double K, double delta_t) {
    return is_bgemm ? N * C * C * delta_t : N * C * K * delta_t;
}

double amp_memory_gain(int is_bgemm, double C, double K, double delta_m) {
    return is_bgemm ? 0.0 : C * K * delta_m;
}

amp_status_t amp_select_ordered(int J, const int32_t* n_choices, const double* gain, const double* mse,
                                double mse_budget, const int32_t* order, int32_t* choice,
                                double* total_gain, double* total_mse) {
    if (J < 0 || (J > 0 && (!n_choices || !gain || !mse || !choice))) return AMP_ERR_INVALID_ARG;
    if (std::isnan(mse_budget)) return AMP_ERR_INVALID_ARG;
    std::vector<size_t> off(J + 1, 0);
    for (int j = 0; j < J; ++j) {
        if (n_choices[j] < 1) return AMP_ERR_INVALID_ARG;
        off[j + 1] = off[j] + (size_t)n_choices[j];
    }
    std::vector<char> seen(J, 0);
    for (int k = 0; k < J; ++k) {
        const int j = order ? order[k] : k;
        if (j < 0 || j >= J || seen[j]) return AMP_ERR_INVALID_ARG;
        seen[j] = 1;
    }
    double d = 0.0, g = 0.0;
    for (int j = 0; j < J; ++j) {
        choice[j] = 0;                                   // column 0 is the high-precision one
        d += mse[off[j]];
        g += gain[off[j]];
    }
    if (d > mse_budget) return AMP_ERR_INFEASIBLE;
    for (int k = 0; k < J; ++k) {
        const int j = order ? order[k] : k;
        int32_t best = 0;
        for (int32_t p = 1; p < n_choices[j]; ++p) {
            const double gp = gain[off[j] + p], gb = gain[off[j] + best];
            if (gp > gb || (gp == gb && mse[off[j] + p] < mse[off[j] + best])) best = p;
        }
        const double nd = d - mse[off[j]] + mse[off[j] + best];
        if (nd > mse_budget) break;                      // the first group that does not fit ends the run
        d = nd;
        g += gain[off[j] + best] - gain[off[j]];
        choice[j] = best;
    }
    if (total_gain) *total_gain = g;
    if (total_mse) *total_mse = d;
    return AMP_OK;
}

}  // extern "C"
