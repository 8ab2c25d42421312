// Graph frontend, host only (AGO Sec. IV and V): operator weights (Eq. 1), topological stages, affix
// sets and the greedy acyclic partition (function Cluster of the "Graph Partition" algorithm), plus the
// Split / Join steps of the reformer layer.  It decides which operators form one subgraph; the fused
// kernels of this library are what such a subgraph runs as.
//
// Representation: the contracted graph is kept as successor / predecessor sets per live hyper node
// (std::set<int>, ids = smallest original id inside).  After every merge the stages are recomputed in
// one Kahn pass over the contracted graph (longest path from a root, roots at 1).
#include "ago_host.hpp"

#include <cmath>
#include <limits>
#include <set>
#include <vector>

namespace ago {
namespace {

struct Contracted {
    int n;
    std::vector<char> alive;
    std::vector<std::set<int>> succ, pred;
    std::vector<double> w;
    std::vector<int> ncomplex;
    std::vector<int> owner;        // original node -> live hyper node
    std::vector<int> stage;

    Contracted(int n_, const double* weight, const unsigned char* is_complex, int n_edges, const int* src,
               const int* dst)
        : n(n_), alive(n_, 1), succ(n_), pred(n_), w(weight, weight + n_), ncomplex(n_, 0), owner(n_), stage(n_, 0) {
        for (int v = 0; v < n; ++v) {
            owner[v] = v;
            if (is_complex) ncomplex[v] = is_complex[v] ? 1 : 0;
        }
        for (int e = 0; e < n_edges; ++e)
            if (src[e] != dst[e]) { succ[src[e]].insert(dst[e]); pred[dst[e]].insert(src[e]); }
    }

    // Longest-path stages by peeling nodes whose predecessors are all done.  Returns false on a cycle.
    bool restage() {
        std::vector<int> missing(n, 0), ready;
        int live = 0;
        for (int v = 0; v < n; ++v) {
            if (!alive[v]) continue;
            ++live;
            missing[v] = (int)pred[v].size();
            stage[v] = 1;
            if (missing[v] == 0) ready.push_back(v);
        }
        int done = 0;
        while (!ready.empty()) {
            const int v = ready.back();
            ready.pop_back();
            ++done;
            for (int s : succ[v]) {
                if (stage[s] < stage[v] + 1) stage[s] = stage[v] + 1;
                if (--missing[s] == 0) ready.push_back(s);
            }
        }
        return done == live;
    }

    // u is absorbed into v's hyper node (or the other way round): the survivor carries the smaller id
    int merge(int u, int v) {
        const int keep = u < v ? u : v, gone = u < v ? v : u;
        for (int s : succ[gone]) { pred[s].erase(gone); if (s != keep) { pred[s].insert(keep); succ[keep].insert(s); } }
        for (int q : pred[gone]) { succ[q].erase(gone); if (q != keep) { succ[q].insert(keep); pred[keep].insert(q); } }
        succ[keep].erase(gone); pred[keep].erase(gone);
        succ[keep].erase(keep); pred[keep].erase(keep);
        succ[gone].clear(); pred[gone].clear();
        w[keep] += w[gone];
        ncomplex[keep] += ncomplex[gone];
        alive[gone] = 0;
        for (int x = 0; x < n; ++x)
            if (owner[x] == gone) owner[x] = keep;
        return keep;
    }
};

// Function Cluster.  part[v] = subgraph of original node v, subgraphs numbered by smallest member.
// Returns the number of subgraphs, or -1 when the edges contain a cycle.
int cluster_impl(int n, const double* weight, const unsigned char* is_complex, int n_edges, const int* src,
                 const int* dst, double td, int max_complex, int* part) {
    Contracted g(n, weight, is_complex, n_edges, src, dst);
    if (!g.restage()) return -1;
    std::vector<char> cand(n, 1);
    for (;;) {
        // the heaviest candidate (lowest id on ties)
        int v = -1;
        for (int x = 0; x < n; ++x)
            if (g.alive[x] && cand[x] && (v < 0 || g.w[x] > g.w[v])) v = x;
        if (v < 0) break;
        // the lightest affix node (a neighbour one stage away) that keeps the pair under the threshold
        int u = -1;
        auto consider = [&](int x) {
            const int ds = g.stage[x] - g.stage[v];
            if (ds != 1 && ds != -1) return;
            if (!(g.w[v] + g.w[x] < td)) return;
            if (max_complex > 0 && g.ncomplex[v] + g.ncomplex[x] > max_complex) return;
            if (u < 0 || g.w[x] < g.w[u] || (g.w[x] == g.w[u] && x < u)) u = x;
        };
        for (int x : g.succ[v]) consider(x);
        for (int x : g.pred[v]) consider(x);
        if (u < 0) { cand[v] = 0; continue; }
        cand[u] = cand[v] = 0;
        const int keep = g.merge(u, v);
        cand[keep] = 1;
        if (!g.restage()) return -1;     // cannot happen for stage-adjacent pairs (theorem of Sec. IV-B)
    }
    std::vector<int> id_of(n, -1);
    int count = 0;
    for (int x = 0; x < n; ++x)
        if (g.alive[x]) id_of[x] = count++;
    for (int x = 0; x < n; ++x) part[x] = id_of[g.owner[x]];
    return count;
}

bool edges_ok(int n, int n_edges, const int* src, const int* dst) {
    for (int e = 0; e < n_edges; ++e)
        if (src[e] < 0 || src[e] >= n || dst[e] < 0 || dst[e] >= n || src[e] == dst[e]) return false;
    return true;
}

}  // namespace
}  // namespace ago

extern "C" {

double ago_graph_op_weight(const int* loop_extents, int n_loops, double c, double b) {
    if (n_loops <= 0 || !loop_extents) return b;
    double prod = 1.0;
    for (int l = 0; l < n_loops; ++l) {
        if (loop_extents[l] < 1) return std::numeric_limits<double>::quiet_NaN();
        prod *= std::log((double)loop_extents[l]);
    }
    return c * prod + b;
}

ago_status ago_graph_topological_stage(int n_nodes, int n_edges, const int* edge_src, const int* edge_dst,
                                       int* stage) {
    if (!stage || (n_edges > 0 && (!edge_src || !edge_dst))) return AGO_ERR_NULL;
    if (n_nodes <= 0 || n_edges < 0 || !ago::edges_ok(n_nodes, n_edges, edge_src, edge_dst)) return AGO_ERR_SHAPE;
    std::vector<double> w(n_nodes, 0.0);
    ago::Contracted g(n_nodes, w.data(), nullptr, n_edges, edge_src, edge_dst);
    if (!g.restage()) return AGO_ERR_SHAPE;
    for (int v = 0; v < n_nodes; ++v) stage[v] = g.stage[v];
    return AGO_OK;
}

ago_status ago_graph_cluster(int n_nodes, const double* weight, const unsigned char* is_complex,
                             int n_edges, const int* edge_src, const int* edge_dst, double td,
                             int max_complex, int* subgraph_of, int* n_subgraphs) {
    if (!weight || !subgraph_of || (n_edges > 0 && (!edge_src || !edge_dst))) return AGO_ERR_NULL;
    if (n_nodes <= 0 || n_edges < 0 || !ago::edges_ok(n_nodes, n_edges, edge_src, edge_dst)) return AGO_ERR_SHAPE;
    if (max_complex > 0 && !is_complex) return AGO_ERR_NULL;
    for (int v = 0; v < n_nodes; ++v)
        if (!(weight[v] >= 0.0)) return AGO_ERR_SHAPE;         // also rejects NaN
    const int count = ago::cluster_impl(n_nodes, weight, is_complex, n_edges, edge_src, edge_dst, td, max_complex,
                                        subgraph_of);
    if (count < 0) return AGO_ERR_SHAPE;                       // the edges contain a cycle
    if (n_subgraphs) *n_subgraphs = count;
    return AGO_OK;
}

ago_status ago_graph_split(int n_nodes, const double* weight, const unsigned char* is_complex, int n_edges,
                           const int* edge_src, const int* edge_dst, const int* subgraph_of, double td_mini,
                           int* mini_of, int* parent_of_mini, int* n_minis) {
    if (!weight || !is_complex || !subgraph_of || !mini_of || !parent_of_mini) return AGO_ERR_NULL;
    if (n_edges > 0 && (!edge_src || !edge_dst)) return AGO_ERR_NULL;
    if (n_nodes <= 0 || n_edges < 0 || !ago::edges_ok(n_nodes, n_edges, edge_src, edge_dst)) return AGO_ERR_SHAPE;
    int n_sub = 0;
    for (int v = 0; v < n_nodes; ++v) {
        if (subgraph_of[v] < 0 || subgraph_of[v] >= n_nodes) return AGO_ERR_SHAPE;
        if (subgraph_of[v] + 1 > n_sub) n_sub = subgraph_of[v] + 1;
    }
    int total = 0;
    std::vector<int> local(n_nodes), ids, es, ed, part;
    std::vector<double> w;
    std::vector<unsigned char> cx;
    for (int sid = 0; sid < n_sub; ++sid) {
        ids.clear(); es.clear(); ed.clear(); w.clear(); cx.clear();
        for (int v = 0; v < n_nodes; ++v)
            if (subgraph_of[v] == sid) { local[v] = (int)ids.size(); ids.push_back(v); w.push_back(weight[v]); cx.push_back(is_complex[v]); }
        if (ids.empty()) continue;
        for (int e = 0; e < n_edges; ++e)
            if (subgraph_of[edge_src[e]] == sid && subgraph_of[edge_dst[e]] == sid) {
                es.push_back(local[edge_src[e]]); ed.push_back(local[edge_dst[e]]);
            }
        part.assign(ids.size(), 0);
        const int count = ago::cluster_impl((int)ids.size(), w.data(), cx.data(), (int)es.size(), es.data(), ed.data(),
                                            td_mini, 1, part.data());
        if (count < 0) return AGO_ERR_SHAPE;
        for (size_t i = 0; i < ids.size(); ++i) mini_of[ids[i]] = total + part[i];
        for (int m = 0; m < count; ++m) parent_of_mini[total + m] = sid;
        total += count;
    }
    if (n_minis) *n_minis = total;
    return AGO_OK;
}

ago_status ago_graph_join(int n_nodes, const int* mini_of, int n_minis, const int* parent_of_mini,
                          int* subgraph_of) {
    if (!mini_of || !parent_of_mini || !subgraph_of) return AGO_ERR_NULL;
    if (n_nodes <= 0 || n_minis <= 0) return AGO_ERR_SHAPE;
    for (int v = 0; v < n_nodes; ++v) {
        if (mini_of[v] < 0 || mini_of[v] >= n_minis) return AGO_ERR_SHAPE;
        subgraph_of[v] = parent_of_mini[mini_of[v]];
    }
    return AGO_OK;
}

}  // extern "C"
