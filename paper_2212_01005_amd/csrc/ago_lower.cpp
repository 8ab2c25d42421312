// From a partitioned operator graph to launches, host only (AGO Sec. III-B and VI name the structures that
// intensive fusion covers: pw -> dw -> pw, the pw / dw pairs, a general convolution under a general convolution,
// matmul -> simple operators -> matmul; Sec. III: sibling operators that share an input belong to one subgraph).
// Inside every subgraph of the partition the operator chains that the fused kernels of this library implement
// are recognised and become one launch each; every other operator is a launch of its own.
//
// A chain starts at the first operator (in topological order) not yet placed and follows single-consumer links
// inside the subgraph; an "add" may take its second operand from outside the chain (a residual), a batched
// product its second operand from anything computed earlier.  The chain's operator kinds are matched, from its
// first operator, against the structures below in order; a structure is taken only if the checks that the kinds
// cannot express hold as well (the residual is the block's own input, strides, dtypes, sizes the kernels have).
#include "ago_host.hpp"

#include <algorithm>
#include <vector>

namespace ago {
namespace {

// one element of a structure: the operator kinds it accepts (bit set over ago_graph_op) and whether it may be absent
struct Elem { unsigned kinds; bool optional; };
constexpr unsigned bit(int op) { return 1u << op; }

struct Structure { int kind; int n; Elem e[9]; };

constexpr Elem one(int op) { return Elem{bit(op), false}; }
constexpr Elem opt(int op) { return Elem{bit(op), true}; }

// longest first
constexpr Structure kStructures[] = {
    {AGO_LAUNCH_INVRES, 9, {one(AGO_GOP_CONV1X1), opt(AGO_GOP_BIAS), one(AGO_GOP_RELU6), one(AGO_GOP_DWCONV), opt(AGO_GOP_BIAS),
                            one(AGO_GOP_RELU6), one(AGO_GOP_CONV1X1), opt(AGO_GOP_BIAS), opt(AGO_GOP_ADD)}},
    {AGO_LAUNCH_CONV_CHAIN, 7, {one(AGO_GOP_CONV3X3), opt(AGO_GOP_BIAS), one(AGO_GOP_RELU), one(AGO_GOP_CONV3X3), opt(AGO_GOP_BIAS),
                                opt(AGO_GOP_ADD), one(AGO_GOP_RELU)}},
    {AGO_LAUNCH_FFN, 5, {one(AGO_GOP_GEMM), opt(AGO_GOP_BIAS),
                         Elem{bit(AGO_GOP_GELU_TANH) | bit(AGO_GOP_RELU) | bit(AGO_GOP_RELU6), false}, one(AGO_GOP_GEMM),
                         opt(AGO_GOP_BIAS)}},
    {AGO_LAUNCH_ATTN, 4, {one(AGO_GOP_BMM_NT), one(AGO_GOP_SCALE), one(AGO_GOP_SOFTMAX), one(AGO_GOP_BMM_NN)}},
    {AGO_LAUNCH_PW_DW, 6, {one(AGO_GOP_CONV1X1), opt(AGO_GOP_BIAS), one(AGO_GOP_RELU6), one(AGO_GOP_DWCONV), opt(AGO_GOP_BIAS),
                           one(AGO_GOP_RELU6)}},
    {AGO_LAUNCH_DW_PW, 5, {one(AGO_GOP_DWCONV), opt(AGO_GOP_BIAS), one(AGO_GOP_RELU6), one(AGO_GOP_CONV1X1), opt(AGO_GOP_BIAS)}},
};

// Length of the prefix of ops[0 .. len) that the structure covers, 0 when it does not match.  An optional element
// never accepts the kind of the element after it, so taking it whenever it fits is the only parse.
int match(const Structure& s, const int* ops, int len) {
    int pos = 0;
    for (int k = 0; k < s.n; ++k) {
        const bool fits = pos < len && (s.e[k].kinds & bit(ops[pos]));
        if (fits) ++pos;
        else if (!s.e[k].optional) return 0;
    }
    return pos;
}

struct GraphView {
    int n;
    const int* op;
    const int* in_begin;
    const int* in_ids;
    const int* attr;        // [n][4]
    const float* attr_f;    // [n]
    const int* sub;
    std::vector<std::vector<int>> cons;
    int n_in(int v) const { return in_begin[v + 1] - in_begin[v]; }
    int in(int v, int k) const { return in_ids[in_begin[v] + k]; }
};

bool contains(const std::vector<int>& ids, int len, int v) { return std::find(ids.begin(), ids.begin() + len, v) != ids.begin() + len; }

// the checks behind a structure match, on the first `len` nodes of the chain
bool admissible(const GraphView& g, int kind, const std::vector<int>& ids, int len, ago_dtype dt) {
    const int first_in = g.n_in(ids[0]) > 0 ? g.in(ids[0], 0) : -1;
    bool has_add = false;
    for (int k = 0; k < len; ++k) {
        const int v = ids[k];
        if (g.op[v] != AGO_GOP_ADD) continue;
        has_add = true;
        int outside = 0, other = -1;
        for (int q = 0; q < g.n_in(v); ++q)
            if (!contains(ids, len, g.in(v, q))) { ++outside; other = g.in(v, q); }
        if (outside != 1 || other != first_in) return false;        // the fused residual is the block's own input
    }
    switch (kind) {
        case AGO_LAUNCH_INVRES: {
            if (!has_add) return true;
            for (int k = 0; k < len; ++k)
                if (g.op[ids[k]] == AGO_GOP_DWCONV) return g.attr[4 * ids[k]] == 1;     // a residual needs stride 1
            return false;
        }
        case AGO_LAUNCH_CONV_CHAIN: return dt == AGO_BF16 && g.attr[4 * ids[0]] == 64;
        case AGO_LAUNCH_FFN: return dt == AGO_BF16;
        case AGO_LAUNCH_ATTN: {
            // the kernel computes softmax(alpha in0 in1^T) v: the probabilities must be the first operand of the
            // second product, alpha positive, the head dimension one the kernel has
            const int t = ids[0], sc = ids[1], sm = ids[2], nn = ids[3];
            const int head_dim = g.attr[4 * t];
            return dt == AGO_BF16 && g.n_in(nn) > 0 && g.in(nn, 0) == sm && g.n_in(sm) > 0 && g.in(sm, 0) == sc &&
                   g.n_in(sc) > 0 && g.in(sc, 0) == t && g.attr_f[sc] > 0.0f && (head_dim == 64 || head_dim == 128);
        }
        default: return true;
    }
}

// Sibling fusion: node i is a product whose input feeds exactly three products of one subgraph with equal weight
// shapes, each followed (or not, all alike) by a bias and then a "to_heads" view.  Fills `out` with the node ids in
// increasing order and returns true, else false.
bool qkv_siblings(const GraphView& g, const std::vector<char>& done, int i, ago_dtype dt, std::vector<int>& out) {
    if (g.op[i] != AGO_GOP_GEMM || dt != AGO_BF16 || g.n_in(i) < 1) return false;
    const int src = g.in(i, 0);
    std::vector<int> sibs;
    for (int j : g.cons[src])
        if (g.op[j] == AGO_GOP_GEMM && !done[j] && g.sub[j] == g.sub[i]) sibs.push_back(j);
    if (sibs.size() != 3 || sibs[0] != i || g.cons[src].size() != 3) return false;
    std::vector<int> chains[3];
    for (int c = 0; c < 3; ++c) {
        chains[c].push_back(sibs[c]);
        for (;;) {
            const int last = chains[c].back();
            if (g.cons[last].size() != 1) break;
            const int nx = g.cons[last][0];
            if ((g.op[nx] != AGO_GOP_BIAS && g.op[nx] != AGO_GOP_TO_HEADS) || g.sub[nx] != g.sub[i]) break;
            chains[c].push_back(nx);
            if (g.op[nx] == AGO_GOP_TO_HEADS) break;
        }
    }
    auto shape_of = [&](const std::vector<int>& c) {        // 2: product, view; 3: product, bias, view; 0: neither
        if (c.size() == 2 && g.op[c[1]] == AGO_GOP_TO_HEADS) return 2;
        if (c.size() == 3 && g.op[c[1]] == AGO_GOP_BIAS && g.op[c[2]] == AGO_GOP_TO_HEADS) return 3;
        return 0;
    };
    const int s0 = shape_of(chains[0]);
    if (s0 == 0 || shape_of(chains[1]) != s0 || shape_of(chains[2]) != s0) return false;
    for (int c = 1; c < 3; ++c) {
        const int a = chains[0][0], b = chains[c][0], ha = chains[0].back(), hb = chains[c].back();
        if (g.attr[4 * a] != g.attr[4 * b] || g.attr[4 * a + 1] != g.attr[4 * b + 1]) return false;        // weight shapes
        if (g.attr[4 * ha] != g.attr[4 * hb] || (g.attr[4 * ha + 1] != 0) != (g.attr[4 * hb + 1] != 0)) return false;
    }
    out.clear();
    for (int c = 0; c < 3; ++c) out.insert(out.end(), chains[c].begin(), chains[c].end());
    std::sort(out.begin(), out.end());
    return true;
}

}  // namespace
}  // namespace ago

extern "C" ago_status ago_graph_lower(int n_nodes, const int* op, const int* input_begin, const int* input_ids,
                                      const int* attr, const float* attr_f, const int* subgraph_of, ago_dtype dt,
                                      int decide_ffn, int* launch_kind, int* launch_begin, int* launch_nodes,
                                      int* n_launches) {
    using namespace ago;
    if (!op || !input_begin || !attr || !attr_f || !subgraph_of || !launch_kind || !launch_begin || !launch_nodes || !n_launches)
        return AGO_ERR_NULL;
    if (n_nodes <= 0 || input_begin[0] != 0) return AGO_ERR_SHAPE;
    if (dt != AGO_F32 && dt != AGO_BF16) return AGO_ERR_DTYPE;
    for (int v = 0; v < n_nodes; ++v) {
        if (op[v] < 0 || op[v] >= AGO_GOP_COUNT || input_begin[v + 1] < input_begin[v]) return AGO_ERR_SHAPE;
        if (input_begin[v + 1] > input_begin[v] && !input_ids) return AGO_ERR_NULL;
        for (int q = input_begin[v]; q < input_begin[v + 1]; ++q)
            if (input_ids[q] < 0 || input_ids[q] >= v) return AGO_ERR_SHAPE;        // topological order: producers first
    }
    GraphView g{n_nodes, op, input_begin, input_ids, attr, attr_f, subgraph_of, {}};
    g.cons.assign(n_nodes, {});
    for (int v = 0; v < n_nodes; ++v)
        for (int q = 0; q < g.n_in(v); ++q) g.cons[g.in(v, q)].push_back(v);

    std::vector<char> done(n_nodes, 0);
    std::vector<int> chain, ops, sib;
    int nl = 0, pos = 0;
    auto emit = [&](int kind, const std::vector<int>& ids, int len) {
        launch_kind[nl] = kind;
        launch_begin[nl] = pos;
        for (int k = 0; k < len; ++k) { launch_nodes[pos++] = ids[k]; done[ids[k]] = 1; }
        ++nl;
    };
    for (int i = 0; i < n_nodes; ++i) {
        if (done[i]) continue;
        if (op[i] == AGO_GOP_INPUT) { done[i] = 1; continue; }
        if (qkv_siblings(g, done, i, dt, sib)) { emit(AGO_LAUNCH_QKV, sib, (int)sib.size()); continue; }
        chain.assign(1, i);
        for (;;) {
            const int last = chain.back();
            if (g.cons[last].size() != 1) break;
            const int j = g.cons[last][0];
            if (done[j] || subgraph_of[j] != subgraph_of[i] || op[j] == AGO_GOP_INPUT) break;
            // operands of j other than the link itself
            int n_other = 0;
            bool later_outsider = false;        // an operand that is computed after the chain's start and is not on the chain
            for (int q = 0; q < g.n_in(j); ++q) {
                const int s = g.in(j, q);
                if (s == last) continue;
                ++n_other;
                if (s >= chain[0] && !contains(chain, (int)chain.size(), s)) later_outsider = true;
            }
            if (op[j] == AGO_GOP_ADD) { if (n_other != 1 || later_outsider) break; }
            else if (op[j] == AGO_GOP_BMM_NT || op[j] == AGO_GOP_BMM_NN) { if (later_outsider) break; }
            else if (n_other != 0) break;
            chain.push_back(j);
        }
        ops.resize(chain.size());
        for (size_t k = 0; k < chain.size(); ++k) ops[k] = op[chain[k]];
        int kind = AGO_LAUNCH_OP, len = 1;
        for (const Structure& s : kStructures) {
            int m = match(s, ops.data(), (int)ops.size());
            if (m > 0 && !admissible(g, s.kind, chain, m, dt)) {
                // the same structure without the residual: match what precedes the first "add"
                int first_add = -1;
                for (int k = 0; k < m; ++k)
                    if (ops[k] == AGO_GOP_ADD) { first_add = k; break; }
                m = first_add >= 0 ? match(s, ops.data(), first_add) : 0;
                if (m > 0 && !admissible(g, s.kind, chain, m, dt)) m = 0;
            }
            if (m > 0) { kind = s.kind; len = m; break; }
        }
        if (kind == AGO_LAUNCH_FFN && decide_ffn) {
            // M rows of the chain's input, K x F and F x K2 weights: the fused kernel only where it is expected to win
            int gemms[2] = {-1, -1}, ng = 0;
            for (int k = 0; k < len && ng < 2; ++k)
                if (op[chain[k]] == AGO_GOP_GEMM) gemms[ng++] = chain[k];
            const int M = attr[4 * gemms[0] + 2], K = attr[4 * gemms[0]], F = attr[4 * gemms[0] + 1], K2 = attr[4 * gemms[1] + 1];
            if (ago_fused_ffn_pays(M, K, F, K2) != 1) kind = AGO_LAUNCH_FFN_EPILOGUE;
        }
        emit(kind, chain, len);
    }
    launch_begin[nl] = pos;
    *n_launches = nl;
    return AGO_OK;
}
