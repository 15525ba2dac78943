// Pattern matcher: enumerates every legal match (v_s, b_i) -> g of the
// registry on a graph (paper Sec. 3 pattern language; the matching step of
// Alg. 1: for a frontier node v_s and a registry entry b_i, the subgraph g).
//
// Readings fixed here (the paper is silent): v_s is the first node of g in the
// order (depth, node id); a match is legal only with a single exit (every
// non-sink node has all consumers inside g and is no graph output), with
// distinct nodes bound to the pattern's operators and with no wildcard bound to
// a non-sink operator of g (a wildcard is an operand from outside the kernel; a
// non-sink value of g lives only inside it); `add` operands are tried as
// written, then swapped; one match is kept per (v_s, pattern), the first found
// scanning sinks in node order; match ids rank (order of v_s, pattern id).
#include <algorithm>
#include <functional>
#include <map>

#include "core.h"

namespace clg {

namespace {

struct Matcher {
    const Graph &g;
    const Pattern &p;
    std::vector<int32_t> bound;    // graph value per pattern node
    Matcher(const Graph &g_, const Pattern &p_) : g(g_), p(p_), bound(p_.nodes.size(), -1) {}

    bool constraints_ok(const clg_pattern_node &pn, int32_t gv) const {
        for (int c = 0; c < pn.n_constraints; ++c) {
            bool ok = false;
            const int64_t v = attr_value(g, gv, pn.constraints[c].attr, &ok);
            if (!ok || v < pn.constraints[c].lo || v > pn.constraints[c].hi) return false;
        }
        return true;
    }

    // Binds pattern node `pi` to graph value `gv` in every possible way and
    // calls `next` once per way, depth first.
    void bind(int pi, int32_t gv, const std::function<void()> &next) {
        const clg_pattern_node &pn = p.nodes[pi];
        if (pn.op == CLG_WILDCARD) {
            bound[pi] = gv;
            next();
            return;
        }
        const Node &nd = g.nodes[gv];
        if (nd.kind != pn.op || (int)nd.in.size() != pn.n_args) return;
        if (!constraints_ok(pn, gv)) return;
        bound[pi] = gv;
        const int n_orders = (pn.op == CLG_OP_ADD && pn.n_args == 2) ? 2 : 1;
        for (int o = 0; o < n_orders; ++o) {
            int32_t operands[CLG_MAX_PATTERN_ARGS];
            for (int k = 0; k < pn.n_args; ++k) operands[k] = nd.in[k];
            if (o == 1) std::swap(operands[0], operands[1]);
            std::function<void(int)> arg = [&](int k) {
                if (k == pn.n_args) {
                    next();
                    return;
                }
                bind(pn.args[k], operands[k], [&, k]() { arg(k + 1); });
            };
            arg(0);
            bound[pi] = gv;
        }
    }
};

bool legal(const Graph &g, const Pattern &p, const std::vector<int32_t> &bound,
           std::vector<int32_t> *ops) {
    ops->clear();
    for (size_t i = 0; i < p.nodes.size(); ++i)
        if (p.nodes[i].op != CLG_WILDCARD) ops->push_back(bound[i]);
    std::vector<int32_t> sorted = *ops;
    std::sort(sorted.begin(), sorted.end());
    if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return false;
    const int32_t sink = ops->back();
    for (size_t i = 0; i < p.nodes.size(); ++i)
        if (p.nodes[i].op == CLG_WILDCARD && bound[i] != sink && std::binary_search(sorted.begin(), sorted.end(), bound[i]))
            return false;
    for (int32_t v : *ops) {
        if (v == sink) continue;
        if (g.is_output[v]) return false;
        for (int32_t c : g.consumers[v])
            if (!std::binary_search(sorted.begin(), sorted.end(), c)) return false;
    }
    return true;
}

}  // namespace

int32_t match_all(Context &ctx, Graph &g) {
    g.finalize();
    std::map<std::pair<int32_t, int32_t>, MatchRec> found;
    std::vector<int32_t> ops;
    for (size_t pi = 0; pi < ctx.patterns.size(); ++pi) {
        const Pattern &p = ctx.patterns[pi];
        const int root = (int)p.nodes.size() - 1;
        int n_ops = 0;
        for (auto &pn : p.nodes) n_ops += pn.op != CLG_WILDCARD;
        if (n_ops > CLG_MAX_MATCH_NODES) continue;
        for (int32_t sink : g.op_ids) {
            Matcher m(g, p);
            m.bind(root, sink, [&]() {
                if (!legal(g, p, m.bound, &ops)) return;
                int32_t first = ops[0];
                for (int32_t v : ops)
                    if (g.rank[v] < g.rank[first]) first = v;
                const auto key = std::make_pair(g.rank[first], (int32_t)pi);
                if (found.count(key)) return;
                MatchRec r;
                r.pattern = (int32_t)pi;
                r.backend = p.backend;
                r.first = first;
                r.sink = ops.back();
                r.binding = ops;
                r.nodes = ops;
                std::sort(r.nodes.begin(), r.nodes.end());
                r.wild = m.bound;
                found.emplace(key, std::move(r));
            });
        }
    }
    g.matches.clear();
    for (auto &kv : found) g.matches.push_back(std::move(kv.second));
    g.matched = true;
    return CLG_OK;
}

}  // namespace clg
