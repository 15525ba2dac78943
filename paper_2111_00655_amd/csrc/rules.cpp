// Pattern generator (paper Sec. 3: pattern rules).  A backend may be described
// by a rule instead of a list of patterns: which operators it runs and which
// groups it fuses.  The generator visits every operator of the graph, registers
// the operator's own pattern if the backend runs it, and widens the group one
// step at a time towards the seed's next post-dominator, registering a pattern
// whenever the rule accepts the widened group.
//
// The rule is data (classes per operator kind), as in the paper's listing:
// "fusable" operators (convolutions, matrix products) may absorb the
// element-wise operators that follow them - the check that every operator
// between seed and sink is element-wise.  A group grows only along a chain: the
// current sink needs exactly one consumer, used once, and must not be a graph
// output (the group is to become one kernel with a single exit); that consumer
// is then the sink's immediate post-dominator.  The other operands of an
// absorbed operator become wildcards.  Visiting order (node order, groups
// smallest first) and "a pattern already registered for this backend is not
// registered again" fix the order of the generated registry.
#include <algorithm>

#include "core.h"

namespace clg {

namespace {

bool same_pattern(const std::vector<clg_pattern_node> &a, const std::vector<clg_pattern_node> &b) {
    if (a.size() != b.size()) return false;
    for (size_t i = 0; i < a.size(); ++i) {
        const clg_pattern_node &x = a[i], &y = b[i];
        if (x.op != y.op || x.n_args != y.n_args || x.n_constraints != y.n_constraints) return false;
        for (int k = 0; k < x.n_args; ++k)
            if (x.args[k] != y.args[k]) return false;
        for (int k = 0; k < x.n_constraints; ++k)
            if (x.constraints[k].attr != y.constraints[k].attr || x.constraints[k].lo != y.constraints[k].lo ||
                x.constraints[k].hi != y.constraints[k].hi)
                return false;
    }
    return true;
}

// Appends operator `kind` with `n_in` operands to a post-order node list: the
// operand at `chain_pos` is the current root (or a wildcard when there is none
// yet), the others are fresh wildcards.
void push_op(std::vector<clg_pattern_node> *nodes, int32_t kind, int n_in, int chain_pos) {
    const int32_t inner = nodes->empty() ? -1 : (int32_t)nodes->size() - 1;
    clg_pattern_node op{};
    op.op = kind;
    op.n_args = n_in;
    for (int k = 0; k < n_in; ++k) {
        if (k == chain_pos && inner >= 0) {
            op.args[k] = inner;
        } else {
            clg_pattern_node w{};
            w.op = CLG_WILDCARD;
            nodes->push_back(w);
            op.args[k] = (int32_t)nodes->size() - 1;
        }
    }
    nodes->push_back(op);
}

}  // namespace

int32_t generate_patterns(Context &ctx, Graph &g, int32_t backend, const clg_pattern_rule &rule, int32_t *n_added) {
    if (backend < 0 || backend >= (int32_t)ctx.backends.size()) return fail(CLG_UNKNOWN_ID, "backend id %d", backend);
    if (rule.max_ops < 1 || rule.max_ops > CLG_MAX_MATCH_NODES)
        return fail(CLG_INVALID_ARG, "max_ops must be 1..%d (got %d)", CLG_MAX_MATCH_NODES, rule.max_ops);
    for (int k = 0; k < CLG_OP_COUNT; ++k)
        if (rule.op_class[k] < CLG_RULE_NONE || rule.op_class[k] > CLG_RULE_ELEMWISE)
            return fail(CLG_INVALID_ARG, "operator kind %d has class %d", k, rule.op_class[k]);
    g.finalize();
    int32_t added = 0;
    auto emit = [&](const std::vector<clg_pattern_node> &nodes) {
        if ((int)nodes.size() > CLG_MAX_PATTERN_NODES) return;
        for (const Pattern &q : ctx.patterns)
            if (q.backend == backend && same_pattern(q.nodes, nodes)) return;
        Pattern p;
        p.backend = backend;
        p.nodes = nodes;
        if (check_pattern(ctx, &p) != CLG_OK) return;        // the backend's kernels do not run this fused kind
        ctx.patterns.push_back(std::move(p));
        ++added;
    };
    for (int32_t v : g.op_ids) {
        const Node &nd = g.nodes[v];
        const int32_t cls = rule.op_class[nd.kind];
        if (cls == CLG_RULE_NONE) continue;
        if ((int)nd.in.size() > CLG_MAX_PATTERN_ARGS) continue;
        std::vector<clg_pattern_node> nodes;
        push_op(&nodes, nd.kind, (int)nd.in.size(), -1);
        emit(nodes);
        if (cls == CLG_RULE_ELEMWISE && !rule.grow_from_elemwise) continue;
        int32_t sink = v;
        for (int size = 1; size < rule.max_ops; ++size) {
            const std::vector<int32_t> &cons = g.consumers[sink];
            if (cons.size() != 1 || g.is_output[sink]) break;
            const Node &u = g.nodes[cons[0]];
            if (rule.op_class[u.kind] != CLG_RULE_ELEMWISE || (int)u.in.size() > CLG_MAX_PATTERN_ARGS) break;
            int pos = -1, uses = 0;
            for (size_t k = 0; k < u.in.size(); ++k)
                if (u.in[k] == sink) {
                    pos = (int)k;
                    ++uses;
                }
            if (uses != 1) break;
            push_op(&nodes, u.kind, (int)u.in.size(), pos);
            emit(nodes);
            sink = cons[0];
        }
    }
    g.matched = false;                       // the registry changed: matches have to be enumerated again
    if (n_added) *n_added = added;
    return CLG_OK;
}

}  // namespace clg
