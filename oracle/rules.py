"""Oracle pattern generator: backend patterns from a pattern rule.

TEST INFRASTRUCTURE ONLY (parity anchor; never imported by the product path).

Paper Sec. 3 (pattern rules, the automatic pattern generator and its figure):
besides enumerating patterns, a backend may give a rule - which operators it
runs, and which groups of operators it fuses - and the generator visits every
operator of the computation graph, emits the operator's own pattern if the
backend runs it, then widens the group one step at a time towards the next
operator every path from the seed must pass (its post-dominator), emitting a
pattern whenever the rule accepts the widened group, until it does not.

The rule used here is the one the paper's listing sketches: operator classes
"fusable" (convolutions, matrix products) and "element-wise"; a group seeded by
a fusable operator may absorb the element-wise operators that follow it (the
check that every operator between seed and sink is element-wise).  Readings
fixed here, the paper being silent:

 * a group grows only along a chain: the current sink must have exactly one
   consumer, used once, and must not be a graph output (otherwise the group
   would not have a single exit and is no kernel); then that consumer is the
   sink's immediate post-dominator;
 * the other operands of an absorbed operator are wildcards, the chain operand
   stays where the graph has it;
 * `grow_from_elemwise`: whether a group seeded by an element-wise operator
   grows as well (element-wise chains);
 * `max_ops` bounds the group size;
 * operators are visited in node order, groups grow smallest first, and a
   pattern already emitted is not emitted again: this fixes the order of the
   generated registry, which the placement search's tie-break depends on.
"""
from __future__ import annotations

WILD = "*"
NONE, FUSABLE, ELEMWISE = 0, 1, 2


def _pattern(kind, n_in, chain_pos, inner):
    args = tuple(inner if k == chain_pos else WILD for k in range(n_in))
    return (kind, args, ())


def generate(graph, op_class: dict, max_ops: int, grow_from_elemwise: bool):
    """Returns the generated patterns (pattern tuples as in the registries:
    (op, args, constraints)) in generation order.  `graph` is an oracle Graph;
    `op_class` maps operator kind -> NONE / FUSABLE / ELEMWISE."""
    out, seen = [], set()

    def emit(p):
        if p not in seen:
            seen.add(p)
            out.append(p)

    for v in graph.op_ids:
        nd = graph.nodes[v]
        cls = op_class.get(nd["kind"], NONE)
        if cls == NONE:
            continue
        pat = _pattern(nd["kind"], len(nd["inputs"]), -1, None)
        emit(pat)
        if cls == ELEMWISE and not grow_from_elemwise:
            continue
        sink, size = v, 1
        while size < max_ops:
            cons = graph.consumers[sink]
            if len(cons) != 1 or sink in graph.outputs:
                break
            u = cons[0]
            und = graph.nodes[u]
            if op_class.get(und["kind"], NONE) != ELEMWISE:
                break
            uses = [k for k, src in enumerate(und["inputs"]) if src == sink]
            if len(uses) != 1:
                break
            pat = _pattern(und["kind"], len(und["inputs"]), uses[0], pat)
            emit(pat)
            sink, size = u, size + 1
    return out
