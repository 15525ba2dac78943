"""Oracle pattern matcher: all matches (v_s, b_i) -> g of a registry on a graph.

TEST INFRASTRUCTURE ONLY (parity anchor; never imported by the product path).

Paper Sec. 3: a pattern is a tree of is_op(name)(args...) nodes, wildcards and
attribute constraints; the matching step of Alg. 1 asks, for a frontier node
v_s and a backend pattern b_i, for the subgraph g at v_s that b_i matches.
Readings the paper leaves open, fixed here:

 * v_s is the first node of g in the total order (depth, node id); the pattern
   text itself is sink-rooted as in the paper's listing.
 * A match is legal as one kernel only if every non-sink node of g has all of
   its consumers inside g and is not a graph output (single exit), the
   pattern's operator nodes bind distinct graph nodes, and no wildcard is bound
   to a non-sink operator of g itself: a wildcard is an operand that comes from
   outside the kernel, while a non-sink value of g exists only inside it (the
   subgraph is lowered to one kernel, Sec. 4.2) and no kernel ever writes it.
 * `add` is commutative: its operands are tried as written, then swapped.
 * At most one match is kept per (v_s, pattern): the first found when sinks are
   scanned in node order and operand orders in the order above.
 * Match ids are ranks in the order (rank of v_s, pattern registration index).
"""
from __future__ import annotations

from dataclasses import dataclass

WILD = "*"


@dataclass(frozen=True)
class Match:
    pattern: int          # index into the registry
    backend: str
    first: int            # v_s
    sink: int
    nodes: tuple          # operator nodes of g, ascending node id
    binding: tuple        # graph node bound to each pattern op node (post-order)


def _attr_value(graph, nid, name):
    nd = graph.nodes[nid]
    a = nd["attrs"]
    if name == "groups":
        return int(a.get("groups", 1))
    if name in ("kernel_h", "kernel_w"):
        idx = 0 if name == "kernel_h" else 1
        if "kernel" in a:
            return int(a["kernel"][idx])
        if len(nd["inputs"]) > 1:
            shp = graph.nodes[nd["inputs"][1]].get("shape")
            if shp is not None and len(shp) == 4:
                return int(shp[2 + idx])
        return None
    if name in ("stride_h", "stride_w"):
        return int(a["stride"][0 if name == "stride_h" else 1]) if "stride" in a else None
    if name in ("pad_h", "pad_w"):
        return int(a["pad"][0 if name == "pad_h" else 1]) if "pad" in a else None
    if name == "transpose_b":
        return int(bool(a.get("transpose_b", True)))
    if name == "axis":
        return int(a.get("axis", 1))
    raise KeyError(name)


def _assignments(graph, pat, nid):
    """All ways to match pattern `pat` with its root bound to graph value
    `nid`; each is a pair (graph nodes bound to the pattern's operators in
    pattern post-order, graph values bound to its wildcards)."""
    if pat == WILD:
        yield [], [nid]
        return
    op, args, constraints = pat
    nd = graph.nodes[nid]
    if nd["kind"] != op or len(nd["inputs"]) != len(args):
        return
    for name, (lo, hi) in constraints:
        v = _attr_value(graph, nid, name)
        if v is None or not (lo <= v <= hi):
            return
    orders = [list(nd["inputs"])]
    if op == "add" and len(args) == 2:
        orders.append([nd["inputs"][1], nd["inputs"][0]])

    def rec(k, operands):
        if k == len(args):
            yield [], []
            return
        for head, hw in _assignments(graph, args[k], operands[k]):
            for tail, tw in rec(k + 1, operands):
                yield head + tail, hw + tw

    for operands in orders:
        for sub, wild in rec(0, operands):
            yield sub + [nid], wild


def _legal(graph, bound, wild):
    if len(set(bound)) != len(bound):
        return False
    sink = bound[-1]
    inside = set(bound)
    if any(v in inside and v != sink for v in wild):
        return False
    outs = set(graph.outputs)
    for v in bound:
        if v == sink:
            continue
        if v in outs:
            return False
        if any(c not in inside for c in graph.consumers[v]):
            return False
    return True


def enumerate_matches(graph, registry):
    found = {}
    for pi, (backend, pat) in enumerate(registry):
        for sink in graph.op_ids:
            for bound, wild in _assignments(graph, pat, sink):
                if not _legal(graph, bound, wild):
                    continue
                first = min(bound, key=lambda v: graph.rank[v])
                key = (graph.rank[first], pi)
                if key not in found:
                    found[key] = Match(pi, backend, first, sink,
                                       tuple(sorted(bound)), tuple(bound))
    return [found[k] for k in sorted(found)]
