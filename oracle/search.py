"""Oracle placement search: the plain optimum and the paper's DP.

TEST INFRASTRUCTURE ONLY (parity anchor; never imported by the product path).

Plain definition (paper Eq. 1 with the additive model of Eq. 2/3):
    P_opt(G) = argmin over placements P(G) of  sum_i ( M(g_i, b_i) + eps ),
a placement being a set of pairwise-disjoint matches whose union is every
operator of G.  `brute_force_subsets` is that sentence written out (every
subset of the match list is tried); `exhaustive` enumerates the same set of
placements without the dead subsets, by always extending at the lowest
uncovered node.  `dp` follows Alg. 1 (priority queue of frontier nodes keyed by
depth, relaxation over the stored sub-placements S) and must return exactly
the plain optimum.

Readings fixed here where the paper is silent:
 * costs are int64 nanoseconds and eps is an int64 parameter, so sums are exact;
 * ties: minimise (total cost, tuple of match ids in order of their first
   nodes) lexicographically; match ids come from oracle.match;
 * the root v_0 is virtual: the first frontier is the lowest node of G in the
   order (depth, node id);
 * S for a match g found at v_s is every stored sub-placement whose lowest
   uncovered node is v_s and that is disjoint from g; the new frontier nodes F
   are the lowest uncovered nodes of s_j + g;
 * a cost of COST_INF or more is the measurer's word for "this backend cannot
   run this match" (Sec. 4.2: the measurer prices what a backend executes; the
   paper always has a fallback backend, so it never meets the case): such a
   match is no candidate, and a graph that only such matches could cover has
   no placement.
"""
from __future__ import annotations

import heapq
from itertools import combinations


COST_INF = 1 << 60


def _usable(costs, i):
    return int(costs[i]) < COST_INF


def _key(total, ids):
    return (int(total), tuple(ids))


def placement_cost(matches, costs, eps, ids):
    return sum(int(costs[i]) + int(eps) for i in ids)


# ---- Eq. 1, literally ---------------------------------------------------------
def brute_force_subsets(graph, matches, costs, eps=0, limit=22):
    m = len(matches)
    if m > limit:
        raise ValueError("too many matches for subset enumeration")
    need = set(graph.op_ids)
    best = None
    for r in range(1, m + 1):
        for ids in combinations(range(m), r):
            covered = set()
            ok = True
            for i in ids:
                g = matches[i].nodes
                if covered.intersection(g):
                    ok = False
                    break
                covered.update(g)
            if not ok or covered != need or not all(_usable(costs, i) for i in ids):
                continue
            k = _key(placement_cost(matches, costs, eps, ids), ids)
            if best is None or k < best:
                best = k
    return best  # (total, ids) or None


# ---- all placements, without the dead subsets -------------------------------------
def all_placements(graph, matches):
    """Yield every valid placement as an ascending tuple of match ids."""
    by_first = {}
    for i, m in enumerate(matches):
        by_first.setdefault(m.first, []).append(i)
    order = graph.order

    def rec(pos, covered, chosen):
        while pos < len(order) and order[pos] in covered:
            pos += 1
        if pos == len(order):
            yield tuple(chosen)
            return
        v = order[pos]
        for i in by_first.get(v, []):
            g = matches[i].nodes
            if covered.isdisjoint(g):
                yield from rec(pos + 1, covered | set(g), chosen + [i])

    yield from rec(0, frozenset(), [])


def exhaustive(graph, matches, costs, eps=0):
    best = None
    count = 0
    for ids in all_placements(graph, matches):
        count += 1
        if not all(_usable(costs, i) for i in ids):
            continue
        k = _key(placement_cost(matches, costs, eps, ids), ids)
        if best is None or k < best:
            best = k
    return best, count


# ---- Alg. 1 ---------------------------------------------------------------------
def dp(graph, registry, matches, costs, eps=0, stats=None):
    """Returns (total, ids) or None when no placement covers G."""
    get_match = {(m.first, m.pattern): i for i, m in enumerate(matches)}
    order = graph.order
    if not order:
        return _key(0, ())
    everything = frozenset(order)

    def lowest_uncovered(covered):
        for v in order:
            if v not in covered:
                return v
        return None

    c_opt = {frozenset(): (0, ())}          # C_opt(s), P_opt(s); C_opt(empty) = 0
    at_frontier = {order[0]: [frozenset()]}   # sub-placements waiting at a node
    queue = [(graph.depth[order[0]], order[0])]
    ever_queued = {order[0]}
    max_s = max_f = max_p = 0
    while queue:
        _, v_s = heapq.heappop(queue)
        n_matched = 0
        for bi in range(len(registry)):
            mid = get_match.get((v_s, bi))
            if mid is None:
                continue
            n_matched += 1
            if not _usable(costs, mid):
                continue
            g = frozenset(matches[mid].nodes)
            S = [s for s in at_frontier.get(v_s, []) if s.isdisjoint(g)]
            max_s = max(max_s, len(S))
            frontier = set()
            for s_j in S:
                s_new = s_j | g
                cand = (c_opt[s_j][0] + int(costs[mid]) + int(eps),
                        c_opt[s_j][1] + (mid,))
                if s_new not in c_opt:
                    c_opt[s_new] = cand
                    v_j = lowest_uncovered(s_new)
                    if v_j is not None:
                        at_frontier.setdefault(v_j, []).append(s_new)
                        frontier.add(v_j)
                elif cand < c_opt[s_new]:
                    c_opt[s_new] = cand
            max_f = max(max_f, len(frontier))
            for v_j in frontier:
                if v_j not in ever_queued:
                    ever_queued.add(v_j)
                    heapq.heappush(queue, (graph.depth[v_j], v_j))
        max_p = max(max_p, n_matched)
    if stats is not None:
        stats.update(N=len(order), P=max_p, F=max_f, S=max_s, states=len(c_opt))
    if everything not in c_opt:
        return None
    return _key(*c_opt[everything])
