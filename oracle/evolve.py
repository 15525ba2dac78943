"""Oracle evolutionary search over digit strings (graph-level placement).

TEST INFRASTRUCTURE ONLY (parity anchor; never imported by the product path).

Paper Sec. 4.3: a placement is written as a string of digits, one per operator
the graph-level backend does not hold yet; 0 keeps the operator-level decision,
1 hands the operator over.  The search starts from a population that contains
the operator-level placement itself (all zeros) and repeats mutation, selection
and two-point crossover; the fitness of a string is measured on the whole
graph, because the graph-level backend's gains are not additive.  It ends at
saturation or at its limit.

The paper names the procedure and its operators and fixes no parameter; the
readings taken here:

 * fitness is a cost (lower is better); the best string ever evaluated is the
   result, and the earlier one wins a tie, so the result never costs more than
   the all-zero seed;
 * population: the seed, then `population - 1` strings whose digits are 1 with
   probability `p_init`; the paper makes the op-level placement "one of the
   seeds" without naming the others: with `seed_ones` the second string is all
   ones (every operator offloaded), the other end of the search space;
 * a generation, in the paper's order: (1) every string is mutated with
   probability `p_mutate`, each of its digits then flipping with probability
   `p_flip`; (2) `population` tournaments of `tournament` entrants drawn with
   replacement pick the next population (an entrant replaces the holder only if
   strictly cheaper); (3) neighbours (0,1), (2,3), ... exchange, with
   probability `p_cross`, the digits in [a, b) for two cut points drawn from
   0..n; (4) the new strings are evaluated;
 * a string is evaluated once (fitness values are kept by string);
 * saturation: `patience` > 0 ends the search after that many generations in a
   row without a new best;
 * randomness comes in as a sequence of 32-bit draws used in order: an event of
   probability p happens when draw / 2^32 < p, an index below m is
   (draw * m) >> 32.  Running out of draws is an error.
"""
from __future__ import annotations


class Draws:
    def __init__(self, rand):
        self.rand = [int(x) for x in rand]
        self.pos = 0

    def u32(self):
        if self.pos >= len(self.rand):
            raise ValueError("random draws exhausted")
        v = self.rand[self.pos]
        self.pos += 1
        return v

    def chance(self, p):
        return self.u32() / 4294967296.0 < p

    def below(self, m):
        return (self.u32() * m) >> 32


def evolve(n, fitness, rand, population=8, generations=10, tournament=3, patience=0,
           p_init=0.25, p_mutate=0.5, p_flip=0.1, p_cross=0.5, seed_ones=False):
    """Returns (best digits, best fitness, evaluations, history) where history[g]
    is the best fitness after generation g-1 (history[0]: the initial population)."""
    d = Draws(rand)
    known = {}
    state = {"best": None, "fit": None}

    def fit(ind):
        key = tuple(ind)
        if key not in known:
            known[key] = float(fitness(list(ind)))
            if state["best"] is None or known[key] < state["fit"]:
                state["best"], state["fit"] = list(ind), known[key]
        return known[key]

    pop = [[0] * n]
    for i in range(1, population):
        if i == 1 and seed_ones:                          # a second seed: every operator offloaded
            pop.append([1] * n)
        else:
            pop.append([1 if d.chance(p_init) else 0 for _ in range(n)])
    for ind in pop:
        fit(ind)
    history = [state["fit"]]
    stale = 0
    for _ in range(generations):
        before = state["fit"]
        for ind in pop:                                   # (1) mutation
            if d.chance(p_mutate):
                for b in range(n):
                    if d.chance(p_flip):
                        ind[b] ^= 1
        fits = [fit(ind) for ind in pop]
        nxt = []
        for _ in range(population):                       # (2) selection
            w = d.below(population)
            for _ in range(tournament - 1):
                c = d.below(population)
                if fits[c] < fits[w]:
                    w = c
            nxt.append(list(pop[w]))
        pop = nxt
        for i in range(0, population - 1, 2):             # (3) two-point crossover
            if d.chance(p_cross) and n >= 2:
                a, b = d.below(n + 1), d.below(n + 1)
                if a > b:
                    a, b = b, a
                pop[i][a:b], pop[i + 1][a:b] = pop[i + 1][a:b], pop[i][a:b]
        for ind in pop:                                   # (4) evaluation
            fit(ind)
        history.append(state["fit"])
        stale = 0 if state["fit"] < before else stale + 1
        if patience and stale >= patience:
            break
    return state["best"], state["fit"], len(known), history
