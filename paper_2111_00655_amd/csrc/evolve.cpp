// Graph-level placement search (paper Sec. 4.3): evolutionary search over
// digit strings.  Digit i = 0 keeps the operator-level decision for item i,
// 1 hands the item to the graph-level backend.  The cost of a string is
// whatever the caller's function measures on the whole graph; it is not
// assumed to be a sum over digits.  The population starts from the all-zero
// string (the operator-level placement) and goes through mutation, tournament
// selection and two-point crossover each generation; the cheapest string ever
// measured is the result.
#include <cstring>
#include <string>
#include <unordered_map>
#include <vector>

#include "core.h"

namespace clg {

namespace {

using Digits = std::vector<uint8_t>;

struct Stream {
    const uint32_t *r;
    size_t n, pos = 0;
    bool dry = false;
    uint32_t next() {
        if (pos >= n) { dry = true; return 0; }
        return r[pos++];
    }
    // probability p: the draw, read as a fraction of 2^32, lies below p
    bool chance(double p) { return (double)next() / 4294967296.0 < p; }
    // uniform index in [0, m)
    uint32_t below(uint32_t m) { return (uint32_t)(((uint64_t)next() * m) >> 32); }
};

struct Ledger {                      // every string measured so far, and the cheapest of them
    clg_fitness_fn fn;
    void *user;
    std::unordered_map<std::string, double> cost;
    Digits best;
    double best_cost = 0;
    bool have = false, failed = false;
    double of(const Digits &d) {
        std::string key((const char *)d.data(), d.size());
        auto it = cost.find(key);
        if (it != cost.end()) return it->second;
        const double c = fn(d.data(), d.size(), user);
        if (!(c == c)) failed = true;                // NaN: the caller's measurement failed
        cost.emplace(std::move(key), c);
        if (!have || c < best_cost) { best = d; best_cost = c; have = true; }
        return c;
    }
};

}  // namespace

int32_t evolve(size_t n, const clg_es_opts &o, const uint32_t *rand, size_t n_rand, clg_fitness_fn fn, void *user,
               uint8_t *best, double *best_cost, int64_t *evaluations, double *history, int32_t *generations_run) {
    const size_t P = (size_t)o.population;
    Stream rs{rand, n_rand};
    Ledger led{fn, user, {}, {}, 0, false, false};
    std::vector<Digits> pop(P, Digits(n, 0));
    for (size_t i = 1; i < P; ++i) {
        if (i == 1 && o.seed_ones) {
            pop[i].assign(n, 1);                   // the second seed: everything handed over
            continue;
        }
        for (size_t b = 0; b < n; ++b) pop[i][b] = rs.chance(o.p_init) ? 1 : 0;
    }
    if (rs.dry) return fail(CLG_INVALID_ARG, "random draws exhausted while building the population");
    for (auto &d : pop) led.of(d);
    if (led.failed) return fail(CLG_INVALID_ARG, "the fitness function returned NaN");
    if (history) history[0] = led.best_cost;
    int32_t gen = 0, stale = 0;
    std::vector<double> cost(P);
    std::vector<Digits> next(P);
    for (; gen < o.generations; ++gen) {
        const double before = led.best_cost;
        for (auto &d : pop)                                           // mutation
            if (rs.chance(o.p_mutate))
                for (size_t b = 0; b < n; ++b)
                    if (rs.chance(o.p_flip)) d[b] ^= 1;
        // a missing draw reads as 0: strings built from such draws are never measured
        if (rs.dry) return fail(CLG_INVALID_ARG, "random draws exhausted in generation %d (%zu given)", gen, n_rand);
        for (size_t i = 0; i < P; ++i) cost[i] = led.of(pop[i]);
        for (size_t i = 0; i < P; ++i) {                              // selection
            uint32_t w = rs.below((uint32_t)P);
            for (int32_t t = 1; t < o.tournament; ++t) {
                const uint32_t c = rs.below((uint32_t)P);
                if (cost[c] < cost[w]) w = c;
            }
            next[i] = pop[w];
        }
        pop.swap(next);
        for (size_t i = 0; i + 1 < P; i += 2) {                       // two-point crossover
            if (!rs.chance(o.p_cross) || n < 2) continue;
            uint32_t a = rs.below((uint32_t)n + 1), b = rs.below((uint32_t)n + 1);
            if (a > b) std::swap(a, b);
            for (uint32_t k = a; k < b; ++k) std::swap(pop[i][k], pop[i + 1][k]);
        }
        if (rs.dry) return fail(CLG_INVALID_ARG, "random draws exhausted in generation %d (%zu given)", gen, n_rand);
        for (auto &d : pop) led.of(d);
        if (led.failed) return fail(CLG_INVALID_ARG, "the fitness function returned NaN");
        if (history) history[gen + 1] = led.best_cost;
        stale = led.best_cost < before ? 0 : stale + 1;
        if (o.patience > 0 && stale >= o.patience) { ++gen; break; }
    }
    if (n) std::memcpy(best, led.best.data(), n);
    *best_cost = led.best_cost;
    if (evaluations) *evaluations = (int64_t)led.cost.size();
    if (generations_run) *generations_run = gen;
    return CLG_OK;
}

}  // namespace clg
