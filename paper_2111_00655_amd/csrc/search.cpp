// Op-level placement search: the dynamic programme of paper Sec. 4.2
// (Eq. 3 and Alg. 1) over a cost table of integer nanoseconds.
//
// Stored sub-placements are keyed by the set of operators they cover.  The
// frontier nodes of Alg. 1 are visited in the order (depth, node id); because
// that order is total, the priority queue is a scan over positions that skips
// positions no sub-placement is waiting at (nodes never enqueued).  A match g
// found at frontier v_s relaxes every waiting sub-placement that is disjoint
// from g (the set S); the result waits at its own lowest uncovered node (the
// new frontier nodes F).  Each placement is generated along exactly one path,
// so the result is the minimum over all placements (Eq. 1).
//
// Ties: (total, ascending match-id list) is minimised lexicographically, which
// makes the answer a pure function of the inputs.
#include <algorithm>
#include <map>

#include "core.h"

namespace clg {

namespace {

using Bits = std::vector<uint64_t>;

struct Sub {                 // one stored sub-placement: C_opt(s), P_opt(s)
    Bits covered;
    int64_t cost = 0;
    int32_t parent = -1;     // sub-placement it extends
    int32_t match = -1;      // match added last
};

bool disjoint(const Bits &a, const Bits &b) {
    for (size_t i = 0; i < a.size(); ++i)
        if (a[i] & b[i]) return false;
    return true;
}

int lowest_clear(const Bits &b, int n) {
    for (size_t w = 0; w < b.size(); ++w) {
        const uint64_t inv = ~b[w];
        if (inv) {
            const int pos = (int)w * 64 + __builtin_ctzll(inv);
            return pos < n ? pos : n;
        }
    }
    return n;
}

void placement_of(const std::vector<Sub> &subs, int32_t idx, int32_t extra,
                  std::vector<int32_t> *out) {
    out->clear();
    if (extra >= 0) out->push_back(extra);
    for (int32_t s = idx; s >= 0 && subs[s].match >= 0; s = subs[s].parent)
        out->push_back(subs[s].match);
    std::reverse(out->begin(), out->end());
}

}  // namespace

int32_t search_dp(Graph &g, size_t, const int64_t *cost, int64_t eps,
                  std::vector<int32_t> *chosen, int64_t *total) {
    g.finalize();
    const int n = (int)g.order.size();
    const size_t words = (size_t)(n + 63) / 64 + 1;    // spare bits stay clear
    const size_t n_matches = g.matches.size();
    for (size_t i = 0; i < n_matches; ++i)
        if (cost[i] < 0) return fail(CLG_INVALID_ARG, "negative cost for match %zu", i);
    if (eps < 0) return fail(CLG_INVALID_ARG, "negative eps");

    std::vector<Bits> mbits(n_matches, Bits(words, 0));
    for (size_t i = 0; i < n_matches; ++i)
        for (int32_t v : g.matches[i].nodes) {
            const int r = g.rank[v];
            mbits[i][r / 64] |= (uint64_t)1 << (r % 64);
        }
    // matches are sorted by (rank of first node, pattern id): one contiguous
    // range per frontier position, already in registry order
    std::vector<size_t> range_begin(n + 1, n_matches);
    for (size_t i = n_matches; i-- > 0;) range_begin[g.rank[g.matches[i].first]] = i;
    for (int p = n - 1; p >= 0; --p)
        if (range_begin[p] == n_matches && p + 1 <= n) range_begin[p] = range_begin[p + 1];

    std::vector<Sub> subs;
    std::map<Bits, int32_t> index;
    std::vector<std::vector<int32_t>> waiting(n + 1);
    subs.push_back(Sub{Bits(words, 0), 0, -1, -1});        // C_opt(empty) = 0
    index[subs[0].covered] = 0;
    waiting[0].push_back(0);

    int64_t max_p = 0, max_f = 0, max_s = 0;
    std::vector<int32_t> pa, pb;
    for (int pos = 0; pos < n; ++pos) {
        if (waiting[pos].empty()) continue;                 // never enqueued
        const std::vector<int32_t> here = waiting[pos];
        int64_t n_here = 0;
        for (size_t mi = range_begin[pos];
             mi < n_matches && g.rank[g.matches[mi].first] == pos; ++mi) {
            ++n_here;
            if (cost[mi] >= CLG_COST_INF) continue;
            int64_t s_size = 0;
            std::vector<int> new_frontiers;
            for (int32_t si : here) {
                if (!disjoint(subs[si].covered, mbits[mi])) continue;
                ++s_size;
                Bits nb = subs[si].covered;
                for (size_t w = 0; w < words; ++w) nb[w] |= mbits[mi][w];
                const int64_t c = subs[si].cost + cost[mi] + eps;
                auto it = index.find(nb);
                if (it == index.end()) {
                    const int32_t id = (int32_t)subs.size();
                    const int f = lowest_clear(nb, n);
                    subs.push_back(Sub{nb, c, si, (int32_t)mi});
                    index.emplace(std::move(nb), id);
                    waiting[f].push_back(id);
                    if (std::find(new_frontiers.begin(), new_frontiers.end(), f) == new_frontiers.end())
                        new_frontiers.push_back(f);
                } else {
                    Sub &old = subs[it->second];
                    bool better = c < old.cost;
                    if (c == old.cost) {
                        placement_of(subs, si, (int32_t)mi, &pa);
                        placement_of(subs, it->second, -1, &pb);
                        better = pa < pb;
                    }
                    if (better) {
                        old.cost = c;
                        old.parent = si;
                        old.match = (int32_t)mi;
                    }
                }
            }
            max_s = std::max(max_s, s_size);
            max_f = std::max<int64_t>(max_f, (int64_t)new_frontiers.size());
        }
        max_p = std::max(max_p, n_here);
    }
    g.stats[0] = n; g.stats[1] = max_p; g.stats[2] = max_f; g.stats[3] = max_s;
    g.stats[4] = (int64_t)subs.size();

    Bits full(words, 0);
    for (int r = 0; r < n; ++r) full[r / 64] |= (uint64_t)1 << (r % 64);
    auto it = index.find(full);
    if (it == index.end())
        return fail(CLG_NOT_A_COVER, "no placement covers every operator of the graph");
    placement_of(subs, it->second, -1, chosen);
    *total = subs[it->second].cost;
    return CLG_OK;
}

}  // namespace clg
