// Placement -> kernel sequence (paper Sec. 4.1: a placement is a set of
// disjoint matches covering G; Sec. 5.1: tensors are handed between backends
// by pointer, without copies), and its execution on a HIP stream.
#include <algorithm>

#include <hip/hip_runtime_api.h>

#include "core.h"

namespace clg {

namespace {

constexpr int64_t kAlign = 256;
int64_t round_up(int64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// First-fit allocator over one linear workspace; tracks the peak.
struct Arena {
    struct Block { int64_t off, size; };
    std::vector<Block> live;     // sorted by offset
    int64_t peak = 0;
    int64_t alloc(int64_t bytes) {
        const int64_t size = round_up(std::max<int64_t>(bytes, 1));
        int64_t off = 0;
        size_t pos = 0;
        for (; pos < live.size(); ++pos) {
            if (live[pos].off - off >= size) break;
            off = live[pos].off + live[pos].size;
        }
        live.insert(live.begin() + (long)pos, Block{off, size});
        peak = std::max(peak, off + size);
        return off;
    }
    void release(int64_t off) {
        for (size_t i = 0; i < live.size(); ++i)
            if (live[i].off == off) {
                live.erase(live.begin() + (long)i);
                return;
            }
    }
};

std::vector<int32_t> operands_of(const KernelCall &c) {
    std::vector<int32_t> v;
    for (int32_t x : {c.a_node, c.b_node, c.c_node})
        if (x >= 0) v.push_back(x);
    for (int32_t x : c.epi_nodes)
        if (x >= 0) v.push_back(x);
    return v;
}

// ---- regions (the graph-level backend, paper Sec. 4.3) -------------------------------------------
// Which several-problems-per-launch kernel could run the call beside siblings of the same class
// (0: none): 1 register-fed dense, 2 register-fed 1x1 convolution, 3 thread-per-output kernels
// (depthwise convolution with its unrolled-tap kernel, window pools), 100 and up separable convolutions.
enum RegionClass { RC_NONE = 0, RC_DENSE = 1, RC_CONV1X1 = 2, RC_PLANE = 3, RC_SEPCONV = 100 };
int region_class(const KernelCall &c) {
    if (c.kind == CALL_SEPCONV) return RC_SEPCONV + sepconv_region_key(c.sep);      // one class per kernel instantiation
    if (c.kind == CALL_DIRECT_CONV) return depthwise_fast_ok(c.dconv) ? RC_PLANE : RC_NONE;
    if (c.kind == CALL_POOL) return plane_region_pool_ok(c.pool) ? RC_PLANE : RC_NONE;
    if (c.kind != CALL_GEMM || !c.gemm.rf_ts || c.gemm.splitk != 1 || !c.pack_bytes) return RC_NONE;
    const GemmArgs &a = c.gemm;
    if (a.rf_tapk == -1) return RC_DENSE;
    return a.rf_tapk == 1 && !a.rf_convt && !a.rf_fold ? RC_CONV1X1 : RC_NONE;
}

// Lowers member `c` again for the leader's kernel shape (tile edge, K-waves per workgroup).
bool relower_for(const Context &ctx, const KernelCall &leader, const KernelCall &c, KernelCall *out) {
    *out = c;
    if (c.kind != CALL_GEMM) return true;                    // thread-per-output kernels: every member runs as it is
    GemmArgs &a = out->gemm;
    const int ts = leader.gemm.rf_ts, wgk = leader.gemm.rf_wgk;
    if (a.rf_ts != ts || a.rf_wgk != wgk || a.rf_nb != leader.gemm.rf_nb) {
        const int flags = epi_fast_flags(a.epi);
        const bool dense = a.rf_tapk == -1;
        if (!dense && (a.KD > 1 || a.rf_fold)) return false;
        const bool ok = dense ? rf_resolve_dense(&a, ts, flags, ctx.n_cus, wgk, leader.gemm.rf_nb == 2 ? 2 : 1)
                              : rf_resolve(&a, ts, flags, ctx.n_cus, wgk);
        if (!ok) return false;
        out->pack_bytes = rf_pack_bytes(a);
        out->scratch_bytes = gemm_scratch_bytes(a);
    }
    return out->scratch_bytes == 0 && rf_same_launch_shape(leader.gemm, a);
}

// Finds the regions of a freshly lowered kernel sequence and moves every member next to its region's
// first one (a member only moves forward past kernels it does not depend on, so the order stays
// topological).  Greedy and deterministic: scanning in order, a kernel of a fusable kind opens a
// region; later kernels of the same family join when everything they read was produced before the
// region's first kernel and the common kernel shape (that of the member with the most flops) takes them.
void find_regions(const Context &ctx, const Graph &g, Plan *plan) {
    std::vector<KernelCall> &calls = plan->calls;
    const size_t nc = calls.size();
    std::vector<int32_t> produced_at(g.nodes.size(), -1);
    for (size_t i = 0; i < nc; ++i) produced_at[calls[i].out_node] = (int32_t)i;
    std::vector<int32_t> reg_of(nc, -1);
    struct Found { std::vector<int32_t> members; std::vector<KernelCall> fused; };
    std::vector<Found> found;
    for (size_t i = 0; i < nc; ++i) {
        const int cls = region_class(calls[i]);
        if (reg_of[i] >= 0 || cls == RC_NONE) continue;
        std::vector<int32_t> cand{(int32_t)i};
        const size_t cap = cls == RC_PLANE ? (size_t)kMaxPlaneRegion : (cls >= RC_SEPCONV ? (size_t)kMaxSepRegion : (size_t)kMaxRegion);
        for (size_t j = i + 1; j < nc && cand.size() < cap; ++j) {
            if (reg_of[j] >= 0 || region_class(calls[j]) != cls) continue;
            bool free = true;
            for (int32_t v : operands_of(calls[j]))
                if (g.nodes[v].is_op() && produced_at[v] >= (int32_t)i) free = false;
            if (free) cand.push_back((int32_t)j);
        }
        if (cand.size() < 2) continue;
        int32_t lead = cand[0];
        for (int32_t c : cand)
            if (calls[c].flops > calls[lead].flops) lead = c;
        Found f;
        for (int32_t c : cand) {
            KernelCall fc;
            if (relower_for(ctx, calls[lead], calls[c], &fc)) {
                f.members.push_back(c);
                f.fused.push_back(std::move(fc));
            }
        }
        if (f.members.size() < 2 || f.members[0] != (int32_t)i) continue;     // the opener must be in (else try from the next kernel)
        for (int32_t c : f.members) reg_of[c] = (int32_t)found.size();
        found.push_back(std::move(f));
    }
    plan->regions.clear();
    plan->region_of.assign(nc, -1);
    plan->fuse_mark.assign(nc, 0);
    if (found.empty()) return;
    // new order: a region's members right behind its first one
    std::vector<int32_t> order, new_pos(nc, -1);
    for (size_t i = 0; i < nc; ++i) {
        if (reg_of[i] >= 0 && found[reg_of[i]].members[0] != (int32_t)i) continue;     // emitted with its region
        if (reg_of[i] < 0) {
            new_pos[i] = (int32_t)order.size();
            order.push_back((int32_t)i);
        } else {
            for (int32_t c : found[reg_of[i]].members) {
                new_pos[c] = (int32_t)order.size();
                order.push_back(c);
            }
        }
    }
    std::vector<KernelCall> moved;
    moved.reserve(nc);
    for (int32_t c : order) moved.push_back(std::move(calls[c]));
    calls.swap(moved);
    for (Found &f : found) {
        Region r;
        for (int32_t c : f.members) {
            r.members.push_back(new_pos[c]);
            plan->region_of[new_pos[c]] = (int32_t)plan->regions.size();
        }
        r.fused = std::move(f.fused);
        r.packed.assign(r.members.size(), nullptr);
        plan->regions.push_back(std::move(r));
    }
}

}  // namespace

size_t plan_num_launches(const Plan &p) {
    size_t n = 0;
    for (size_t i = 0; i < p.calls.size(); ++i) n += p.elided[i] ? 0 : 1;
    if (p.max_lanes > 1 || p.handed.empty()) return n;
    for (const Region &r : p.regions) {
        size_t in = 0;
        for (int32_t c : r.members) in += p.handed[c] ? 1 : 0;
        if (in >= 2) n -= in - 1;
    }
    return n;
}

int32_t compile_plan(Context &ctx, Graph &g, const int32_t *ids, size_t n, Plan *plan) {
    g.finalize();
    if (!g.matched) return fail(CLG_INVALID_ARG, "clg_match_all has not been called on this graph");
    const int n_nodes = (int)g.nodes.size();
    std::vector<int32_t> owner(n_nodes, -1);
    for (size_t i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= (int32_t)g.matches.size())
            return fail(CLG_UNKNOWN_ID, "match id %d (the graph has %zu matches)", ids[i], g.matches.size());
        for (int32_t v : g.matches[ids[i]].nodes) {
            if (owner[v] >= 0)
                return fail(CLG_OVERLAP, "matches %d and %d both contain node %d", owner[v], ids[i], v);
            owner[v] = ids[i];
        }
    }
    for (int32_t v : g.op_ids)
        if (owner[v] < 0) return fail(CLG_NOT_A_COVER, "operator node %d (%s) is not covered", v, op_name(g.nodes[v].kind));

    // a group reads other groups only through their sinks, so ordering groups
    // by the position of their sink is a topological order of the quotient graph
    std::vector<int32_t> seq(ids, ids + n);
    std::sort(seq.begin(), seq.end(), [&](int32_t a, int32_t b) {
        return g.rank[g.matches[a].sink] < g.rank[g.matches[b].sink];
    });

    plan->ctx = &ctx;
    plan->graph = &g;
    plan->calls.clear();
    for (int32_t id : seq) {
        KernelCall c;
        const int32_t rc = lower_match(ctx, g, id, &c);
        if (rc != CLG_OK) return rc;
        plan->calls.push_back(std::move(c));
    }
    find_regions(ctx, g, plan);

    // every operand must be a leaf or the sink of an earlier group
    const size_t nc = plan->calls.size();
    std::vector<int32_t> produced_at(n_nodes, -1);
    for (size_t i = 0; i < nc; ++i) {
        for (int32_t v : operands_of(plan->calls[i])) {
            if (!g.nodes[v].is_op()) continue;
            if (produced_at[v] < 0)
                return fail(CLG_INVALID_ARG, "kernel %zu reads node %d before any kernel has produced it", i, v);
        }
        produced_at[plan->calls[i].out_node] = (int32_t)i;
    }

    // Concatenation without a copy (Sec. 5.1 hands tensors over by pointer): when the extents before the
    // axis are all 1, every operand is one contiguous piece of the result.  If each operand is produced by a
    // kernel of this plan, has no buffer of its own to go to (not a graph output), is not already part of
    // another concatenation and starts on a 16-byte boundary, its producer writes it straight into its place
    // in the result and the concatenation launches nothing.  Such results nest (root = outermost one).
    plan->value_offset.assign(n_nodes, -1);
    plan->value_output.assign(n_nodes, -1);
    plan->scratch_offset.assign(nc, -1);
    plan->elided.assign(nc, 0);
    std::vector<int32_t> alias_of(n_nodes, -1);
    std::vector<int64_t> alias_delta(n_nodes, 0);
    for (size_t k = 0; k < g.outputs.size(); ++k) plan->value_output[g.outputs[k]] = (int32_t)k;
    for (size_t i = 0; i < nc; ++i) {
        const KernelCall &c = plan->calls[i];
        if (c.kind != CALL_CONCAT || c.cat.outer != 1) continue;
        bool ok = true;
        int64_t off = 0;
        for (int k = 0; k < c.cat.n && ok; ++k) {
            const int32_t v = c.epi_nodes[k];
            ok = g.nodes[v].is_op() && plan->value_output[v] < 0 && alias_of[v] < 0 && off % 16 == 0;
            for (int j = 0; j < k; ++j) ok = ok && c.epi_nodes[j] != v;
            off += 4 * c.cat.chunk[k];
        }
        if (!ok) continue;
        off = 0;
        for (int k = 0; k < c.cat.n; ++k) {
            alias_of[c.epi_nodes[k]] = c.out_node;
            alias_delta[c.epi_nodes[k]] = off;
            off += 4 * c.cat.chunk[k];
        }
        plan->elided[i] = 1;
        plan->calls[i].name += "_alias";
        plan->calls[i].bytes = 0;
    }
    std::vector<int32_t> root(n_nodes);
    std::vector<int64_t> delta(n_nodes, 0);                  // byte offset of a value inside its root's buffer
    for (int v = n_nodes - 1; v >= 0; --v) {                 // a result comes after its operands: roots resolve first
        root[v] = alias_of[v] < 0 ? v : root[alias_of[v]];
        delta[v] = alias_of[v] < 0 ? 0 : delta[alias_of[v]] + alias_delta[v];
    }

    // workspace: one buffer per root value that is not a graph output, reused once the last reader of the
    // root or of any value inside it has run; per-call scratch lives for its call only
    plan->value_delta.assign(n_nodes, 0);
    std::vector<int32_t> release_at(n_nodes, -1);            // root -> call after which its buffer is free
    for (size_t i = 0; i < nc; ++i) {
        const int32_t r = root[plan->calls[i].out_node];
        release_at[r] = std::max(release_at[r], (int32_t)i);
        for (int32_t v : operands_of(plan->calls[i])) release_at[root[v]] = std::max(release_at[root[v]], (int32_t)i);
    }
    std::vector<std::vector<int32_t>> releases(nc);
    for (int v = 0; v < n_nodes; ++v)
        if (root[v] == v && release_at[v] >= 0 && g.nodes[v].is_op() && plan->value_output[v] < 0)
            releases[(size_t)release_at[v]].push_back(v);
    Arena arena;
    auto place_output = [&](size_t i) {
        const int32_t v = plan->calls[i].out_node, r = root[v];
        if (plan->value_output[r] >= 0) {
            if (v != r) {
                plan->value_output[v] = plan->value_output[r];
                plan->value_delta[v] = delta[v];
            }
        } else {
            if (plan->value_offset[r] < 0) plan->value_offset[r] = arena.alloc(4 * g.nodes[r].shape.numel());
            plan->value_offset[v] = plan->value_offset[r] + delta[v];
        }
    };
    // The members of a region may run as one launch: all their results are placed before any of them
    // runs, and what they read is released only after the last of them.  The plan so made holds for
    // every choice of digits (members run one by one use the same buffers in the same order).
    for (size_t i = 0; i < nc; ++i) {
        const KernelCall &c = plan->calls[i];
        const int32_t ri = plan->region_of[i];
        const bool first_of_region = ri >= 0 && plan->regions[ri].members.front() == (int32_t)i;
        const bool last_of_region = ri >= 0 && plan->regions[ri].members.back() == (int32_t)i;
        if (ri < 0) place_output(i);
        else if (first_of_region)
            for (int32_t m : plan->regions[ri].members) place_output((size_t)m);
        if (c.scratch_bytes) {
            plan->scratch_offset[i] = arena.alloc((int64_t)c.scratch_bytes);
            arena.release(plan->scratch_offset[i]);
        }
        if (ri < 0) {
            for (int32_t r2 : releases[i]) arena.release(plan->value_offset[r2]);
        } else if (last_of_region) {
            for (int32_t m : plan->regions[ri].members)
                for (int32_t r2 : releases[(size_t)m]) arena.release(plan->value_offset[r2]);
        }
    }
    plan->workspace_bytes = (size_t)arena.peak;
    schedule_lanes(plan);

    // kernels that read their weights in a packed order get a private copy,
    // written once here and owned by the plan
    plan->packed.assign(nc, nullptr);
    if (ctx.device >= 0) {
        bool any = false;
        for (size_t i = 0; i < nc; ++i) {
            const KernelCall &c = plan->calls[i];
            if (!c.pack_bytes) continue;
            const void *w = g.nodes[c.b_node].dev_ptr;
            if (!w) return fail(CLG_INVALID_ARG, "constant node %d has no device pointer", c.b_node);
            if (hipMalloc(&plan->packed[i], c.pack_bytes) != hipSuccess) {
                (void)hipGetLastError();
                plan->packed[i] = nullptr;
                return fail(CLG_OUT_OF_MEMORY, "allocation of %zu bytes for packed weights failed", c.pack_bytes);
            }
            const int32_t rc = pack_weights(c, w, plan->packed[i], nullptr);
            if (rc != CLG_OK) return rc;
            any = true;
        }
        // a region member whose kernel shape differs inside the region reads a second packed copy
        for (Region &r : plan->regions)
            for (size_t k = 0; k < r.members.size(); ++k) {
                const KernelCall &own = plan->calls[(size_t)r.members[k]], &fc = r.fused[k];
                if (fc.gemm.rf_ts == own.gemm.rf_ts && fc.gemm.rf_wgk == own.gemm.rf_wgk && fc.pack_bytes == own.pack_bytes) continue;
                const void *w = g.nodes[fc.b_node].dev_ptr;
                if (hipMalloc(&r.packed[k], fc.pack_bytes) != hipSuccess) {
                    (void)hipGetLastError();
                    r.packed[k] = nullptr;
                    return fail(CLG_OUT_OF_MEMORY, "allocation of %zu bytes for packed weights failed", fc.pack_bytes);
                }
                const int32_t rc = pack_weights(fc, w, r.packed[k], nullptr);
                if (rc != CLG_OK) return rc;
                any = true;
            }
        if (any && hipStreamSynchronize(nullptr) != hipSuccess)
            return fail(CLG_HIP_ERROR, "weight packing failed: %s", hipGetErrorString(hipGetLastError()));
    }
    return CLG_OK;
}

Plan::~Plan() {
    if (counted && graph) --graph->live_plans;
    for (void *p : packed)
        if (p) (void)hipFree(p);
    for (Region &r : regions)
        for (void *p : r.packed)
            if (p) (void)hipFree(p);
    for (void *e : events)
        if (e) (void)hipEventDestroy((hipEvent_t)e);
    for (void *e : ev_end)
        if (e) (void)hipEventDestroy((hipEvent_t)e);
    if (ev_begin) (void)hipEventDestroy((hipEvent_t)ev_begin);
    for (void *s : side_streams)
        if (s) (void)hipStreamDestroy((hipStream_t)s);
}

int32_t set_plan_lanes(Plan &p, int32_t lanes) {
    for (void *s : p.side_streams)
        if (s && hipStreamSynchronize((hipStream_t)s) != hipSuccess)
            return fail(CLG_HIP_ERROR, "synchronising a lane failed: %s", hipGetErrorString(hipGetLastError()));
    for (void *e : p.events)
        if (e) (void)hipEventDestroy((hipEvent_t)e);
    for (void *e : p.ev_end)
        if (e) (void)hipEventDestroy((hipEvent_t)e);
    if (p.ev_begin) (void)hipEventDestroy((hipEvent_t)p.ev_begin);
    for (void *s : p.side_streams)
        if (s) (void)hipStreamDestroy((hipStream_t)s);
    p.events.clear();
    p.ev_end.clear();
    p.ev_begin = nullptr;
    p.side_streams.clear();
    p.max_lanes = lanes;
    schedule_lanes(&p);
    return CLG_OK;
}

// Lane schedule.  A placement's quotient graph has independent branches (the
// projection shortcut next to the main path of a residual block; the query, key
// and value projections of an attention layer), and at batch 1 one kernel rarely
// fills the chip, so such branches run on different HIP streams.  Dependencies
// are the data dependencies between kernels plus every reuse of a workspace
// region (the workspace was planned for the sequential order).  Kernels are
// still enqueued in plan order; a kernel stays on the lane of its latest
// dependency when everything queued there is among its (transitive)
// dependencies, and otherwise moves to another lane, waiting on events for what
// it needs from elsewhere.
void schedule_lanes(Plan *plan) {
    const Graph &g = *plan->graph;
    const size_t nc = plan->calls.size();
    plan->lane.assign(nc, 0);
    plan->waits.assign(nc, {});
    plan->signals.assign(nc, 0);
    plan->n_lanes = 1;
    if (plan->max_lanes <= 1 || nc < 3) return;

    struct Region { int64_t lo, hi; };
    auto overlap = [](const std::vector<Region> &a, const std::vector<Region> &b) {
        for (const Region &x : a)
            for (const Region &y : b)
                if (x.lo < y.hi && y.lo < x.hi) return true;
        return false;
    };
    std::vector<std::vector<Region>> rd(nc), wr(nc);
    std::vector<int32_t> produced_at(g.nodes.size(), -1);
    for (size_t i = 0; i < nc; ++i) {
        const KernelCall &c = plan->calls[i];
        for (int32_t v : operands_of(c))
            if (plan->value_offset[v] >= 0)
                rd[i].push_back({plan->value_offset[v], plan->value_offset[v] + round_up(4 * g.nodes[v].shape.numel())});
        if (plan->value_offset[c.out_node] >= 0)
            wr[i].push_back({plan->value_offset[c.out_node],
                             plan->value_offset[c.out_node] + round_up(4 * g.nodes[c.out_node].shape.numel())});
        if (plan->scratch_offset[i] >= 0)
            wr[i].push_back({plan->scratch_offset[i], plan->scratch_offset[i] + round_up((int64_t)c.scratch_bytes)});
        produced_at[c.out_node] = (int32_t)i;
    }
    // direct dependencies and their transitive closure (bit sets over calls)
    const size_t words = (nc + 63) / 64;
    std::vector<std::vector<int32_t>> deps(nc);
    std::vector<std::vector<uint64_t>> reach(nc, std::vector<uint64_t>(words, 0));
    for (size_t j = 0; j < nc; ++j) {
        for (int32_t v : operands_of(plan->calls[j])) {
            const int32_t i = g.nodes[v].is_op() ? produced_at[v] : -1;
            if (i >= 0 && (size_t)i < j) deps[j].push_back(i);
        }
        for (size_t i = 0; i < j; ++i)
            if (overlap(wr[j], rd[i]) || overlap(wr[j], wr[i]) || overlap(rd[j], wr[i])) deps[j].push_back((int32_t)i);
        std::sort(deps[j].begin(), deps[j].end());
        deps[j].erase(std::unique(deps[j].begin(), deps[j].end()), deps[j].end());
        for (int32_t i : deps[j]) {
            reach[j][(size_t)i / 64] |= (uint64_t)1 << (i % 64);
            for (size_t w = 0; w < words; ++w) reach[j][w] |= reach[i][w];
        }
    }
    auto depends = [&](size_t j, int32_t i) { return i < 0 || ((reach[j][(size_t)i / 64] >> (i % 64)) & 1) != 0; };

    const int lanes = std::min<int>(plan->max_lanes, 4);
    std::vector<int32_t> last(lanes, -1);            // last call queued on each lane
    for (size_t j = 0; j < nc; ++j) {
        int pick = (!plan->handed.empty() && !plan->handed[j]) ? 0 : -1;   // not handed over: the caller's stream
        const int home = deps[j].empty() ? 0 : plan->lane[deps[j].back()];
        if (pick < 0 && depends(j, last[home])) pick = home;
        for (int l = 0; l < lanes && pick < 0; ++l)
            if (depends(j, last[l])) pick = l;         // a lane whose queue this call follows anyway (or an idle one)
        if (pick < 0) {                                // every lane holds unrelated work: join the least recently used
            pick = 0;
            for (int l = 1; l < lanes; ++l)
                if (last[l] < last[pick]) pick = l;
        }
        plan->lane[j] = pick;
        last[pick] = (int32_t)j;
        plan->n_lanes = std::max(plan->n_lanes, pick + 1);
        // wait for the latest direct dependency on every other lane (a lane runs in order)
        std::vector<int32_t> latest(lanes, -1);
        for (int32_t i : deps[j])
            if (plan->lane[i] != pick) latest[plan->lane[i]] = std::max(latest[plan->lane[i]], i);
        for (int l = 0; l < lanes; ++l)
            if (latest[l] >= 0) {
                plan->waits[j].push_back(latest[l]);
                plan->signals[latest[l]] = 1;
            }
    }
}

int32_t measure_plan(Plan &p, const void *const *inputs, void *const *outputs, void *workspace, size_t ws_bytes,
                     void *stream, const clg_measure_opts &o, int64_t *ns) {
    if (p.ctx->device < 0) return fail(CLG_HIP_ERROR, "host-only context: no device to execute on");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return fail(CLG_HIP_ERROR, "hipEventCreate failed");
    }
    int32_t rc = CLG_OK;
    double best = -1;
    for (int32_t i = 0; i < o.warmup && rc == CLG_OK; ++i)
        rc = execute_plan(p, inputs, outputs, workspace, ws_bytes, stream, nullptr);
    for (int32_t b = 0; b < o.batches && rc == CLG_OK; ++b) {
        (void)hipEventRecord(e0, (hipStream_t)stream);
        for (int32_t i = 0; i < o.reps && rc == CLG_OK; ++i)
            rc = execute_plan(p, inputs, outputs, workspace, ws_bytes, stream, nullptr);
        (void)hipEventRecord(e1, (hipStream_t)stream);
        if (hipEventSynchronize(e1) != hipSuccess && rc == CLG_OK)
            rc = fail(CLG_HIP_ERROR, "waiting for a timed batch failed: %s", hipGetErrorString(hipGetLastError()));
        float ms = 0.f;
        if (rc == CLG_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = fail(CLG_HIP_ERROR, "hipEventElapsedTime failed");
        const double per = (double)ms * 1.0e6 / o.reps;
        if (best < 0 || per < best) best = per;
    }
    if (rc != CLG_OK) (void)hipStreamSynchronize((hipStream_t)stream);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == CLG_OK) *ns = (int64_t)(best + 0.5);
    return rc;
}

int32_t pack_weights(const KernelCall &c, const void *w, void *dst, void *stream) {
    const int err = c.kind == CALL_SEPCONV ? launch_sepconv_pack(c.sep, (const float *)w, (float *)dst, stream)
                                           : launch_rf_pack(c.gemm, (const float *)w, (float *)dst, stream);
    if (err != 0) return fail(CLG_HIP_ERROR, "weight packing launch failed: %s", hipGetErrorString((hipError_t)err));
    return CLG_OK;
}

int32_t bind_gemm(const KernelCall &c, const void *a, const void *b, void *out, const void *const *epi_ptrs,
                  void *scratch, const void *packed, GemmArgs *kp) {
    GemmArgs &k = *kp;
    k = c.gemm;
    k.A = (const float *)a; k.B = (const float *)b; k.C = (float *)out;
    if (c.gemm_swap) {                               // A = weights, B = activations
        k.A = (const float *)b; k.B = (const float *)a;
    }
    if (c.pack_bytes) {
        if (!packed) return fail(CLG_INVALID_ARG, "%s needs packed weights, none were prepared", c.name.c_str());
        if (c.gemm.rf_tapk == -1) k.B = (const float *)packed;      // dense: the weights are the second operand
        else k.A = (const float *)packed;
    }
    k.partial = (float *)scratch;
    for (int s = 0; s < k.epi.n; ++s) k.epi.s[s].ptr = (const float *)epi_ptrs[s];
    return CLG_OK;
}

int32_t launch_call(const KernelCall &c, const void *a, const void *b, const void *c3, void *out,
                    const void *const *epi_ptrs, void *scratch, const void *packed, void *stream) {
    auto bind = [&](Epilogue e) {
        for (int s = 0; s < e.n; ++s) e.s[s].ptr = (const float *)epi_ptrs[s];
        return e;
    };
    int err = 0;
    switch (c.kind) {
    case CALL_GEMM: {
        GemmArgs k;
        const int32_t rc = bind_gemm(c, a, b, out, epi_ptrs, scratch, packed, &k);
        if (rc != CLG_OK) return rc;
        err = launch_gemm(k, stream);
        break;
    }
    case CALL_DIRECT_CONV: {
        DirectConvArgs k = c.dconv;
        k.x = (const float *)a; k.w = (const float *)b; k.y = (float *)out;
        k.epi = bind(c.dconv.epi);
        err = launch_direct_conv(k, stream);
        break;
    }
    case CALL_POOL: {
        PoolArgs k = c.pool;
        k.x = (const float *)a; k.y = (float *)out;
        k.epi = bind(c.pool.epi);
        err = launch_pool(k, stream);
        break;
    }
    case CALL_ROWWISE: {
        RowwiseArgs k = c.row;
        k.x = (const float *)a; k.gamma = (const float *)b; k.beta = (const float *)c3; k.y = (float *)out;
        k.pro = bind(c.row.pro);
        for (int t = 0; t < k.n_gather; ++t) {           // an embedding: tables and id lists ride in the step slots
            k.tab[t] = (const float *)epi_ptrs[t];
            k.gid[t] = (const int32_t *)epi_ptrs[3 + t];
        }
        if (k.n_gather) k.x = nullptr;
        err = launch_rowwise(k, stream);
        break;
    }
    case CALL_ELTWISE: {
        EltwiseArgs k = c.elt;
        k.x = (const float *)a; k.ids = (const int32_t *)b; k.y = (float *)out;
        k.epi = bind(c.elt.epi);
        err = launch_eltwise(k, stream);
        break;
    }
    case CALL_LAYOUT: {
        LayoutArgs k = c.layout;
        k.x = (const float *)a; k.y = (float *)out;
        err = launch_layout(k, stream);
        break;
    }
    case CALL_SEPCONV: {
        if (!packed) return fail(CLG_INVALID_ARG, "%s needs packed weights, none were prepared", c.name.c_str());
        SepConvArgs k = c.sep;
        k.x = (const float *)a; k.wp = (const float *)packed; k.wd = (const float *)c3; k.y = (float *)out;
        k.epi = bind(c.sep.epi);
        err = launch_sepconv(k, stream);
        break;
    }
    case CALL_ATTENTION: {
        AttentionArgs k = c.att;
        k.q = (const float *)a; k.k = (const float *)b; k.v = (const float *)c3; k.y = (float *)out;
        err = launch_attention(k, stream);
        break;
    }
    case CALL_CONCAT: {
        ConcatArgs k = c.cat;
        for (int s = 0; s < k.n; ++s) k.src[s] = (const float *)epi_ptrs[s];
        k.y = (float *)out;
        err = launch_concat(k, stream);
        break;
    }
    default:
        return fail(CLG_INVALID_ARG, "unknown call kind %d", c.kind);
    }
    if (err != 0)
        return fail(CLG_HIP_ERROR, "launch of %s failed: %s", c.name.c_str(), hipGetErrorString((hipError_t)err));
    return CLG_OK;
}

int32_t execute_plan(Plan &p, const void *const *inputs, void *const *outputs, void *workspace,
                     size_t ws_bytes, void *stream, int64_t *kernel_ns) {
    Context &ctx = *p.ctx;
    Graph &g = *p.graph;
    if (ctx.device < 0) return fail(CLG_HIP_ERROR, "host-only context: no device to execute on");
    if (ws_bytes < p.workspace_bytes)
        return fail(CLG_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, the plan needs %zu", ws_bytes, p.workspace_bytes);
    if (p.workspace_bytes && !workspace) return fail(CLG_INVALID_ARG, "workspace is null");
    if (((uintptr_t)workspace & 255) != 0) return fail(CLG_INVALID_ARG, "workspace is not 256-byte aligned");
    if ((g.n_inputs && !inputs) || (!g.outputs.empty() && !outputs)) return fail(CLG_INVALID_ARG, "inputs/outputs is null");
    for (int i = 0; i < g.n_inputs; ++i)
        if (!inputs[i]) return fail(CLG_INVALID_ARG, "input %d is null", i);
    for (size_t i = 0; i < g.outputs.size(); ++i)
        if (!outputs[i]) return fail(CLG_INVALID_ARG, "output %zu is null", i);

    auto ptr_of = [&](int32_t v) -> const void * {
        if (v < 0) return nullptr;
        const Node &nd = g.nodes[v];
        if (nd.kind == NODE_CONST) return nd.dev_ptr;
        if (nd.kind == NODE_INPUT) return inputs[nd.input_index];
        if (p.value_output[v] >= 0) return (const char *)outputs[p.value_output[v]] + p.value_delta[v];
        return (const char *)workspace + p.value_offset[v];
    };
    std::vector<hipEvent_t> ev;
    if (kernel_ns) {
        ev.resize(2 * p.calls.size());
        for (auto &e : ev)
            if (hipEventCreate(&e) != hipSuccess) return fail(CLG_HIP_ERROR, "hipEventCreate failed");
    }
    // lanes: per-kernel timing runs everything on the caller's stream
    const bool lanes = !kernel_ns && p.n_lanes > 1;
    hipError_t he = hipSuccess;
    if (lanes) {
        if (p.side_streams.empty()) {                  // first execution: the plan's own streams and events
            p.side_streams.assign((size_t)p.n_lanes - 1, nullptr);
            p.ev_end.assign((size_t)p.n_lanes - 1, nullptr);
            p.events.assign(p.calls.size(), nullptr);
            for (auto &s : p.side_streams)
                if (he == hipSuccess) he = hipStreamCreateWithFlags((hipStream_t *)&s, hipStreamNonBlocking);
            for (auto &e : p.ev_end)
                if (he == hipSuccess) he = hipEventCreateWithFlags((hipEvent_t *)&e, hipEventDisableTiming);
            if (he == hipSuccess) he = hipEventCreateWithFlags((hipEvent_t *)&p.ev_begin, hipEventDisableTiming);
            for (size_t i = 0; i < p.calls.size(); ++i)
                if (p.signals[i] && he == hipSuccess)
                    he = hipEventCreateWithFlags((hipEvent_t *)&p.events[i], hipEventDisableTiming);
            if (he != hipSuccess) {
                p.n_lanes = 1;                         // the partly built set is released with the plan
                return fail(CLG_HIP_ERROR, "creating the plan's streams and events failed: %s", hipGetErrorString(he));
            }
        }
        // the side lanes start after everything already queued on the caller's stream
        he = hipEventRecord((hipEvent_t)p.ev_begin, (hipStream_t)stream);
        for (void *s : p.side_streams)
            if (he == hipSuccess) he = hipStreamWaitEvent((hipStream_t)s, (hipEvent_t)p.ev_begin, 0);
        if (he != hipSuccess) return fail(CLG_HIP_ERROR, "lane fork failed: %s", hipGetErrorString(he));
    }
    auto stream_of = [&](size_t i) -> void * {
        return (lanes && p.lane[i] > 0) ? p.side_streams[(size_t)p.lane[i] - 1] : stream;
    };
    int32_t rc = CLG_OK;
    // regions: with one lane, the handed-over members of a region (two or more) go out as one launch
    const bool fuse = p.max_lanes <= 1 && !p.handed.empty() && !p.regions.empty();
    std::vector<char> &done = p.fuse_mark;             // sized at compile time: nothing is allocated here
    if (fuse) std::fill(done.begin(), done.end(), 0);
    for (size_t i = 0; i < p.calls.size() && rc == CLG_OK; ++i) {
        const KernelCall &c = p.calls[i];
        if (fuse && done[i]) continue;
        if (fuse && p.region_of[i] >= 0 && p.handed[i]) {
            const Region &r = p.regions[(size_t)p.region_of[i]];
            const bool sep = c.kind == CALL_SEPCONV;
            const bool plane = c.kind != CALL_GEMM && !sep;          // a region of thread-per-output kernels
            GemmArgs members[kMaxRegion];
            SepConvArgs smembers[kMaxSepRegion];
            PlaneMultiArgs &pm = p.plane_args;           // (part of the plan: nothing this large goes on the stack per call)
            size_t idx[kMaxPlaneRegion];
            int nm = 0;
            for (size_t k = 0; k < r.members.size(); ++k) {
                const size_t ci = (size_t)r.members[k];
                if (ci < i || !p.handed[ci]) continue;
                const KernelCall &fc = r.fused[k];
                const void *fepi[kMaxEpi];
                for (int s = 0; s < kMaxEpi; ++s) fepi[s] = ptr_of(fc.epi_nodes[s]);
                if (sep) {
                    if (!p.packed[ci]) rc = fail(CLG_INVALID_ARG, "%s needs packed weights, none were prepared", fc.name.c_str());
                    SepConvArgs &k2 = smembers[nm];
                    k2 = fc.sep;
                    k2.x = (const float *)ptr_of(fc.a_node); k2.wp = (const float *)p.packed[ci];
                    k2.wd = (const float *)ptr_of(fc.c_node);
                    k2.y = (float *)const_cast<void *>(ptr_of(fc.out_node));
                    for (int s = 0; s < k2.epi.n; ++s) k2.epi.s[s].ptr = (const float *)fepi[s];
                } else if (plane) {
                    if (fc.kind == CALL_DIRECT_CONV) {
                        DirectConvArgs &k2 = pm.p[nm].dw;
                        k2 = fc.dconv;
                        k2.x = (const float *)ptr_of(fc.a_node); k2.w = (const float *)ptr_of(fc.b_node);
                        k2.y = (float *)const_cast<void *>(ptr_of(fc.out_node));
                        for (int s = 0; s < k2.epi.n; ++s) k2.epi.s[s].ptr = (const float *)fepi[s];
                        pm.kind[nm] = k2.KH;
                    } else {
                        PoolArgs &k2 = pm.p[nm].pool;
                        k2 = fc.pool;
                        k2.x = (const float *)ptr_of(fc.a_node);
                        k2.y = (float *)const_cast<void *>(ptr_of(fc.out_node));
                        for (int s = 0; s < k2.epi.n; ++s) k2.epi.s[s].ptr = (const float *)fepi[s];
                        pm.kind[nm] = k2.mode == 0 ? 10 : 11;
                    }
                } else {
                    const void *pk = r.packed[k] ? r.packed[k] : p.packed[ci];
                    rc = bind_gemm(fc, ptr_of(fc.a_node), ptr_of(fc.b_node), const_cast<void *>(ptr_of(fc.out_node)), fepi,
                                   nullptr, pk, &members[nm]);
                }
                if (rc != CLG_OK) break;
                idx[nm++] = ci;
            }
            if (rc != CLG_OK) break;
            if (nm >= 2) {
                if (kernel_ns) (void)hipEventRecord(ev[2 * i], (hipStream_t)stream);
                pm.n = nm;
                const int err = sep ? launch_sepconv_region(smembers, nm, stream)
                                    : (plane ? launch_plane_region(pm, stream) : launch_gemm_region(members, nm, stream));
                if (kernel_ns) (void)hipEventRecord(ev[2 * i + 1], (hipStream_t)stream);
                if (err != 0) rc = fail(CLG_HIP_ERROR, "launch of the region around %s failed: %s", c.name.c_str(),
                                        hipGetErrorString((hipError_t)err));
                for (int k = 0; k < nm; ++k) done[idx[k]] = 1;
                done[i] = 2;                         // carries the region's time
                continue;
            }
        }
        const void *epi[kMaxEpi];
        for (int s = 0; s < kMaxEpi; ++s) epi[s] = ptr_of(c.epi_nodes[s]);
        for (int32_t v : {c.a_node, c.b_node, c.c_node})
            if (v >= 0 && !ptr_of(v)) rc = fail(CLG_INVALID_ARG, "constant node %d has no device pointer", v);
        if (rc != CLG_OK) break;
        void *scratch = p.scratch_offset[i] >= 0 ? (char *)workspace + p.scratch_offset[i] : nullptr;
        void *st = stream_of(i);
        if (lanes)
            for (int32_t w : p.waits[i])
                if (hipStreamWaitEvent((hipStream_t)st, (hipEvent_t)p.events[w], 0) != hipSuccess)
                    rc = fail(CLG_HIP_ERROR, "hipStreamWaitEvent failed");
        if (rc != CLG_OK) break;
        if (kernel_ns && !p.elided[i]) (void)hipEventRecord(ev[2 * i], (hipStream_t)stream);
        if (!p.elided[i])                                // an aliased concatenation: its operands are already in place
            rc = launch_call(c, ptr_of(c.a_node), ptr_of(c.b_node), ptr_of(c.c_node),
                             const_cast<void *>(ptr_of(c.out_node)), epi, scratch, p.packed[i], st);
        if (kernel_ns && !p.elided[i]) (void)hipEventRecord(ev[2 * i + 1], (hipStream_t)stream);
        if (lanes && p.signals[i] && rc == CLG_OK && hipEventRecord((hipEvent_t)p.events[i], (hipStream_t)st) != hipSuccess)
            rc = fail(CLG_HIP_ERROR, "hipEventRecord failed");
    }
    if (lanes) {
        // join: the caller's stream continues after every side lane (also after a failed launch, so that
        // nothing the plan queued is left running behind the caller's back)
        for (size_t l = 0; l < p.side_streams.size(); ++l) {
            he = hipEventRecord((hipEvent_t)p.ev_end[l], (hipStream_t)p.side_streams[l]);
            if (he == hipSuccess) he = hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)p.ev_end[l], 0);
            if (he != hipSuccess && rc == CLG_OK) rc = fail(CLG_HIP_ERROR, "lane join failed: %s", hipGetErrorString(he));
        }
    }
    if (kernel_ns) {
        if (rc == CLG_OK && hipStreamSynchronize((hipStream_t)stream) != hipSuccess)
            rc = fail(CLG_HIP_ERROR, "stream synchronisation failed: %s", hipGetErrorString(hipGetLastError()));
        for (size_t i = 0; i < p.calls.size() && rc == CLG_OK; ++i) {
            float ms = 0.f;
            if (p.elided[i] || (fuse && done[i] == 1)) {     // nothing launched, or launched with its region's first kernel
                kernel_ns[i] = 0;
                continue;
            }
            if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess)
                rc = fail(CLG_HIP_ERROR, "hipEventElapsedTime failed");
            kernel_ns[i] = (int64_t)((double)ms * 1.0e6 + 0.5);
        }
        for (auto &e : ev) (void)hipEventDestroy(e);
    }
    return rc;
}

}  // namespace clg
