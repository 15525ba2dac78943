// The C ABI (include/collage_mi.h): argument checking and marshalling only.
#include <cstdio>
#include <map>
#include <new>
#include <string>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "core.h"

using namespace clg;

#define CLG_TRY try {
#define CLG_CATCH                                                                     \
    } catch (const std::bad_alloc &) {                                                \
        return fail(CLG_OUT_OF_MEMORY, "host allocation failed");                     \
    } catch (const std::exception &e) {                                               \
        return fail(CLG_INVALID_ARG, "internal error: %s", e.what());                 \
    } catch (...) {                                                                   \
        return fail(CLG_INVALID_ARG, "internal error");                               \
    }
#define NEED(p) do { if (!(p)) return fail(CLG_INVALID_ARG, "%s: %s is null", __func__, #p); } while (0)

extern "C" {

int32_t clg_version(void) { return 102; }
const char *clg_last_error(void) { return last_error(); }

int32_t clg_create(clg_ctx **out, int32_t device) {
    CLG_TRY
    NEED(out);
    *out = nullptr;
    if (device < -1) return fail(CLG_INVALID_ARG, "device %d", device);
    clg_ctx *c = new clg_ctx();
    c->c.device = device;
    if (device >= 0) {
        int n = 0;
        hipError_t e = hipGetDeviceCount(&n);
        if (e != hipSuccess || device >= n) {
            delete c;
            return fail(CLG_HIP_ERROR, "device %d is not available (%d devices: %s)", device, n,
                        hipGetErrorString(e));
        }
        if ((e = hipSetDevice(device)) != hipSuccess) {
            delete c;
            return fail(CLG_HIP_ERROR, "hipSetDevice(%d): %s", device, hipGetErrorString(e));
        }
        const int32_t src = static_workspace_init(device);
        if (src != CLG_OK) {
            delete c;
            return src;
        }
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0)
            c->c.n_cus = cus;
    }
    *out = c;
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_destroy(clg_ctx *ctx) {
    if (!ctx) return CLG_OK;
    if (ctx->c.prof_ptr) (void)hipFree(ctx->c.prof_ptr);
    delete ctx;
    return CLG_OK;
}

int32_t clg_graph_create(clg_ctx *ctx, clg_graph **out) {
    CLG_TRY
    NEED(ctx); NEED(out);
    *out = new clg_graph();
    (*out)->g.ctx = &ctx->c;
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_graph_destroy(clg_graph *g) {
    if (g && g->g.live_plans > 0)
        return fail(CLG_INVALID_ARG, "the graph still has %d compiled plan(s): destroy them first", g->g.live_plans);
    delete g;
    return CLG_OK;
}

// A plan keeps node kinds, shapes and constant pointers of its graph by reference.
static int32_t graph_is_open(const clg_graph *g) {
    if (g->g.live_plans > 0)
        return fail(CLG_INVALID_ARG, "the graph has %d compiled plan(s) and can no longer be changed", g->g.live_plans);
    return CLG_OK;
}

static int32_t add_leaf(clg_graph *g, int32_t kind, int32_t dtype, int32_t ndim, const int64_t *dims,
                        const void *ptr, int32_t *node) {
    NEED(g); NEED(dims); NEED(node);
    if (graph_is_open(g) != CLG_OK) return CLG_INVALID_ARG;
    if (dtype != CLG_F32 && dtype != CLG_I32) return fail(CLG_INVALID_ARG, "dtype %d", dtype);
    if (ndim < 1 || ndim > CLG_MAX_DIMS) return fail(CLG_INVALID_ARG, "ndim %d", ndim);
    Node nd;
    nd.kind = kind;
    nd.dtype = dtype;
    nd.shape.ndim = ndim;
    for (int i = 0; i < ndim; ++i) {
        if (dims[i] < 1) return fail(CLG_INVALID_ARG, "dims[%d] = %lld", i, (long long)dims[i]);
        nd.shape.d[i] = dims[i];
    }
    if (nd.shape.numel() > kMaxTensorElems) return fail(CLG_INVALID_ARG, "tensor has more than 2^29 elements");
    nd.dev_ptr = ptr;
    if (kind == NODE_INPUT) nd.input_index = g->g.n_inputs++;
    g->g.nodes.push_back(nd);
    g->g.finalized = false;
    g->g.matched = false;
    *node = (int32_t)g->g.nodes.size() - 1;
    return CLG_OK;
}

int32_t clg_graph_input(clg_graph *g, int32_t dtype, int32_t ndim, const int64_t *dims, int32_t *node) {
    CLG_TRY
    return add_leaf(g, NODE_INPUT, dtype, ndim, dims, nullptr, node);
    CLG_CATCH
}

int32_t clg_graph_const(clg_graph *g, int32_t dtype, int32_t ndim, const int64_t *dims, const void *dev_ptr,
                        int32_t *node) {
    CLG_TRY
    return add_leaf(g, NODE_CONST, dtype, ndim, dims, dev_ptr, node);
    CLG_CATCH
}

int32_t clg_graph_op(clg_graph *g, int32_t op_kind, int32_t n_in, const int32_t *in_nodes, const clg_attrs *attrs,
                     int32_t *node) {
    CLG_TRY
    NEED(g); NEED(node);
    if (graph_is_open(g) != CLG_OK) return CLG_INVALID_ARG;
    if (n_in < 1 || n_in > CLG_MAX_PATTERN_ARGS) return fail(CLG_INVALID_ARG, "n_in %d", n_in);
    NEED(in_nodes);
    Node nd;
    nd.kind = op_kind;
    for (int i = 0; i < n_in; ++i) {
        if (in_nodes[i] < 0 || in_nodes[i] >= (int32_t)g->g.nodes.size())
            return fail(CLG_UNKNOWN_ID, "operand %d: node id %d", i, in_nodes[i]);
        nd.in.push_back(in_nodes[i]);
    }
    if (attrs) nd.attrs = *attrs;
    const int32_t rc = infer_shape(g->g, op_kind, nd.in, nd.attrs, &nd.shape, &nd.dtype);
    if (rc != CLG_OK) return rc;
    g->g.nodes.push_back(nd);
    g->g.finalized = false;
    g->g.matched = false;
    *node = (int32_t)g->g.nodes.size() - 1;
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_graph_mark_output(clg_graph *g, int32_t node) {
    CLG_TRY
    NEED(g);
    if (graph_is_open(g) != CLG_OK) return CLG_INVALID_ARG;
    if (node < 0 || node >= (int32_t)g->g.nodes.size()) return fail(CLG_UNKNOWN_ID, "node id %d", node);
    if (!g->g.nodes[node].is_op()) return fail(CLG_INVALID_ARG, "node %d is not an operator", node);
    for (int32_t o : g->g.outputs)
        if (o == node) return fail(CLG_INVALID_ARG, "node %d is already an output", node);
    g->g.outputs.push_back(node);
    g->g.finalized = false;
    g->g.matched = false;
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_graph_num_nodes(const clg_graph *g, int32_t *n) {
    NEED(g); NEED(n);
    *n = (int32_t)g->g.nodes.size();
    return CLG_OK;
}

int32_t clg_graph_node_shape(const clg_graph *g, int32_t node, int32_t *dtype, int32_t *ndim, int64_t *dims) {
    NEED(g); NEED(ndim); NEED(dims);
    if (node < 0 || node >= (int32_t)g->g.nodes.size()) return fail(CLG_UNKNOWN_ID, "node id %d", node);
    const Node &nd = g->g.nodes[node];
    if (dtype) *dtype = nd.dtype;
    *ndim = nd.shape.ndim;
    for (int i = 0; i < nd.shape.ndim; ++i) dims[i] = nd.shape.d[i];
    return CLG_OK;
}

int32_t clg_register_backend(clg_ctx *ctx, const char *name, int32_t *backend) {
    CLG_TRY
    NEED(ctx); NEED(name); NEED(backend);
    static const struct { const char *name; int32_t family, tile, no_split, rf_waves; } kKnown[] = {
        {"igemm", FAM_IGEMM, TILE_AUTO, 0, 0}, {"igemm_s", FAM_IGEMM, TILE_S, 0, 0}, {"igemm_m", FAM_IGEMM, TILE_M, 0, 0},
        {"igemm_l", FAM_IGEMM, TILE_L, 0, 0}, {"igemm_s8", FAM_IGEMM, TILE_S8, 0, 0}, {"igemm_s16", FAM_IGEMM, TILE_S16, 0, 0},
        {"igemm_r32", FAM_IGEMM, TILE_R32, 1, 0}, {"igemm_r16", FAM_IGEMM, TILE_R16, 1, 0},
        {"igemm_r32_w4", FAM_IGEMM, TILE_R32, 1, 4}, {"igemm_r32_w8", FAM_IGEMM, TILE_R32, 1, 8},
        {"igemm_r16_w4", FAM_IGEMM, TILE_R16, 1, 4}, {"igemm_r16_w8", FAM_IGEMM, TILE_R16, 1, 8},
        {"igemm_r16x2_w4", FAM_IGEMM, TILE_R16X2, 1, 4}, {"igemm_r16x2_w8", FAM_IGEMM, TILE_R16X2, 1, 8},
        {"igemm_r16_sk", FAM_IGEMM, TILE_R16, 0, 0}, {"igemm_r16_sk_w4", FAM_IGEMM, TILE_R16, 0, 4}, {"igemm_r32_sk", FAM_IGEMM, TILE_R32, 0, 0},
        {"igemm_s_nk", FAM_IGEMM, TILE_S, 1, 0}, {"igemm_s8_nk", FAM_IGEMM, TILE_S8, 1, 0}, {"igemm_s16_nk", FAM_IGEMM, TILE_S16, 1, 0},
        {"sepconv", FAM_SEPCONV, 0, 0, 0}, {"attention", FAM_ATTENTION, 0, 0, 0}, {"direct", FAM_DIRECT, 0, 0, 0}, {"rowwise", FAM_ROWWISE, 0, 0, 0}, {"eltwise", FAM_ELTWISE, 0, 0, 0}};
    const std::string s(name);
    for (size_t i = 0; i < ctx->c.backends.size(); ++i)
        if (ctx->c.backends[i].name == s) {
            *backend = (int32_t)i;
            return CLG_OK;
        }
    for (auto &k : kKnown)
        if (s == k.name) {
            ctx->c.backends.push_back(Backend{s, k.family, k.tile, k.no_split, k.rf_waves});
            *backend = (int32_t)ctx->c.backends.size() - 1;
            return CLG_OK;
        }
    return fail(CLG_UNKNOWN_ID, "no kernel family is called '%s'", name);
    CLG_CATCH
}

int32_t clg_register_pattern(clg_ctx *ctx, int32_t backend, const clg_pattern_node *nodes, int32_t n,
                             int32_t *pattern) {
    CLG_TRY
    NEED(ctx); NEED(nodes); NEED(pattern);
    if (backend < 0 || backend >= (int32_t)ctx->c.backends.size()) return fail(CLG_UNKNOWN_ID, "backend id %d", backend);
    if (n < 1 || n > CLG_MAX_PATTERN_NODES) return fail(CLG_INVALID_ARG, "pattern has %d nodes", n);
    Pattern p;
    p.backend = backend;
    p.nodes.assign(nodes, nodes + n);
    const int32_t rc = check_pattern(ctx->c, &p);
    if (rc != CLG_OK) return rc;
    ctx->c.patterns.push_back(std::move(p));
    *pattern = (int32_t)ctx->c.patterns.size() - 1;
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_num_patterns(const clg_ctx *ctx, int32_t *n) {
    NEED(ctx); NEED(n);
    *n = (int32_t)ctx->c.patterns.size();
    return CLG_OK;
}

int32_t clg_get_pattern(const clg_ctx *ctx, int32_t pattern, int32_t *backend, clg_pattern_node *nodes, int32_t cap,
                        int32_t *n) {
    NEED(ctx); NEED(n);
    if (pattern < 0 || pattern >= (int32_t)ctx->c.patterns.size()) return fail(CLG_UNKNOWN_ID, "pattern id %d", pattern);
    const Pattern &p = ctx->c.patterns[pattern];
    *n = (int32_t)p.nodes.size();
    if (backend) *backend = p.backend;
    if (cap == 0) return CLG_OK;
    NEED(nodes);
    if (cap < *n) return fail(CLG_INVALID_ARG, "pattern has %d nodes, room for %d", *n, cap);
    std::copy(p.nodes.begin(), p.nodes.end(), nodes);
    return CLG_OK;
}

int32_t clg_generate_patterns(clg_ctx *ctx, clg_graph *g, int32_t backend, const clg_pattern_rule *rule,
                              int32_t *n_added) {
    CLG_TRY
    NEED(ctx); NEED(g); NEED(rule);
    if (g->g.ctx != &ctx->c) return fail(CLG_INVALID_ARG, "graph belongs to another context");
    return generate_patterns(ctx->c, g->g, backend, *rule, n_added);
    CLG_CATCH
}

int32_t clg_match_all(clg_ctx *ctx, clg_graph *g, clg_match *out, size_t cap, size_t *n) {
    CLG_TRY
    NEED(ctx); NEED(g); NEED(n);
    if (g->g.ctx != &ctx->c) return fail(CLG_INVALID_ARG, "graph belongs to another context");
    const int32_t rc = match_all(ctx->c, g->g);
    if (rc != CLG_OK) return rc;
    *n = g->g.matches.size();
    if (cap == 0 && !out) return CLG_OK;
    NEED(out);
    if (cap < *n) return fail(CLG_BUFFER_TOO_SMALL, "%zu matches, room for %zu", *n, cap);
    for (size_t i = 0; i < *n; ++i) {
        const MatchRec &m = g->g.matches[i];
        clg_match &o = out[i];
        std::memset(&o, 0, sizeof o);
        o.pattern = m.pattern;
        o.backend = m.backend;
        o.first = m.first;
        o.sink = m.sink;
        o.n_nodes = (int32_t)m.nodes.size();
        for (size_t k = 0; k < m.nodes.size(); ++k) {
            o.nodes[k] = m.nodes[k];
            o.binding[k] = m.binding[k];
        }
    }
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_profile_match(clg_ctx *ctx, clg_graph *g, int32_t match, const clg_profile_opts *opts, int64_t *cost_ns) {
    CLG_TRY
    NEED(ctx); NEED(g); NEED(cost_ns);
    if (g->g.ctx != &ctx->c) return fail(CLG_INVALID_ARG, "graph belongs to another context");
    return profile_match(ctx->c, g->g, match, opts, cost_ns);
    CLG_CATCH
}

int32_t clg_profile_all(clg_ctx *ctx, clg_graph *g, const clg_profile_opts *opts, int64_t *cost_ns, size_t cap) {
    CLG_TRY
    NEED(ctx); NEED(g); NEED(cost_ns);
    if (g->g.ctx != &ctx->c) return fail(CLG_INVALID_ARG, "graph belongs to another context");
    if (!g->g.matched) return fail(CLG_INVALID_ARG, "clg_match_all has not been called on this graph");
    if (cap < g->g.matches.size()) return fail(CLG_BUFFER_TOO_SMALL, "%zu matches, room for %zu", g->g.matches.size(), cap);
    // Two passes some seconds apart, the smaller figure kept: now and then a whole measurement (all its
    // batches) comes out 1.3 - 1.6 times too long (the device's clocks, for some milliseconds), and a
    // candidate priced that way would lose the search for no reason.  The second pass measures what the
    // first one measured (not what the cost log already held) and serves everything else from the log.
    const size_t n = g->g.matches.size();
    std::vector<char> fresh(n, 0);
    for (size_t i = 0; i < n; ++i) {
        bool f = false;
        const int32_t rc = profile_match(ctx->c, g->g, (int32_t)i, opts, &cost_ns[i], &f);
        if (rc != CLG_OK) return rc;
        fresh[i] = f ? 1 : 0;
    }
    const bool cached = !opts || opts->no_cache == 0;
    for (size_t i = 0; i < n && cached; ++i) {
        if (fresh[i]) {
            const int32_t rc = profile_match(ctx->c, g->g, (int32_t)i, opts, &cost_ns[i], nullptr, true);
            if (rc != CLG_OK) return rc;
        }
    }
    for (size_t i = 0; i < n && cached; ++i) {          // matches that share a key share the final figure
        if (cost_ns[i] >= CLG_COST_INF) continue;
        const int32_t rc = profile_match(ctx->c, g->g, (int32_t)i, opts, &cost_ns[i]);
        if (rc != CLG_OK) return rc;
    }
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_profile_empty(clg_ctx *ctx, const clg_profile_opts *opts, int64_t *cost_ns) {
    CLG_TRY
    NEED(ctx); NEED(cost_ns);
    return profile_empty(ctx->c, opts, cost_ns);
    CLG_CATCH
}

int32_t clg_cost_log_load(clg_ctx *ctx, const char *path) {
    CLG_TRY
    NEED(ctx); NEED(path);
    return cost_log_load(ctx->c, path);
    CLG_CATCH
}

int32_t clg_cost_log_save(const clg_ctx *ctx, const char *path) {
    CLG_TRY
    NEED(ctx); NEED(path);
    return cost_log_save(ctx->c, path);
    CLG_CATCH
}

int32_t clg_cost_log_size(const clg_ctx *ctx, size_t *n) {
    NEED(ctx); NEED(n);
    *n = ctx->c.cost_log.size();
    return CLG_OK;
}

int32_t clg_match_key(clg_ctx *ctx, clg_graph *g, int32_t match, char *buf, size_t cap) {
    CLG_TRY
    NEED(ctx); NEED(g); NEED(buf);
    if (!g->g.matched) return fail(CLG_INVALID_ARG, "clg_match_all has not been called on this graph");
    KernelCall c;
    const int32_t rc = lower_match(ctx->c, g->g, match, &c);
    if (rc != CLG_OK) return rc;
    if (c.key.size() + 1 > cap) return fail(CLG_BUFFER_TOO_SMALL, "key needs %zu bytes", c.key.size() + 1);
    std::memcpy(buf, c.key.c_str(), c.key.size() + 1);
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_search_dp(clg_ctx *ctx, clg_graph *g, const int64_t *cost_ns, size_t n_costs, int64_t eps_ns,
                      int32_t *chosen, size_t cap, size_t *n_chosen, int64_t *total_ns) {
    CLG_TRY
    NEED(ctx); NEED(g); NEED(n_chosen); NEED(total_ns);
    if (g->g.ctx != &ctx->c) return fail(CLG_INVALID_ARG, "graph belongs to another context");
    if (!g->g.matched) return fail(CLG_INVALID_ARG, "clg_match_all has not been called on this graph");
    if (n_costs != g->g.matches.size())
        return fail(CLG_INVALID_ARG, "%zu costs for %zu matches", n_costs, g->g.matches.size());
    if (n_costs) NEED(cost_ns);
    std::vector<int32_t> sel;
    const int32_t rc = search_dp(g->g, ctx->c.patterns.size(), cost_ns, eps_ns, &sel, total_ns);
    if (rc != CLG_OK) return rc;
    *n_chosen = sel.size();
    if (sel.size() > cap) return fail(CLG_BUFFER_TOO_SMALL, "%zu chosen matches, room for %zu", sel.size(), cap);
    if (!sel.empty()) NEED(chosen);
    for (size_t i = 0; i < sel.size(); ++i) chosen[i] = sel[i];
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_search_stats(const clg_graph *g, int64_t stats[5]) {
    NEED(g); NEED(stats);
    for (int i = 0; i < 5; ++i) stats[i] = g->g.stats[i];
    return CLG_OK;
}

int32_t clg_compile(clg_ctx *ctx, clg_graph *g, const int32_t *matches, size_t n, clg_plan **out) {
    CLG_TRY
    NEED(ctx); NEED(g); NEED(out);
    *out = nullptr;
    if (n) NEED(matches);
    if (g->g.ctx != &ctx->c) return fail(CLG_INVALID_ARG, "graph belongs to another context");
    clg_plan *p = new clg_plan();
    const int32_t rc = compile_plan(ctx->c, g->g, matches, n, &p->p);
    if (rc != CLG_OK) {
        delete p;
        return rc;
    }
    ++g->g.live_plans;
    p->p.counted = true;
    *out = p;
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_plan_destroy(clg_plan *plan) {
    delete plan;
    return CLG_OK;
}

int32_t clg_plan_reads_constant(const clg_plan *plan, int32_t node, int32_t *reads, size_t *packed_bytes) {
    CLG_TRY
    NEED(plan); NEED(reads);
    const Plan &p = plan->p;
    if (node < 0 || node >= (int32_t)p.graph->nodes.size() || p.graph->nodes[node].kind != NODE_CONST)
        return fail(CLG_UNKNOWN_ID, "node %d is not a constant of the plan's graph", node);
    *reads = 0;
    size_t packed = 0;
    for (size_t i = 0; i < p.calls.size(); ++i) {
        const KernelCall &c = p.calls[i];
        if (c.pack_bytes && c.b_node == node) packed += c.pack_bytes;      // this kernel reads its packed copy instead
        else if (c.a_node == node || c.b_node == node || c.c_node == node) *reads = 1;
        for (int32_t v : c.epi_nodes)
            if (v == node) *reads = 1;
    }
    for (const Region &r : p.regions)
        for (size_t k = 0; k < r.members.size(); ++k)
            if (r.packed[k] && r.fused[k].b_node == node) packed += r.fused[k].pack_bytes;
    if (packed_bytes) *packed_bytes = packed;
    return CLG_OK;
    CLG_CATCH
}

int32_t clg_plan_workspace_bytes(const clg_plan *plan, size_t *bytes) {
    NEED(plan); NEED(bytes);
    *bytes = plan->p.workspace_bytes;
    return CLG_OK;
}

int32_t clg_plan_num_kernels(const clg_plan *plan, size_t *n) {
    NEED(plan); NEED(n);
    *n = plan->p.calls.size();
    return CLG_OK;
}

static int32_t check_es_opts(const clg_es_opts *o) {
    if (o->population < 2 || o->population > 4096) return fail(CLG_INVALID_ARG, "population must be 2..4096 (got %d)", o->population);
    if (o->generations < 0) return fail(CLG_INVALID_ARG, "generations %d", o->generations);
    if (o->tournament < 1 || o->tournament > 4096) return fail(CLG_INVALID_ARG, "tournament must be 1..4096 (got %d)", o->tournament);
    if (o->patience < 0) return fail(CLG_INVALID_ARG, "patience %d", o->patience);
    if (o->seed_ones != 0 && o->seed_ones != 1) return fail(CLG_INVALID_ARG, "seed_ones %d", o->seed_ones);
    for (double p : {o->p_init, o->p_mutate, o->p_flip, o->p_cross})
        if (!(p >= 0.0 && p <= 1.0)) return fail(CLG_INVALID_ARG, "a probability is outside [0, 1]");
    return CLG_OK;
}

int32_t clg_evolve(size_t n, const clg_es_opts *opts, const uint32_t *rand, size_t n_rand, clg_fitness_fn fitness,
                   void *user, uint8_t *best, double *best_cost, int64_t *evaluations, double *history,
                   int32_t *generations_run) {
    CLG_TRY
    NEED(opts); NEED(fitness); NEED(best_cost);
    if (n && !best) return fail(CLG_INVALID_ARG, "clg_evolve: best is null");
    if (n_rand && !rand) return fail(CLG_INVALID_ARG, "clg_evolve: rand is null");
    if (n > (1u << 20)) return fail(CLG_INVALID_ARG, "%zu digits", n);
    const int32_t rc = check_es_opts(opts);
    if (rc != CLG_OK) return rc;
    return evolve(n, *opts, rand, n_rand, fitness, user, best, best_cost, evaluations, history, generations_run);
    CLG_CATCH
}

static int32_t check_measure_opts(const clg_measure_opts *m) {
    if (m->warmup < 0 || m->batches < 1 || m->reps < 1 || m->batches > 1000 || m->reps > 100000)
        return fail(CLG_INVALID_ARG, "measure options: warmup %d batches %d reps %d", m->warmup, m->batches, m->reps);
    return CLG_OK;
}

int32_t clg_plan_set_handover(clg_plan *plan, const uint8_t *digits, size_t n, int32_t lanes) {
    CLG_TRY
    NEED(plan);
    if (n != plan->p.calls.size()) return fail(CLG_INVALID_ARG, "%zu digits for a plan of %zu kernels", n, plan->p.calls.size());
    if (n && !digits) return fail(CLG_INVALID_ARG, "clg_plan_set_handover: digits is null");
    if (lanes < 1 || lanes > 4) return fail(CLG_INVALID_ARG, "lanes must be 1..4 (got %d)", lanes);
    for (size_t i = 0; i < n; ++i)
        if (digits[i] > 1) return fail(CLG_INVALID_ARG, "digit %zu is %d", i, (int)digits[i]);
    plan->p.handed.assign(digits, digits + n);
    return set_plan_lanes(plan->p, lanes);
    CLG_CATCH
}

int32_t clg_plan_measure(clg_plan *plan, const void *const *inputs, void *const *outputs, void *workspace,
                         size_t workspace_bytes, void *stream, const clg_measure_opts *opts, int64_t *ns) {
    CLG_TRY
    NEED(plan); NEED(opts); NEED(ns);
    const int32_t rc = check_measure_opts(opts);
    if (rc != CLG_OK) return rc;
    return measure_plan(plan->p, inputs, outputs, workspace, workspace_bytes, stream, *opts, ns);
    CLG_CATCH
}

namespace {
struct GraphLevelJob {
    clg_plan *plan;
    const void *const *inputs;
    void *const *outputs;
    void *workspace;
    size_t ws_bytes;
    void *stream;
    int32_t lanes;
    clg_measure_opts m;
    int32_t rc = CLG_OK;
    std::string message;
    int64_t seed_ns = -1;
    std::map<std::vector<uint8_t>, int64_t> timed;     // launch sequence (see below) -> its measured time
};

// With one lane a digit changes the launch sequence only where its kernel sits in a region and at least one
// other member of that region is handed over too.  Strings that differ elsewhere run the very same launches:
// they are timed once and share the figure, so the search spends its measurements on distinct sequences and
// is not steered by the noise between two timings of one sequence.
void launch_sequence_key(const Plan &p, const uint8_t *digits, size_t n, std::vector<uint8_t> &key) {
    key.assign(n, 0);
    for (const Region &r : p.regions) {
        int in = 0;
        for (int32_t c : r.members) in += digits[c] ? 1 : 0;
        if (in >= 2)
            for (int32_t c : r.members) key[(size_t)c] = digits[c] ? 1 : 0;
    }
}

// fitness of the evolutionary search: set the string, time the whole sequence
double graph_level_cost(const uint8_t *digits, size_t n, void *user) {
    GraphLevelJob &j = *(GraphLevelJob *)user;
    if (j.rc != CLG_OK) return 0.0 / 0.0;
    int64_t ns = 0;
    std::vector<uint8_t> key;
    if (j.lanes == 1 && n == j.plan->p.calls.size()) {
        launch_sequence_key(j.plan->p, digits, n, key);
        const auto it = j.timed.find(key);
        if (it != j.timed.end()) return (double)it->second;
    }
    j.rc = clg_plan_set_handover(j.plan, digits, n, j.lanes);
    if (j.rc == CLG_OK) j.rc = measure_plan(j.plan->p, j.inputs, j.outputs, j.workspace, j.ws_bytes, j.stream, j.m, &ns);
    if (j.rc != CLG_OK) {
        j.message = last_error();
        return 0.0 / 0.0;
    }
    if (j.seed_ns < 0) j.seed_ns = ns;                 // the first string measured is the all-zero seed
    if (j.lanes == 1) j.timed.emplace(std::move(key), ns);
    return (double)ns;
}
}  // namespace

int32_t clg_search_graph_level(clg_plan *plan, const void *const *inputs, void *const *outputs, void *workspace,
                               size_t workspace_bytes, void *stream, int32_t lanes, const clg_es_opts *opts,
                               const uint32_t *rand, size_t n_rand, const clg_measure_opts *measure, uint8_t *best,
                               int64_t *best_ns, int64_t *seed_ns, int64_t *evaluations, double *history,
                               int32_t *generations_run) {
    CLG_TRY
    NEED(plan); NEED(opts); NEED(measure); NEED(best); NEED(best_ns);
    if (n_rand && !rand) return fail(CLG_INVALID_ARG, "clg_search_graph_level: rand is null");
    if (lanes < 1 || lanes > 4) return fail(CLG_INVALID_ARG, "lanes must be 1..4 (got %d)", lanes);
    int32_t rc = check_es_opts(opts);
    if (rc == CLG_OK) rc = check_measure_opts(measure);
    if (rc != CLG_OK) return rc;
    GraphLevelJob job{plan, inputs, outputs, workspace, workspace_bytes, stream, lanes, *measure, CLG_OK, {}, -1, {}};
    const size_t n = plan->p.calls.size();
    double cost = 0;
    rc = evolve(n, *opts, rand, n_rand, graph_level_cost, &job, best, &cost, evaluations, history, generations_run);
    if (job.rc != CLG_OK || rc != CLG_OK) {
        // leave the plan as the op-level placement, not as whatever string was tried last
        const std::string msg = job.rc != CLG_OK ? job.message : std::string(last_error());
        const std::vector<uint8_t> zeros(n, 0);
        (void)clg_plan_set_handover(plan, zeros.data(), n, lanes);
        return fail(job.rc != CLG_OK ? job.rc : rc, "%s", msg.c_str());
    }
    *best_ns = (int64_t)cost;
    if (seed_ns) *seed_ns = job.seed_ns;
    return clg_plan_set_handover(plan, best, n, lanes);
    CLG_CATCH
}

int32_t clg_plan_set_lanes(clg_plan *plan, int32_t lanes) {
    CLG_TRY
    NEED(plan);
    if (lanes < 1 || lanes > 4) return fail(CLG_INVALID_ARG, "lanes must be 1..4 (got %d)", lanes);
    plan->p.handed.clear();                            // every kernel may move
    return set_plan_lanes(plan->p, lanes);
    CLG_CATCH
}

int32_t clg_plan_num_launches(const clg_plan *plan, size_t *n) {
    NEED(plan); NEED(n);
    *n = plan_num_launches(plan->p);
    return CLG_OK;
}

int32_t clg_plan_region_of(const clg_plan *plan, size_t index, int32_t *region) {
    NEED(plan); NEED(region);
    if (index >= plan->p.calls.size()) return fail(CLG_UNKNOWN_ID, "kernel index %zu", index);
    *region = plan->p.region_of.empty() ? -1 : plan->p.region_of[index];
    return CLG_OK;
}

int32_t clg_plan_num_lanes(const clg_plan *plan, int32_t *lanes) {
    NEED(plan); NEED(lanes);
    *lanes = plan->p.n_lanes;
    return CLG_OK;
}

int32_t clg_plan_kernel_info(const clg_plan *plan, size_t index, clg_kernel_info *info) {
    NEED(plan); NEED(info);
    if (index >= plan->p.calls.size()) return fail(CLG_UNKNOWN_ID, "kernel index %zu", index);
    const KernelCall &c = plan->p.calls[index];
    std::memset(info, 0, sizeof *info);
    std::snprintf(info->name, sizeof info->name, "%s", c.name.c_str());
    info->match = c.match;
    info->bound = c.bound;
    info->flops = c.flops;
    info->bytes = c.bytes;
    return CLG_OK;
}

int32_t clg_execute(clg_plan *plan, const void *const *inputs, void *const *outputs, void *workspace,
                    size_t ws_bytes, void *stream) {
    CLG_TRY
    NEED(plan);
    return execute_plan(plan->p, inputs, outputs, workspace, ws_bytes, stream, nullptr);
    CLG_CATCH
}

int32_t clg_execute_static(clg_plan *plan, const void *const *inputs, void *const *outputs, void *stream) {
    CLG_TRY
    NEED(plan);
    return execute_plan_static(plan->p, inputs, outputs, stream);
    CLG_CATCH
}

int32_t clg_execute_timed(clg_plan *plan, const void *const *inputs, void *const *outputs, void *workspace,
                          size_t ws_bytes, void *stream, int64_t *kernel_ns, size_t cap) {
    CLG_TRY
    NEED(plan); NEED(kernel_ns);
    if (cap < plan->p.calls.size()) return fail(CLG_BUFFER_TOO_SMALL, "%zu kernels, room for %zu", plan->p.calls.size(), cap);
    return execute_plan(plan->p, inputs, outputs, workspace, ws_bytes, stream, kernel_ns);
    CLG_CATCH
}

}  // extern "C"
