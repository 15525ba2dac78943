// The measurer M of paper Sec. 4.2: given a placement it reports what the
// placement really costs at run time.  It is asked about one matched subgraph,
// i.e. one kernel, at a time; pricing means building the kernel and running it
// several times on the device, and every result is kept in a log for reuse.
//
// Protocol: a few launches to size the batches, untimed batches until two in a
// row agree within a tenth (the measurer's host work between two candidates
// leaves the GPU idle long enough for its clocks to drop; launches bring them
// back up), then
// `batches` timed batches of back-to-back launches between two HIP events; the
// cost is the smallest batch time per launch, rounded once to integer
// nanoseconds.  (The smallest, not the median:
// on a shared host the enqueueing thread is descheduled for milliseconds at a
// time, which inflates whole batches by 2-3x; such a stall can only add time,
// so the undisturbed batch is the fastest one.)  The figure is launch-inclusive
// (it contains the dispatch gap between consecutive kernels), so the search
// can use eps = 0.
//
// Operands rotate: inside a network a kernel finds neither its weights nor its
// input in the L2 of the compute die it runs on (the weights of a whole model
// pass through between two uses; the input was just written by another
// kernel), while the same launch repeated on the same buffers finds everything
// there and looks up to a third cheaper - and looks cheaper by different
// amounts for different kernel variants, which misleads the search.  So the
// measurer keeps several copies of the large operands (inputs, output, packed
// or plain weights), 64 MB in all or at most 32 copies, and launch i works on
// copy i mod R: every launch misses the L2 and hits the memory-side cache, as
// in the network.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <fstream>

#include <hip/hip_runtime_api.h>

#include "core.h"

namespace clg {

namespace {

// One growing device allocation held by the context and reused across matches.
int32_t ensure_block(Context &ctx, size_t need) {
    if (need <= ctx.prof_bytes) return CLG_OK;
    if (ctx.prof_ptr) (void)hipFree(ctx.prof_ptr);
    ctx.prof_ptr = nullptr;
    ctx.prof_bytes = 0;
    if (hipMalloc(&ctx.prof_ptr, need) != hipSuccess) {
        (void)hipGetLastError();
        ctx.prof_ptr = nullptr;
        return fail(CLG_OUT_OF_MEMORY, "profiler scratch allocation of %zu bytes failed", need);
    }
    ctx.prof_bytes = need;
    return CLG_OK;
}

struct Opts { int warmup, batches, min_batch_us, max_launches; uint64_t seed; bool cache; };

Opts resolve(const clg_profile_opts *o) {
    Opts r{20, 7, 200, 2000, 1, true};
    if (!o) return r;
    if (o->warmup > 0) r.warmup = o->warmup;
    if (o->batches > 0) r.batches = o->batches;
    if (o->min_batch_us > 0) r.min_batch_us = o->min_batch_us;
    if (o->max_launches > 0) r.max_launches = o->max_launches;
    if (o->seed) r.seed = o->seed;
    r.cache = o->no_cache == 0;
    return r;
}

int32_t hip_fail(const char *what, hipError_t e) {
    return fail(CLG_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
}

// Times `launch(i)` (which enqueues the kernel once on the default stream; i counts the launches).
template <class F>
int32_t time_launches(const Opts &o, F &&launch, int64_t *cost_ns) {
    int launched = 0;
    hipEvent_t e0, e1;
    hipError_t he;
    if ((he = hipEventCreate(&e0)) != hipSuccess) return hip_fail("hipEventCreate", he);
    if ((he = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail("hipEventCreate", he); }
    int32_t rc = CLG_OK;
    auto run = [&](int n, double *ms_total) -> int32_t {
        (void)hipEventRecord(e0, nullptr);
        for (int i = 0; i < n; ++i) {
            const int32_t r = launch(launched++);
            if (r != CLG_OK) return r;
        }
        (void)hipEventRecord(e1, nullptr);
        if ((he = hipEventSynchronize(e1)) != hipSuccess) return hip_fail("hipEventSynchronize", he);
        float ms = 0.f;
        if ((he = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) return hip_fail("hipEventElapsedTime", he);
        *ms_total = ms;
        return CLG_OK;
    };
    double ms = 0;
    rc = run(o.warmup, &ms);
    int n = 10;
    if (rc == CLG_OK) {
        const double per_us = std::max(ms * 1000.0 / o.warmup, 0.05);
        n = (int)std::min<double>(o.max_launches, std::max(5.0, std::ceil(o.min_batch_us / per_us)));
    }
    // untimed batches until two in a row agree within a tenth (at most six): the fills and packing in
    // front of a measurement and the host work between candidates let the clocks drop, and short kernels
    // would otherwise be timed while they ramp up again (whole measurements came out at twice their value)
    double prev = -1;
    for (int settle = 0; settle < 6 && rc == CLG_OK; ++settle) {
        rc = run(n, &ms);
        if (prev > 0 && std::fabs(ms - prev) <= 0.1 * std::min(ms, prev)) break;
        prev = ms;
    }
    std::vector<double> per;
    for (int b = 0; b < o.batches && rc == CLG_OK; ++b) {
        rc = run(n, &ms);
        per.push_back(ms * 1.0e6 / n);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != CLG_OK) return rc;
    *cost_ns = std::max<int64_t>(1, (int64_t)std::llround(*std::min_element(per.begin(), per.end())));
    return CLG_OK;
}

}  // namespace

int32_t profile_empty(Context &ctx, const clg_profile_opts *opts, int64_t *cost_ns) {
    if (ctx.device < 0) return fail(CLG_HIP_ERROR, "host-only context: no device to profile on");
    const Opts o = resolve(opts);
    return time_launches(o, [&](int) -> int32_t {
        const int e = launch_empty(nullptr);
        return e ? hip_fail("empty kernel launch", (hipError_t)e) : CLG_OK;
    }, cost_ns);
}

int32_t profile_match(Context &ctx, Graph &g, int32_t match, const clg_profile_opts *opts, int64_t *cost_ns, bool *fresh,
                      bool again) {
    if (fresh) *fresh = false;
    if (ctx.device < 0) return fail(CLG_HIP_ERROR, "host-only context: no device to profile on");
    if (!g.matched) return fail(CLG_INVALID_ARG, "clg_match_all has not been called on this graph");
    const Opts o = resolve(opts);
    KernelCall c;
    const int32_t lrc = lower_match(ctx, g, match, &c);
    if (lrc == CLG_NO_KERNEL) {
        *cost_ns = CLG_COST_INF;
        return CLG_OK;
    }
    if (lrc != CLG_OK) return lrc;
    if (o.cache && !again) {
        auto it = ctx.cost_log.find(c.key);
        if (it != ctx.cost_log.end()) {
            *cost_ns = it->second;
            return CLG_OK;
        }
    }
    // operands: small constants in place; inputs, output, scratch and the large constant operand (the
    // weights, packed or plain) in R rotating copies inside one scratch block
    std::vector<int32_t> vals;
    for (int32_t v : {c.a_node, c.b_node, c.c_node}) vals.push_back(v);
    for (int32_t v : c.epi_nodes) vals.push_back(v);
    vals.push_back(c.out_node);
    const size_t nv = vals.size();
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    constexpr size_t kRotateBytes = (size_t)64 << 20, kBigConst = (size_t)256 << 10;
    std::vector<size_t> offs(nv, 0);
    std::vector<char> rotated(nv, 0);
    size_t set_bytes = 0;
    for (size_t i = 0; i < nv; ++i) {
        const int32_t v = vals[i];
        if (v < 0) continue;
        const bool is_out = i + 1 == nv;
        const size_t bytes = 4 * (size_t)g.nodes[v].shape.numel();
        if (!is_out && g.nodes[v].kind == NODE_CONST) {
            if (!g.nodes[v].dev_ptr) return fail(CLG_INVALID_ARG, "constant node %d has no device pointer", v);
            // the weights a kernel reads in place get copies too; packed ones are copied as packed (below);
            // a gather's table is not read as a whole and stays where it is
            const bool table = (c.kind == CALL_ELTWISE && c.elt.table_rows > 0 && i == 0) || (c.kind == CALL_ROWWISE && c.row.n_gather);
            if (i != 1 || c.pack_bytes || bytes < kBigConst || table) continue;
        }
        rotated[i] = 1;
        offs[i] = set_bytes;
        set_bytes += up(bytes);
    }
    const size_t scratch_off = set_bytes;
    set_bytes += up(c.scratch_bytes);
    const size_t pack_off = set_bytes;
    set_bytes += up(c.pack_bytes);
    set_bytes = std::max<size_t>(set_bytes, 256);
    const int R = (int)std::min<size_t>(32, std::max<size_t>(1, (kRotateBytes + set_bytes - 1) / set_bytes));
    int32_t rc = ensure_block(ctx, set_bytes * (size_t)R);
    if (rc != CLG_OK) return rc;
    char *base = (char *)ctx.prof_ptr;
    if (c.pack_bytes && g.nodes[c.b_node].kind != NODE_CONST) return fail(CLG_INVALID_ARG, "packed weights must be a constant");
    for (int r = 0; r < R; ++r) {
        char *set = base + (size_t)r * set_bytes;
        for (size_t i = 0; i < nv; ++i) {
            const int32_t v = vals[i];
            if (v < 0 || !rotated[i] || i + 1 == nv) continue;
            const int64_t n = g.nodes[v].shape.numel();
            if (g.nodes[v].kind == NODE_CONST) {
                const hipError_t he = hipMemcpyAsync(set + offs[i], g.nodes[v].dev_ptr, 4 * (size_t)n, hipMemcpyDeviceToDevice, nullptr);
                if (he != hipSuccess) return hip_fail("copy of a constant operand", he);
            } else if (g.nodes[v].dtype == CLG_I32) {
                // the only int32 operand is a gather's row ids: seeded ids spread over the table (all zeros would
                // time the gather of one cache-hot row)
                int32_t rows = c.kind == CALL_ELTWISE && c.elt.table_rows > 0 ? c.elt.table_rows : 1;
                if (c.kind == CALL_ROWWISE && c.row.n_gather && i >= 6 && i < 9) rows = c.row.tab_rows[i - 6];
                const int e = launch_fill_ids((int32_t *)(set + offs[i]), n, rows, o.seed + 7919u * (uint64_t)i + 104729u * (uint64_t)r, nullptr);
                if (e) return hip_fail("id fill kernel", (hipError_t)e);
            } else {
                const int e = launch_fill((float *)(set + offs[i]), n, o.seed + 7919u * (uint64_t)i, nullptr);
                if (e) return hip_fail("fill kernel", (hipError_t)e);
            }
        }
        if (c.pack_bytes) {                  // one-time weight re-packing is not part of the measured cost
            rc = pack_weights(c, g.nodes[c.b_node].dev_ptr, set + pack_off, nullptr);
            if (rc != CLG_OK) return rc;
        }
    }
    rc = time_launches(o, [&](int launch_no) -> int32_t {
        char *set = base + (size_t)(launch_no % R) * set_bytes;
        const void *ptrs[3 + kMaxEpi + 1];
        for (size_t i = 0; i < nv; ++i)
            ptrs[i] = vals[i] < 0 ? nullptr : (rotated[i] ? (const void *)(set + offs[i]) : g.nodes[vals[i]].dev_ptr);
        return launch_call(c, ptrs[0], ptrs[1], ptrs[2], const_cast<void *>(ptrs[nv - 1]), ptrs + 3,
                           c.scratch_bytes ? set + scratch_off : nullptr, c.pack_bytes ? set + pack_off : nullptr, nullptr);
    }, cost_ns);
    if (rc != CLG_OK) return rc;
    if (fresh) *fresh = true;
    if (o.cache) {
        auto it = ctx.cost_log.find(c.key);
        if (again && it != ctx.cost_log.end()) *cost_ns = std::min(*cost_ns, it->second);
        ctx.cost_log[c.key] = *cost_ns;
    }
    return CLG_OK;
}

int32_t cost_log_load(Context &ctx, const char *path) {
    std::ifstream f(path);
    if (!f) return fail(CLG_IO_ERROR, "cannot open %s", path);
    std::string line;
    size_t lineno = 0;
    while (std::getline(f, line)) {
        ++lineno;
        if (line.empty() || line[0] == '#') continue;
        const size_t tab = line.rfind('\t');
        if (tab == std::string::npos) return fail(CLG_IO_ERROR, "%s:%zu: no tab", path, lineno);
        char *end = nullptr;
        const long long v = std::strtoll(line.c_str() + tab + 1, &end, 10);
        if (end == line.c_str() + tab + 1 || v < 0) return fail(CLG_IO_ERROR, "%s:%zu: bad cost", path, lineno);
        ctx.cost_log[line.substr(0, tab)] = (int64_t)v;
    }
    return CLG_OK;
}

int32_t cost_log_save(const Context &ctx, const char *path) {
    std::ofstream f(path);
    if (!f) return fail(CLG_IO_ERROR, "cannot open %s for writing", path);
    f << "# fused-kernel cost log: key<TAB>nanoseconds per launch\n";
    for (auto &kv : ctx.cost_log) f << kv.first << '\t' << kv.second << '\n';
    f.flush();
    if (!f) return fail(CLG_IO_ERROR, "write to %s failed", path);
    return CLG_OK;
}

}  // namespace clg
