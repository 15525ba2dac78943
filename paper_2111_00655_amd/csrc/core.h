// Internal data structures of the host side: graph G, registry B, matches,
// lowered kernel calls and plans.  Nothing here crosses the C ABI.
#pragma once

#include <cstdint>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "../../include/collage_mi.h"
#include "kernels.h"

namespace clg {

// ---- errors -------------------------------------------------------------------
// Records the message for clg_last_error() and returns `code`.
int32_t fail(int32_t code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void set_error(const char *msg);

// ---- graph -----------------------------------------------------------------------
enum NodeKind : int32_t { NODE_INPUT = -3, NODE_CONST = -2 };   // else clg_op_kind

// Largest tensor the library takes: the kernels index with 32-bit element and byte offsets.
constexpr int64_t kMaxTensorElems = (int64_t)1 << 29;

struct Shape {
    int32_t ndim = 0;
    int64_t d[CLG_MAX_DIMS] = {0, 0, 0, 0, 0, 0};
    // Element count; saturates just above kMaxTensorElems so that absurd extents cannot wrap around.
    int64_t numel() const {
        int64_t n = 1;
        for (int i = 0; i < ndim; ++i) {
            if (d[i] <= 0) return 0;
            if (d[i] > kMaxTensorElems || n * d[i] > kMaxTensorElems) return kMaxTensorElems + 1;
            n *= d[i];
        }
        return n;
    }
    bool operator==(const Shape &o) const {
        if (ndim != o.ndim) return false;
        for (int i = 0; i < ndim; ++i)
            if (d[i] != o.d[i]) return false;
        return true;
    }
    std::string str() const;
};

struct Node {
    int32_t kind = 0;                 // NODE_INPUT, NODE_CONST or clg_op_kind
    std::vector<int32_t> in;
    clg_attrs attrs{};
    Shape shape;
    int32_t dtype = CLG_F32;
    const void *dev_ptr = nullptr;    // constants only (borrowed)
    int32_t input_index = -1;         // inputs: position in the inputs[] array
    bool is_op() const { return kind >= 0; }
};

struct MatchRec {
    int32_t pattern = 0, backend = 0, first = 0, sink = 0;
    std::vector<int32_t> nodes;       // ascending node id
    std::vector<int32_t> binding;     // op pattern nodes in pattern order
    std::vector<int32_t> wild;        // graph value bound to each pattern node
                                      // (all pattern nodes, wildcards included)
};

struct Context;

struct Graph {
    Context *ctx = nullptr;
    std::vector<Node> nodes;
    std::vector<int32_t> outputs;
    int32_t n_inputs = 0;
    // derived (rebuilt lazily by finalize())
    bool finalized = false;
    std::vector<std::vector<int32_t>> consumers;
    std::vector<int32_t> depth;
    std::vector<int32_t> op_ids;      // operator nodes by ascending id
    std::vector<int32_t> order;       // operator nodes sorted by (depth, id)
    std::vector<int32_t> rank;        // node -> position in order, -1 for leaves
    std::vector<char> is_output;
    // last enumeration / search
    std::vector<MatchRec> matches;
    bool matched = false;
    int64_t stats[5] = {0, 0, 0, 0, 0};
    int32_t live_plans = 0;           // compiled plans that still refer to this graph
    void finalize();
};

// ---- registry ------------------------------------------------------------------------
enum Family : int32_t { FAM_IGEMM = 0, FAM_DIRECT = 1, FAM_ROWWISE = 2, FAM_ELTWISE = 3, FAM_SEPCONV = 4,
                        FAM_ATTENTION = 5 };

struct Backend {
    std::string name;
    int32_t family = 0;
    int32_t tile = 0;                 // igemm: GemmTile
    int32_t no_split = 0;             // igemm: 1 = never split K across workgroups
    int32_t rf_waves = 0;             // register-fed kernels: at most this many K-waves per workgroup (0: one chunk per wave)
};

struct Pattern {
    int32_t backend = 0;
    std::vector<clg_pattern_node> nodes;   // post-order, root last
    // chain view, computed at registration: chain[0] = anchor ... back() = root;
    // main_arg[t] = which argument of chain[t] holds chain[t-1] (-1 for the anchor)
    std::vector<int32_t> chain;
    std::vector<int32_t> main_arg;
    // the one tree-shaped fused kind: layer_norm(add(add(take, take), take), *, *) - an embedding's rows
    // gathered, summed and normalised in one kernel; gather[k] = pattern node of the k-th take, in the
    // order the sums are taken ((0 + 1) + 2)
    std::vector<int32_t> gather;
};

struct Context {
    int32_t device = -1;
    std::vector<Backend> backends;
    std::vector<Pattern> patterns;
    std::map<std::string, int64_t> cost_log;
    int32_t n_cus = 256;
    void *prof_ptr = nullptr;         // measurer's scratch operands (device)
    size_t prof_bytes = 0;
};

// ---- lowering: one match -> one kernel call -------------------------------------------
// Where an operand pointer comes from at execution time.
struct Operand {
    int32_t node = -1;                // graph value
};

enum CallKind : int32_t {
    CALL_GEMM = 0, CALL_DIRECT_CONV, CALL_POOL, CALL_GAP, CALL_ROWWISE,
    CALL_ELTWISE, CALL_LAYOUT, CALL_CONCAT, CALL_SEPCONV, CALL_ATTENTION
};

struct KernelCall {
    int32_t kind = 0;
    int32_t match = -1;
    std::string name;
    std::string key;                  // cost-log key: backend|fused kind|attrs|shapes
    double flops = 0, bytes = 0;
    int32_t bound = 1;                // 0 MFMA, 1 HBM
    size_t scratch_bytes = 0;         // per-call device scratch (split-K partials)
    bool gemm_swap = false;           // GEMM: A = second graph operand (weights), B = first
    size_t pack_bytes = 0;            // register-fed conv: size of the re-packed copy of the weights (b_node)
    int32_t out_node = -1;
    // pointer slots to fill at execution: each refers to a graph value
    int32_t a_node = -1, b_node = -1, c_node = -1;     // main operands
    int32_t epi_nodes[kMaxEpi];                        // operand of each epilogue step or -1
    // kernel arguments with the pointer fields still null
    GemmArgs gemm{};
    DirectConvArgs dconv{};
    PoolArgs pool{};
    RowwiseArgs row{};
    EltwiseArgs elt{};
    LayoutArgs layout{};
    ConcatArgs cat{};                                  // operands in epi_nodes[0..n)
    AttentionArgs att{};                               // a = q, b = k, c = v
    SepConvArgs sep{};                                 // a = x, b = 1x1 weights (packed by the plan), c = depthwise weights
    KernelCall() { for (auto &e : epi_nodes) e = -1; }
};

// Builds the kernel call of match `m`.  Returns CLG_OK, or CLG_NO_KERNEL (with
// a message) when the backend's family cannot run this match.
int32_t lower_match(const Context &ctx, const Graph &g, int32_t match_id, KernelCall *out);
// Structure check at registration time.
int32_t check_pattern(const Context &ctx, Pattern *p);
// Pattern generator (rules.cpp).
int32_t generate_patterns(Context &ctx, Graph &g, int32_t backend, const clg_pattern_rule &rule, int32_t *n_added);

// ---- plan -----------------------------------------------------------------------------
// A region: kernels of the plan that do not depend on each other and run the same kind of
// register-fed kernel, so that those of them that are handed over (clg_plan_set_handover) can
// share one launch.  Members are adjacent in the plan's order.
struct Region {
    std::vector<int32_t> members;          // call indices, ascending
    std::vector<KernelCall> fused;         // per member: the call lowered again for the region's common kernel shape
    std::vector<void *> packed;            // per member: weights packed for that shape (owned by the plan)
};

struct Plan {
    Context *ctx = nullptr;
    Graph *graph = nullptr;            // read at every execution: the graph outlives its plans, unchanged
    bool counted = false;              // this plan is among graph->live_plans
    std::vector<KernelCall> calls;
    PlaneMultiArgs plane_args{};           // argument block of a region of thread-per-output kernels, refilled per launch
    std::vector<int64_t> value_offset;     // node -> workspace byte offset, -1 none
    std::vector<int32_t> value_output;     // node -> index in outputs[] of the buffer it lives in, -1 none
    std::vector<int64_t> value_delta;      // node -> byte offset inside that output buffer (a piece of a concatenation)
    std::vector<char> elided;              // call -> launches nothing (a concatenation whose operands are written in place)
    std::vector<int64_t> scratch_offset;   // call -> workspace byte offset of its scratch
    std::vector<void *> packed;            // call -> re-packed weights (device memory owned by the plan) or null
    std::vector<Region> regions;
    std::vector<int32_t> region_of;        // call -> index into regions, -1 none
    std::vector<char> fuse_mark;           // per call, scratch of an execution: 1 launched with its region, 2 carried its region
    size_t workspace_bytes = 0;
    // concurrent lanes: kernels of independent branches go to different HIP streams
    int32_t max_lanes = 1;                 // 1 = everything on the caller's stream (default: see clg_plan_set_lanes)
    int32_t n_lanes = 1;                   // lanes the schedule uses
    std::vector<char> handed;              // call -> the lane scheduler may move it off the caller's stream (empty: all)
    std::vector<int32_t> lane;             // call -> lane (0 = the caller's stream)
    std::vector<std::vector<int32_t>> waits;   // call -> earlier calls on other lanes it must wait for
    std::vector<char> signals;             // call -> some later call on another lane waits for it
    std::vector<void *> side_streams;      // hipStream_t of lanes 1.., created at the first execution
    std::vector<void *> events;            // hipEvent_t per call (null unless it signals)
    void *ev_begin = nullptr;
    std::vector<void *> ev_end;            // per side lane
    Plan() = default;
    Plan(const Plan &) = delete;
    Plan &operator=(const Plan &) = delete;
    ~Plan();
};

// `packed`: the re-packed weights when c.pack_bytes != 0 (see pack_weights), else ignored.
int32_t launch_call(const KernelCall &c, const void *a, const void *b, const void *c3,
                    void *out, const void *const *epi_ptrs, void *scratch, const void *packed, void *stream);
// The kernel arguments of a CALL_GEMM call with every pointer bound.
int32_t bind_gemm(const KernelCall &c, const void *a, const void *b, void *out, const void *const *epi_ptrs,
                  void *scratch, const void *packed, GemmArgs *k);
// Kernel-list entries that launch something under the plan's current digits (aliased concatenations
// launch nothing; the handed-over members of a region share one launch).
size_t plan_num_launches(const Plan &p);
// Runs the weight re-packing kernel of call `c` (c.pack_bytes != 0): w -> dst.
int32_t pack_weights(const KernelCall &c, const void *w, void *dst, void *stream);

// shape inference for one operator; returns CLG_OK or SHAPE_MISMATCH / INVALID_ARG
int32_t infer_shape(const Graph &g, int32_t kind, const std::vector<int32_t> &in,
                    const clg_attrs &a, Shape *out, int32_t *dtype);
int64_t attr_value(const Graph &g, int32_t node, int32_t attr, bool *ok);
const char *op_name(int32_t kind);

// Evolutionary search over digit strings (evolve.cpp); arguments as clg_evolve.
int32_t evolve(size_t n, const clg_es_opts &o, const uint32_t *rand, size_t n_rand, clg_fitness_fn fn, void *user,
               uint8_t *best, double *best_cost, int64_t *evaluations, double *history, int32_t *generations_run);

int32_t match_all(Context &ctx, Graph &g);
int32_t compile_plan(Context &ctx, Graph &g, const int32_t *ids, size_t n, Plan *plan);
// (Re)computes the lane schedule of a compiled plan for at most plan->max_lanes lanes.
void schedule_lanes(Plan *plan);
// Changes the lane limit: waits for the plan's own streams, releases them and their events, reschedules.
int32_t set_plan_lanes(Plan &p, int32_t lanes);
// Whole-sequence time: `warmup` executions, then `batches` batches of `reps` executions between two
// events on `stream`; *ns = the smallest batch mean.
int32_t measure_plan(Plan &p, const void *const *inputs, void *const *outputs, void *workspace, size_t ws_bytes,
                     void *stream, const clg_measure_opts &o, int64_t *ns);
int32_t execute_plan(Plan &p, const void *const *inputs, void *const *outputs, void *workspace,
                     size_t ws_bytes, void *stream, int64_t *kernel_ns);
// static_ws.hip: execution with the library's own fixed workspace (no allocation anywhere)
int32_t static_workspace_init(int32_t device);
int32_t execute_plan_static(Plan &p, const void *const *inputs, void *const *outputs, void *stream);
// fresh (may be null): set to whether this call measured (false: served from the cost log, or no kernel).
// again: measure even if the log has the key, and keep the smaller of the two figures.
int32_t profile_match(Context &ctx, Graph &g, int32_t match, const clg_profile_opts *opts, int64_t *cost_ns,
                      bool *fresh = nullptr, bool again = false);
int32_t profile_empty(Context &ctx, const clg_profile_opts *opts, int64_t *cost_ns);
int32_t cost_log_load(Context &ctx, const char *path);
int32_t cost_log_save(const Context &ctx, const char *path);
const char *last_error();
int32_t search_dp(Graph &g, size_t n_patterns, const int64_t *cost, int64_t eps,
                  std::vector<int32_t> *chosen, int64_t *total);

}  // namespace clg

struct clg_ctx { clg::Context c; };
struct clg_graph { clg::Graph g; };
struct clg_plan { clg::Plan p; };
