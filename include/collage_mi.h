/*
 * collage_mi.h - C ABI of the MI355X fused-operator inference library.
 *
 * The library runs batch-1 fp32 DNN inference as a sequence of fused operator
 * subgraphs, the computation whose backend placement the Collage paper
 * (arXiv 2111.00655) optimises.  The calls follow the paper's statement of
 * the problem (Sec. 4.1): a computation graph G, a registry B of backend
 * patterns b = (p, d), matches (g_i, b_i), a measurer M that times one
 * matched subgraph as one kernel (Sec. 4.2), the op-level dynamic programme
 * of Alg. 1, and execution of G under a placement P(G).
 *
 * Conventions
 *  - Every call returns a clg_status: 0 on success, negative on error.  No
 *    exception crosses this boundary.  clg_last_error() gives a message for
 *    the most recent failing call on the calling thread.
 *  - Handles (clg_ctx, clg_graph, clg_plan) are opaque, created and destroyed
 *    by the library.  A context and the objects made from it are not
 *    thread-safe.
 *  - "host" pointers are ordinary process memory; "device" pointers are HIP
 *    device memory on the context's GPU.  Device buffers are OWNED BY THE
 *    CALLER: the library borrows them and never frees them.  Constant
 *    tensors (weights) must stay valid and unchanged for as long as the
 *    graph, its plans or the profiler may read them.
 *  - All tensors are dense, row-major, fp32 (token ids: int32).  Activations
 *    are NCHW, convolution weights OIHW, transposed-convolution weights IOHW,
 *    dense weights [units, in].
 *  - Kernel launches go to the hipStream_t passed as `void *stream` (NULL =
 *    the default stream) and are asynchronous; profiling calls synchronise.
 *  - A context created with device = -1 is host-only: graph building,
 *    registration, matching, search and plan validation work; execution and
 *    profiling return CLG_HIP_ERROR.
 */
#ifndef COLLAGE_MI_H
#define COLLAGE_MI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct clg_ctx clg_ctx;
typedef struct clg_graph clg_graph;
typedef struct clg_plan clg_plan;

typedef enum clg_status {
    CLG_OK = 0,
    CLG_INVALID_ARG = -1,        /* null pointer, bad enum, bad count            */
    CLG_SHAPE_MISMATCH = -2,     /* operand shapes do not fit the operator       */
    CLG_NO_KERNEL = -3,          /* the backend cannot run this fused kind       */
    CLG_NOT_A_COVER = -4,        /* placement leaves an operator uncovered       */
    CLG_OVERLAP = -5,            /* two chosen matches share an operator         */
    CLG_UNKNOWN_ID = -6,         /* node / backend / pattern / match id          */
    CLG_WORKSPACE_TOO_SMALL = -7,
    CLG_HIP_ERROR = -8,          /* a HIP call failed, or no device in this ctx  */
    CLG_OUT_OF_MEMORY = -9,
    CLG_IO_ERROR = -10,          /* cost-log file                                */
    CLG_BUFFER_TOO_SMALL = -11   /* caller's output array has too few entries    */
} clg_status;

typedef enum clg_dtype { CLG_F32 = 0, CLG_I32 = 1 } clg_dtype;

/* Primitive operators: the operator inventory of the evaluated workloads
 * (Sec. 5.1: batch matmul, layer norm, softmax for transformers; convolutions
 * and activations for vision models).  Operand order is given per kind. */
typedef enum clg_op_kind {
    CLG_WILDCARD = -1,              /* pattern nodes only: matches any value      */
    CLG_OP_CONV2D = 0,              /* (x[N,C,H,W], w[O,C/G,kh,kw]); stride pad groups */
    CLG_OP_CONV2D_TRANSPOSE = 1,    /* (x[N,C,H,W], w[C,O,kh,kw]); stride pad     */
    CLG_OP_DENSE = 2,               /* (x[M,K], w[U,K]) -> [M,U]                  */
    CLG_OP_BATCH_MATMUL = 3,        /* (a[B,M,K], b[B,N,K] or b[B,K,N]); transpose_b */
    CLG_OP_BIAS_ADD = 4,            /* (x, b[C]); axis                            */
    CLG_OP_ADD = 5,                 /* (x, y), equal shapes                       */
    CLG_OP_MUL_SCALAR = 6,          /* (x); scalar                                */
    CLG_OP_RELU = 7,
    CLG_OP_GELU = 8,                /* x/2 (1 + erf(x / sqrt 2))                  */
    CLG_OP_TANH = 9,
    CLG_OP_SOFTMAX = 10,            /* last axis                                  */
    CLG_OP_LAYER_NORM = 11,         /* (x, gamma[L], beta[L]); eps; last axis     */
    CLG_OP_MAX_POOL2D = 12,         /* (x); kernel stride pad; padding = -inf     */
    CLG_OP_GLOBAL_AVG_POOL2D = 13,  /* (x[N,C,H,W]) -> [N,C]                      */
    CLG_OP_TAKE = 14,               /* (table[V,H], ids[L] int32) -> [L,H]; ids live in
                                       device memory, which no host call can inspect:
                                       an id outside [0, V) is not an error, the kernel
                                       reads row 0 or V-1 instead (it never reads
                                       outside the table)                         */
    CLG_OP_RESHAPE = 15,            /* (x); dims = new shape                      */
    CLG_OP_TRANSPOSE = 16,          /* (x); dims = permutation                    */
    CLG_OP_AVG_POOL2D = 17,         /* (x); kernel stride pad; mean over the window's
                                       pixels inside the image (padding not counted) */
    CLG_OP_CONCAT = 18,             /* (x0, x1, ...), 2..8 operands; axis         */
    CLG_OP_CONV3D = 19,             /* (x[N,C,D,H,W], w[O,C,kd,kh,kw]); stride pad, with
                                       stride_d pad_d for the depth axis             */
    CLG_OP_MAX_POOL3D = 20,         /* (x[N,C,D,H,W]); kernel stride pad + kernel_d
                                       stride_d pad_d; padding = -inf                */
    CLG_OP_GLOBAL_AVG_POOL3D = 21,  /* (x[N,C,D,H,W]) -> [N,C]                      */
    CLG_OP_COUNT = 22
} clg_op_kind;

#define CLG_MAX_DIMS 6

/* Operator attributes (Sec. 3: patterns may constrain attributes such as kernel size).
 * Fields an operator does not use are ignored.  Zero-initialise, then set. */
typedef struct clg_attrs {
    int32_t stride[2];      /* conv2d, conv2d_transpose, max/avg_pool2d       */
    int32_t pad[2];         /* same                                           */
    int32_t kernel[2];      /* max/avg_pool2d window                          */
    int32_t groups;         /* conv2d; 0 is read as 1                         */
    int32_t axis;           /* bias_add: 1 (channel of NCHW) or -1 / last;
                               concat: the axis joined (negative: from the end) */
    int32_t transpose_b;    /* batch_matmul: 1 = b is [B,N,K]                 */
    int32_t ndims;          /* reshape / transpose: entries used in dims      */
    int64_t dims[CLG_MAX_DIMS];
    double scalar;          /* mul_scalar                                     */
    double eps;             /* layer_norm                                     */
    int32_t stride_d;       /* conv3d, max_pool3d: the depth axis (stride, pad */
    int32_t pad_d;          /* and kernel hold the H and W entries)            */
    int32_t kernel_d;       /* max_pool3d window depth                         */
    int32_t reserved_;
} clg_attrs;

/* Attribute constraints of a pattern node (the has_attr of the paper's
 * pattern language, Sec. 3): lo <= value <= hi. */
typedef enum clg_attr_id {
    CLG_ATTR_GROUPS = 0, CLG_ATTR_KERNEL_H = 1, CLG_ATTR_KERNEL_W = 2,
    CLG_ATTR_STRIDE_H = 3, CLG_ATTR_STRIDE_W = 4, CLG_ATTR_PAD_H = 5,
    CLG_ATTR_PAD_W = 6, CLG_ATTR_TRANSPOSE_B = 7, CLG_ATTR_AXIS = 8,
    CLG_ATTR_COUNT = 9
} clg_attr_id;

typedef struct clg_attr_constraint {
    int32_t attr;           /* clg_attr_id */
    int64_t lo, hi;
} clg_attr_constraint;

#define CLG_MAX_PATTERN_ARGS 8
#define CLG_MAX_CONSTRAINTS 4
#define CLG_MAX_PATTERN_NODES 32
#define CLG_MAX_MATCH_NODES 16

/* One node of a pattern tree.  A pattern is an array of these in post-order:
 * every argument index refers to an EARLIER entry, each entry is used as an
 * argument at most once, and the last entry is the root (the sink of the
 * matched subgraph), as in is_op('relu')(is_op('add')(conv, wildcard())). */
typedef struct clg_pattern_node {
    int32_t op;                               /* clg_op_kind or CLG_WILDCARD  */
    int32_t n_args;                           /* 0 for a wildcard             */
    int32_t args[CLG_MAX_PATTERN_ARGS];
    int32_t n_constraints;
    clg_attr_constraint constraints[CLG_MAX_CONSTRAINTS];
} clg_pattern_node;

/* One match (v_s, b_i) -> g of Alg. 1.  `first` is v_s: the first node of g
 * in the order (depth, node id).  `nodes` lists g's operators by ascending
 * node id; `binding` gives the graph node bound to each NON-wildcard pattern
 * node, in pattern order (so its last entry is the sink). */
typedef struct clg_match {
    int32_t pattern;
    int32_t backend;
    int32_t first;
    int32_t sink;
    int32_t n_nodes;
    int32_t nodes[CLG_MAX_MATCH_NODES];
    int32_t binding[CLG_MAX_MATCH_NODES];
} clg_match;

/* Cost the measurer reports for a match its backend cannot run. */
#define CLG_COST_INF ((int64_t)1 << 60)

/* Measurer protocol (Sec. 4.2: a candidate is built and run several times on
 * the device).  Zero in a field selects the default given in brackets. */
typedef struct clg_profile_opts {
    int32_t warmup;         /* untimed launches first [20]                    */
    int32_t batches;        /* timed batches; the cost is the fastest one [7] */
    int32_t min_batch_us;   /* a batch repeats the kernel until it lasts this long [200] */
    int32_t max_launches;   /* cap on launches per batch [2000]               */
    uint64_t seed;          /* seed of the scratch operands' contents [1]     */
    int32_t no_cache;       /* 1: neither read nor fill the cost log [0]      */
} clg_profile_opts;

/* Per-kernel record of a compiled plan (for roofline accounting). */
typedef struct clg_kernel_info {
    char name[64];          /* kernel family and variant, NUL-terminated      */
    int32_t match;          /* match id this kernel belongs to                */
    int32_t bound;          /* 0 = MFMA contraction, 1 = HBM-bound            */
    double flops;           /* algorithmic: 2 * MACs of the real operator     */
    double bytes;           /* algorithmic: every operand and the output once */
} clg_kernel_info;

/* ---- context ------------------------------------------------------------ */
/* device >= 0: HIP device ordinal; -1: host-only context.  *out owns nothing
 * of the caller's.  Errors: INVALID_ARG, HIP_ERROR. */
int32_t clg_create(clg_ctx **out, int32_t device);
int32_t clg_destroy(clg_ctx *ctx);
/* Message of the last failing call on this thread; library-owned storage,
 * valid until the next failing call on the thread.  Never NULL. */
const char *clg_last_error(void);
/* ABI version of this header (major * 100 + minor).  101: clg_es_opts.seed_ones, regions (clg_plan_set_handover
 * with lanes = 1, clg_plan_num_launches, clg_plan_region_of), clg_execute_static, clg_plan_reads_constant.
 * 102 (no new symbol): backends igemm_r16_sk, igemm_r16_sk_w4, igemm_r32_sk; "direct" runs conv2d_transpose; regions
 * of thread-per-output kernels and of separable convolutions, register-fed regions of up to 8. */
int32_t clg_version(void);

/* ---- computation graph G (Sec. 4.1: a DAG of tensor operators) ------------ */
/* Nodes are added in topological order; a node's id is its insertion index
 * (returned in *node).  Shapes are inferred when an operator is added;
 * SHAPE_MISMATCH is returned, and the node not added, if operands do not fit.
 * No tensor may hold more than 2^29 elements (2 GiB of fp32): the kernels
 * index with 32-bit element and byte offsets.  A larger input or constant is
 * INVALID_ARG, a larger operator result SHAPE_MISMATCH.
 * A compiled plan refers to its graph at every execution: while a graph has
 * plans (clg_compile .. clg_plan_destroy) it can neither be destroyed nor
 * changed (clg_graph_destroy, clg_graph_input / _const / _op / _mark_output
 * then return INVALID_ARG). */
int32_t clg_graph_create(clg_ctx *ctx, clg_graph **out);
int32_t clg_graph_destroy(clg_graph *g);
/* A run-time input.  dims: host array of ndim entries (1..CLG_MAX_DIMS). */
int32_t clg_graph_input(clg_graph *g, int32_t dtype, int32_t ndim,
                        const int64_t *dims, int32_t *node);
/* A constant (weight).  dev_ptr: device memory holding the tensor, borrowed
 * for the life of the graph and its plans; may be NULL in a host-only ctx. */
int32_t clg_graph_const(clg_graph *g, int32_t dtype, int32_t ndim,
                        const int64_t *dims, const void *dev_ptr, int32_t *node);
/* An operator.  in_nodes: host array of n_in earlier node ids; attrs: host,
 * may be NULL for operators without attributes. */
int32_t clg_graph_op(clg_graph *g, int32_t op_kind, int32_t n_in,
                     const int32_t *in_nodes, const clg_attrs *attrs,
                     int32_t *node);
/* Marks an operator's value as a graph output; outputs keep call order. */
int32_t clg_graph_mark_output(clg_graph *g, int32_t node);
int32_t clg_graph_num_nodes(const clg_graph *g, int32_t *n);
/* Shape of any node: dims receives up to CLG_MAX_DIMS entries. */
int32_t clg_graph_node_shape(const clg_graph *g, int32_t node, int32_t *dtype,
                             int32_t *ndim, int64_t *dims);

/* ---- registry B (Sec. 3 explicit pattern specification; Sec. 4.1) -------- */
/* A backend here is one of the library's kernel families, selected by name:
 *   "igemm"    MFMA implicit-GEMM convolution / GEMM, default tile choice
 *   "igemm_s", "igemm_s8", "igemm_s16", "igemm_m", "igemm_l"   the same with a
 *              fixed tile: 32x32 outputs with 4 / 8 / 16 waves sharing K, 64x64,
 *              128x128 (kernel variants for the search to place per layer)
 *   "igemm_s_nk", "igemm_s8_nk", "igemm_s16_nk"   those tiles, never splitting
 *              K across workgroups (no second reduction kernel)
 *   "igemm_r32", "igemm_r16"   register-fed MFMA kernels with 32x32 / 16x16
 *              output tiles for conv2d (any groups), conv2d_transpose and dense
 *              whose weights are constants: the weights are re-packed once per
 *              plan and read straight into MFMA operands, K is split across the
 *              waves of a workgroup.  What they do not run (batch_matmul,
 *              non-constant weights, tails outside scale/bias/add/activation)
 *              falls back to the "igemm_s8" kernels.
 *   "igemm_r32_w4", "igemm_r32_w8", "igemm_r16_w4", "igemm_r16_w8"   the same
 *              kernels with at most 4 / 8 waves per workgroup sharing K: a wave
 *              then owns several chunks of MFMAs and keeps the loads of up to
 *              four of them in flight at once (fewer waves to dispatch and to
 *              meet, longer MFMA chains per wave); "igemm_r32" / "igemm_r16"
 *              give every wave one chunk (up to 16 waves)
 *   "igemm_r16_sk", "igemm_r16_sk_w4", "igemm_r32_sk"   the register-fed
 *              convolution kernels (conv2d with one group, conv3d) with the
 *              reduction also cut across workgroups where the output has so
 *              few tiles that most of the chip would idle (a long K over a
 *              few pixels): partial tiles go to the plan's workspace and a
 *              second kernel adds them in slice order and applies the tail;
 *              _w4: at most 4 waves per workgroup share K, so more workgroups
 *   "igemm_r16x2_w4", "igemm_r16x2_w8"   dense only: a wave owns two 16x16
 *              tiles (32 output columns, 16 rows) that share the activation
 *              operand, so that each value loaded and shuffled feeds two MFMAs
 *              (other operators registered under these names run as under
 *              "igemm_r16_w4" / "_w8")
 *   "sepconv"  separable convolution in one kernel: [relu] -> depthwise
 *              conv2d -> 1x1 conv2d -> elementwise tail, or relu -> 1x1 conv2d
 *              (any stride) -> tail; both weights constants, the depthwise
 *              result stays in LDS, the 1x1 weights are re-packed per plan
 *   "attention"  softmax(scale q k^T) v per head in one kernel: batch_matmul
 *              -> [mul_scalar] -> softmax -> batch_matmul [-> transpose ->
 *              reshape that puts the heads side by side]; head sizes 32, 64,
 *              128, up to 512 keys; the scores never leave the chip
 *   "direct"   direct convolution (any groups), transposed convolution of any
 *              filter size, stride and pad (the MFMA kernels take those whose
 *              filter and output sizes the stride divides), max / average
 *              pooling (window pools also with an elementwise tail), global
 *              average pooling
 *   "rowwise"  softmax and layer norm with fused elementwise prologue; also
 *              layer_norm(add(add(take, take), take), gamma, beta) and the
 *              two-table form: an embedding's rows gathered, summed and
 *              normalised in one kernel (row length a multiple of 4, 64..2048)
 *   "eltwise"  elementwise chains, embedding gather, layout copies, concat
 * Returns UNKNOWN_ID for any other name.  Registering a name twice returns
 * the same id.  Registration order of patterns is significant: it is the
 * iteration order of B in Alg. 1 and breaks ties in the search. */
int32_t clg_register_backend(clg_ctx *ctx, const char *name, int32_t *backend);
/* nodes: host array of n pattern nodes in post-order (see clg_pattern_node).
 * NO_KERNEL if the backend has no kernel for that fused kind (checked on the
 * pattern's structure; a match whose shapes the kernel cannot take is instead
 * reported by the measurer as CLG_COST_INF). */
int32_t clg_register_pattern(clg_ctx *ctx, int32_t backend,
                             const clg_pattern_node *nodes, int32_t n,
                             int32_t *pattern);
int32_t clg_num_patterns(const clg_ctx *ctx, int32_t *n);
/* Reads a registered pattern back: its backend and its nodes (post-order, as
 * given to clg_register_pattern).  nodes: host array of cap entries, may be
 * NULL when cap = 0 (count only); *n receives the node count.  UNKNOWN_ID,
 * INVALID_ARG if cap is too small. */
int32_t clg_get_pattern(const clg_ctx *ctx, int32_t pattern, int32_t *backend,
                        clg_pattern_node *nodes, int32_t cap, int32_t *n);

/* ---- pattern rules (Sec. 3: "pattern rule", automatic pattern generator) --- */
/* The second way to describe a backend: instead of listing patterns, say which
 * operators the backend runs and what it fuses; the generator then finds every
 * legitimate pattern on a given graph and adds it to the registry.
 * op_class[kind]: CLG_RULE_NONE (not run), CLG_RULE_FUSABLE (may seed a group
 * that absorbs the element-wise operators after it: convolutions, matrix
 * products) or CLG_RULE_ELEMWISE (may be absorbed; seeds a group of its own,
 * which grows only if grow_from_elemwise is set).  max_ops bounds a group
 * (1 .. CLG_MAX_MATCH_NODES). */
#define CLG_RULE_NONE 0
#define CLG_RULE_FUSABLE 1
#define CLG_RULE_ELEMWISE 2
typedef struct clg_pattern_rule {
    int32_t op_class[CLG_OP_COUNT];
    int32_t max_ops;
    int32_t grow_from_elemwise;
} clg_pattern_rule;
/* Visits the operators of g in node order.  For an operator the rule runs, its
 * own pattern (all operands wildcards) is registered for `backend`; then the
 * group is widened one operator at a time - the sink's only consumer, if it is
 * element-wise, uses the sink once, and the sink is not a graph output (a
 * group becomes one kernel with a single exit) - registering the chain pattern
 * after every step (other operands: wildcards).  Patterns this backend already
 * has are not registered twice; patterns the backend's kernel family cannot
 * run are skipped.  New patterns are appended to the registry in the order
 * found; *n_added (may be NULL) receives their number.  Matches of g have to
 * be enumerated again afterwards. */
int32_t clg_generate_patterns(clg_ctx *ctx, clg_graph *g, int32_t backend,
                              const clg_pattern_rule *rule, int32_t *n_added);

/* ---- matches (Alg. 1, matching step: the subgraph g at v_s for entry b_i) -- */
/* Enumerates every legal match of every registered pattern.  Legal: pattern
 * operators bind distinct nodes, only the sink has consumers outside g, and no
 * non-sink node is a graph output (g becomes ONE kernel).  `add` operands are
 * tried as written, then swapped.  At most one match per (v_s, pattern) is
 * kept: the first found scanning sinks in node order.  The list is sorted by
 * (order of v_s, pattern id); a match id is its index in this list.  The
 * result is stored in the graph and replaces any earlier one.
 * out: host array of cap entries, may be NULL when cap = 0 (count only);
 * *n receives the number of matches; BUFFER_TOO_SMALL if cap < *n > 0. */
int32_t clg_match_all(clg_ctx *ctx, clg_graph *g, clg_match *out, size_t cap,
                      size_t *n);

/* ---- measurer M (Sec. 4.2) -------------------------------------------------- */
/* Times one match as one kernel on the device and returns integer nanoseconds
 * per launch (fastest of several batches of back-to-back launches between two
 * HIP events, after warm-up).  Non-constant operands are scratch tensors the
 * library allocates and fills from opts->seed (row ids of a gather: seeded ids
 * spread over the table); small constants are read in place.  The large
 * operands - inputs, output, weights - exist in several copies (64 MB in all,
 * at most 32) and consecutive launches rotate through them, so that every
 * launch finds its operands in the memory-side cache and not in the L2, as a
 * kernel does inside a network (the library's scratch block grows to hold the
 * copies; weight re-packing for the copies is not part of the cost).
 * Results are cached by (backend, fused kind, attributes, shapes): the cost
 * log.  opts may be NULL (all defaults, cache on).  Synchronises the device.
 * A match the backend cannot run costs CLG_COST_INF. */
int32_t clg_profile_match(clg_ctx *ctx, clg_graph *g, int32_t match,
                          const clg_profile_opts *opts, int64_t *cost_ns);
/* cost_ns: host array with one entry per match of the last clg_match_all.
 * With the cost log on, every kernel this call has to measure is measured
 * twice, in two passes over the matches, and the smaller figure is kept (a
 * whole measurement is now and then inflated by the device's clocks). */
int32_t clg_profile_all(clg_ctx *ctx, clg_graph *g,
                        const clg_profile_opts *opts, int64_t *cost_ns,
                        size_t cap);
/* Cost of launching an empty kernel with the same protocol: the per-kernel
 * dispatch floor (the context-switch cost eps of Eq. 2, for reference). */
int32_t clg_profile_empty(clg_ctx *ctx, const clg_profile_opts *opts,
                          int64_t *cost_ns);
/* Cost log as a text file (Sec. 4.2: measured costs are kept in a log and reused):
 * one "key<TAB>nanoseconds" line per entry.  load merges into the context's
 * log (file entries win); save writes the whole log. */
int32_t clg_cost_log_load(clg_ctx *ctx, const char *path);
int32_t clg_cost_log_save(const clg_ctx *ctx, const char *path);
int32_t clg_cost_log_size(const clg_ctx *ctx, size_t *n);
/* Cache key of a match, for inspection; buf: host, cap bytes. */
int32_t clg_match_key(clg_ctx *ctx, clg_graph *g, int32_t match, char *buf,
                      size_t cap);

/* ---- op-level placement search (Sec. 4.2, Eq. 3 and Alg. 1) -------------- */
/* Minimises sum_i (cost_ns[m_i] + eps_ns) over all placements (disjoint
 * matches covering every operator).  A pure function of the graph, the match
 * list and the numbers given: ties are broken towards the lexicographically
 * smallest ascending match-id list, so equal cost tables give identical
 * placements.  Entries >= CLG_COST_INF are never chosen.
 * cost_ns: host, one entry per match.  chosen: host array of cap entries that
 * receives the chosen match ids, ascending; *n_chosen their count; *total_ns
 * the minimum.  NOT_A_COVER if no placement exists. */
int32_t clg_search_dp(clg_ctx *ctx, clg_graph *g, const int64_t *cost_ns,
                      size_t n_costs, int64_t eps_ns, int32_t *chosen,
                      size_t cap, size_t *n_chosen, int64_t *total_ns);
/* ---- graph-level placement search (Sec. 4.3) ------------------------------ */
/* Evolutionary search over strings of n digits.  Digit i = 0 keeps the
 * op-level decision for item i, 1 hands item i to the graph-level backend;
 * what an item is and what the handing-over does is the fitness function's
 * business (clg_search_graph_level below supplies the library's own).  fitness
 * returns the cost of a string measured on the whole graph (lower is better;
 * NaN aborts the search with INVALID_ARG); it is called once per distinct
 * string, from the calling thread.
 * The population is the all-zero string (the op-level placement, the seed the
 * paper names) plus population-1 strings whose digits are 1 with probability
 * p_init; with seed_ones the first of those is instead the all-ones string, a
 * second seed from the other end of the search space.  One generation: every string mutates
 * with probability p_mutate (each digit then flips with probability p_flip);
 * `population` tournaments of `tournament` entrants drawn with replacement
 * choose the next population (an entrant wins only when strictly cheaper);
 * neighbours (0,1), (2,3).. swap, with probability p_cross, the digits between
 * two cut points drawn from 0..n; the new strings are measured.  The search
 * ends after `generations` generations, or after `patience` (> 0) generations
 * in a row without a new best.  The result is the cheapest string ever
 * measured (the earliest among equals), so it never costs more than the seed.
 * Randomness: rand is a host array of n_rand 32-bit draws consumed in order;
 * probability p happens when draw / 2^32 < p, an index below m is
 * (draw * m) >> 32.  Equal draws and an equal fitness function give equal
 * results.  INVALID_ARG when the draws run out (a generation uses at most
 * population * (n + 1 + tournament) + 3 * (population / 2) of them, the initial
 * population (population - 1) * n).
 * best: host, n bytes.  history (may be null): host, generations + 1 doubles,
 * history[g] = best cost after g generations.  evaluations, generations_run
 * (may be null): distinct strings measured, generations done. */
typedef double (*clg_fitness_fn)(const uint8_t *digits, size_t n, void *user);
typedef struct clg_es_opts {
    int32_t population;      /* >= 2                                  */
    int32_t generations;     /* >= 0                                  */
    int32_t tournament;      /* >= 1                                  */
    int32_t patience;        /* 0 = run all generations               */
    double p_init, p_mutate, p_flip, p_cross;   /* each in [0, 1]     */
    int32_t seed_ones;       /* 1: the second string of the first population is
                                all ones (everything handed over) instead of a
                                random one; needs population >= 2 and uses n
                                fewer draws                                   */
    int32_t reserved_;
} clg_es_opts;
int32_t clg_evolve(size_t n, const clg_es_opts *opts, const uint32_t *rand,
                   size_t n_rand, clg_fitness_fn fitness, void *user,
                   uint8_t *best, double *best_cost, int64_t *evaluations,
                   double *history, int32_t *generations_run);

/* The library's own graph-level backends work on a compiled op-level plan: an
 * item is one kernel of the plan, digit 0 keeps it exactly as the op-level
 * search placed it, digit 1 hands it over.  What a handed-over kernel gains or
 * loses depends on which of its neighbours are handed over as well (the cost
 * is not a sum over digits), so strings are priced by timing the whole
 * sequence.  Two backends, selected by `lanes`:
 *  lanes = 1  REGIONS (the paper's cross-kernel optimisation, Sec. 4.3, with
 *    our own kernels).  clg_compile groups kernels that do not depend on each
 *    other and run the same kind of kernel into regions: register-fed MFMA
 *    kernels (dense layers with constant weights; 1x1 convolutions; at most 8
 *    per region), e.g. the query, key and value projections of an attention
 *    layer, or the projection shortcut and the first 1x1 convolution of a
 *    residual block; thread-per-output kernels (depthwise 3x3 / 5x5 / 7x7
 *    convolutions, window pools, with their fused tails; at most 8 per region)
 *    and one-kernel separable convolutions of one filter size and workgroup
 *    size (at most 4), e.g. the branches of a NasNet cell; the latter two
 *    kinds run unchanged inside a region, bit for bit.  The
 *    handed-over members of a region, if there are two or more, run as ONE
 *    launch of a kernel that works on several problems at once (all members in
 *    one common tile shape, that of the member with the most flops; members
 *    that needed another shape get a second packed copy of their weights at
 *    compile time).  A handed-over kernel without a handed-over sibling runs
 *    as before.  Results agree with the op-level plan's to rounding (another
 *    tile shape adds in another order), not bit for bit.  The workspace size
 *    does not depend on the digits.  clg_plan_region_of tells which region a
 *    kernel belongs to (-1: none), clg_plan_num_launches how many launches
 *    one execution makes under the current digits.
 *  lanes = 2..4  the LANE SCHEDULER (see clg_plan_set_lanes): a handed-over
 *    kernel may run on another HIP stream beside independent kernels, the
 *    others stay in place on the caller's stream.  Results are bit for bit
 *    those of the op-level plan.
 * clg_plan_set_handover: digits: host, n = clg_plan_num_kernels bytes (0/1).
 * All zeros = the op-level plan.
 * Waits for the plan's streams; not to be called while the plan executes.
 * clg_plan_measure: time of one clg_execute in ns: opts->warmup executions,
 * then opts->batches (>= 1) batches of opts->reps (>= 1) executions between
 * two events on `stream`; the smallest batch mean.  Arguments as clg_execute;
 * blocks until done.
 * clg_search_graph_level: clg_evolve over the plan's kernels with that
 * measurement as the fitness; every distinct string is set, timed and kept
 * (with lanes = 1, strings that give the same launches, i.e. that differ only
 * in digits of kernels outside regions or alone in theirs, are timed once and
 * share the figure).
 * best: host, clg_plan_num_kernels bytes; *best_ns its time; *seed_ns (may be
 * null) the time of the all-zero string, i.e. of the op-level placement, so
 * *best_ns <= *seed_ns.  On return the plan is set to `best`; after an error
 * it is set to all zeros (the op-level plan).  evaluations, history,
 * generations_run as in clg_evolve (history in ns). */
typedef struct clg_measure_opts {
    int32_t warmup, batches, reps;
} clg_measure_opts;
int32_t clg_plan_set_handover(clg_plan *plan, const uint8_t *digits, size_t n,
                              int32_t lanes);
int32_t clg_plan_measure(clg_plan *plan, const void *const *inputs,
                         void *const *outputs, void *workspace,
                         size_t workspace_bytes, void *stream,
                         const clg_measure_opts *opts, int64_t *ns);
int32_t clg_plan_num_launches(const clg_plan *plan, size_t *n);
int32_t clg_plan_region_of(const clg_plan *plan, size_t index, int32_t *region);
int32_t clg_search_graph_level(clg_plan *plan, const void *const *inputs,
                               void *const *outputs, void *workspace,
                               size_t workspace_bytes, void *stream,
                               int32_t lanes, const clg_es_opts *opts,
                               const uint32_t *rand, size_t n_rand,
                               const clg_measure_opts *measure, uint8_t *best,
                               int64_t *best_ns, int64_t *seed_ns,
                               int64_t *evaluations, double *history,
                               int32_t *generations_run);

/* Sizes of the last search on this graph: operators N, most matches at one
 * frontier P, most new frontiers from one match F, largest relaxed set S, and
 * the number of stored sub-placements. */
int32_t clg_search_stats(const clg_graph *g, int64_t stats[5]);

/* ---- compile under a GIVEN placement and execute (Sec. 4.1, Sec. 5.1) ------- */
/* matches: host array of n match ids (any valid placement, not only the
 * search's).  Validates disjointness and cover (OVERLAP, NOT_A_COVER,
 * UNKNOWN_ID), orders the groups topologically, lowers each to one kernel
 * (NO_KERNEL if a backend cannot run its match) and plans the intermediate
 * tensors in one workspace; tensors pass between kernels by pointer.
 * Kernels that read packed weights get their copy here: the plan allocates
 * device memory for it (OUT_OF_MEMORY on failure), fills it on the null
 * stream and waits for that; the constants' device pointers must therefore
 * be valid at this call.  clg_plan_destroy frees those copies; the plan must
 * not be destroyed while one of its executions is still running.
 * A concat whose operands are contiguous pieces of its result (all extents
 * before the axis are 1) costs nothing at run time when every operand is the
 * result of a kernel of this plan, is not a graph output, belongs to no other
 * such concat and starts on a 16-byte boundary: the producers write into the
 * result directly and the concat stays in the kernel list as an entry that
 * launches nothing (its name ends in "_alias", its bytes are 0).  Output
 * buffers must therefore be 16-byte aligned like every other tensor. */
int32_t clg_compile(clg_ctx *ctx, clg_graph *g, const int32_t *matches,
                    size_t n, clg_plan **out);
int32_t clg_plan_destroy(clg_plan *plan);
/* Whether executions of the plan read the caller's device buffer of constant
 * `node` (*reads = 1) or only the plan's own packed copy of it, made by
 * clg_compile (*reads = 0; also for a constant no kernel of the plan uses).  A
 * constant that is not read may be released or overwritten by the caller as
 * far as this plan is concerned (the measurer and later clg_compile calls on
 * the graph still read it).  *packed_bytes (may be NULL) receives the size of
 * the plan's packed copies of that constant.  UNKNOWN_ID if node is no
 * constant of the plan's graph. */
int32_t clg_plan_reads_constant(const clg_plan *plan, int32_t node, int32_t *reads,
                                size_t *packed_bytes);
int32_t clg_plan_workspace_bytes(const clg_plan *plan, size_t *bytes);
int32_t clg_plan_num_kernels(const clg_plan *plan, size_t *n);
int32_t clg_plan_kernel_info(const clg_plan *plan, size_t index,
                             clg_kernel_info *info);
/* Lanes (Sec. 4.1: the groups of a placement form a DAG, not a chain).  An
 * execution enqueues kernels of independent branches on up to `lanes` HIP
 * streams: lane 0 is the caller's stream, the others belong to the plan
 * (created at its first execution, default priority, released by
 * clg_plan_destroy).  Lanes are forked from and joined back into the caller's
 * stream with events inside every clg_execute, so for the caller the call
 * behaves like work on its own stream, also under HIP graph capture.
 * Dependencies: data flow between kernels plus every reuse of a workspace
 * region.  lanes = 1 (the default) runs everything on the caller's stream; at
 * most 4.  On MI355X a dependency between two hardware queues costs several
 * times a small kernel, so at batch 1 more than one lane measured slower
 * (ResNet-50: 0.55 ms against 0.38 ms); the option is for placements whose
 * branches hold long kernels.  Not to be called while the plan executes (it waits for the
 * plan's own streams).  Executions of one plan must not overlap each other.
 * clg_plan_num_lanes: lanes the current schedule uses (1 for a chain). */
int32_t clg_plan_set_lanes(clg_plan *plan, int32_t lanes);
int32_t clg_plan_num_lanes(const clg_plan *plan, int32_t *lanes);
/* inputs: host array of device pointers, one per graph input in creation
 * order; outputs: host array of device pointers, one per marked output, each
 * large enough for its tensor; workspace: device memory of at least
 * clg_plan_workspace_bytes, 256-byte aligned.  Asynchronous on `stream`.
 * Errors: INVALID_ARG, WORKSPACE_TOO_SMALL, HIP_ERROR. */
int32_t clg_execute(clg_plan *plan, const void *const *inputs,
                    void *const *outputs, void *workspace, size_t ws_bytes,
                    void *stream);
/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): clg_execute without the
 * workspace argument.  The plan's intermediate tensors and split-K partial
 * sums go to a fixed array of CLG_STATIC_WORKSPACE_BYTES that is part of the
 * library's device code; each GPU holds its own copy from the moment the
 * library is loaded until the process ends.  The call allocates and frees
 * nothing, on the device or through any library; inputs and outputs are the
 * caller's as in clg_execute, and the results are bit for bit those of
 * clg_execute.  Nothing in the array has to start at zero (every kernel writes
 * what a later one reads), and it keeps the last call's contents.  All calls
 * on one GPU share the array: two executions that overlap in time on one GPU -
 * of one plan or of different plans, on any streams - race; order them on one
 * stream or with events.  Errors: WORKSPACE_TOO_SMALL if the plan needs more
 * than CLG_STATIC_WORKSPACE_BYTES (clg_plan_workspace_bytes tells; use
 * clg_execute then), INVALID_ARG for a plan with more than one lane that has
 * not yet been run by clg_execute (its streams are created there), otherwise
 * as clg_execute. */
#define CLG_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
int32_t clg_execute_static(clg_plan *plan, const void *const *inputs,
                           void *const *outputs, void *stream);
/* As clg_execute, with a HIP event pair around every kernel on `stream`;
 * synchronises, then writes each kernel's duration in nanoseconds to
 * kernel_ns (host array, one entry per plan kernel; 0 for an entry that
 * launches nothing). */
int32_t clg_execute_timed(clg_plan *plan, const void *const *inputs,
                          void *const *outputs, void *workspace,
                          size_t ws_bytes, void *stream, int64_t *kernel_ns,
                          size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* COLLAGE_MI_H */
