// Computation graph G (paper Sec. 4.1): nodes, shape inference, derived order.
#include <algorithm>
#include <cstdarg>
#include <cstdio>

#include "core.h"

namespace clg {

static thread_local char g_err[512] = "";

void set_error(const char *msg) {
    std::snprintf(g_err, sizeof g_err, "%s", msg);
}

int32_t fail(int32_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

const char *last_error() { return g_err; }

static const char *kOpNames[CLG_OP_COUNT] = {
    "conv2d", "conv2d_transpose", "dense", "batch_matmul", "bias_add", "add",
    "mul_scalar", "relu", "gelu", "tanh", "softmax", "layer_norm", "max_pool2d",
    "global_avg_pool2d", "take", "reshape", "transpose", "avg_pool2d", "concat", "conv3d", "max_pool3d",
    "global_avg_pool3d"};

const char *op_name(int32_t kind) {
    if (kind >= 0 && kind < CLG_OP_COUNT) return kOpNames[kind];
    if (kind == NODE_INPUT) return "input";
    if (kind == NODE_CONST) return "const";
    return "?";
}

std::string Shape::str() const {
    std::string s = "[";
    for (int i = 0; i < ndim; ++i) {
        if (i) s += ",";
        s += std::to_string(d[i]);
    }
    return s + "]";
}

static int n_operands(int32_t kind) {
    switch (kind) {
    case CLG_OP_CONV2D: case CLG_OP_CONV2D_TRANSPOSE: case CLG_OP_DENSE:
    case CLG_OP_BATCH_MATMUL: case CLG_OP_BIAS_ADD: case CLG_OP_ADD: case CLG_OP_TAKE: case CLG_OP_CONV3D:
        return 2;
    case CLG_OP_LAYER_NORM:
        return 3;
    default:
        return 1;
    }
}

int32_t infer_shape(const Graph &g, int32_t kind, const std::vector<int32_t> &in,
                    const clg_attrs &a, Shape *out, int32_t *dtype) {
    if (kind < 0 || kind >= CLG_OP_COUNT) return fail(CLG_INVALID_ARG, "unknown op kind %d", kind);
    if (kind == CLG_OP_CONCAT) {
        if (in.size() < 2 || in.size() > CLG_MAX_PATTERN_ARGS)
            return fail(CLG_INVALID_ARG, "concat takes 2..%d operands, got %zu", CLG_MAX_PATTERN_ARGS, in.size());
    } else if ((int)in.size() != n_operands(kind)) {
        return fail(CLG_INVALID_ARG, "%s takes %d operands, got %zu", op_name(kind),
                    n_operands(kind), in.size());
    }
    const Shape &x = g.nodes[in[0]].shape;
    *dtype = CLG_F32;
    auto f32 = [&](int i) { return g.nodes[in[i]].dtype == CLG_F32; };
    auto bad = [&](const char *why) {
        std::string s = std::string(op_name(kind)) + ": " + why + " (";
        for (size_t i = 0; i < in.size(); ++i) s += (i ? " " : "") + g.nodes[in[i]].shape.str();
        s += ")";
        return fail(CLG_SHAPE_MISMATCH, "%s", s.c_str());
    };
    const bool first_is_f32 = f32(0);
    if (!first_is_f32) return bad("first operand must be fp32");
    Shape y;
    switch (kind) {
    case CLG_OP_CONV2D: {
        const Shape &w = g.nodes[in[1]].shape;
        const int G = a.groups > 0 ? a.groups : 1;
        if (x.ndim != 4 || w.ndim != 4 || !f32(1)) return bad("needs x[N,C,H,W], w[O,C/G,kh,kw]");
        if (a.stride[0] < 1 || a.stride[1] < 1 || a.pad[0] < 0 || a.pad[1] < 0) return bad("stride/pad");
        if (x.d[1] % G || w.d[0] % G || w.d[1] != x.d[1] / G) return bad("channels vs groups");
        const int64_t ho = (x.d[2] + 2 * a.pad[0] - w.d[2]) / a.stride[0] + 1;
        const int64_t wo = (x.d[3] + 2 * a.pad[1] - w.d[3]) / a.stride[1] + 1;
        if (x.d[2] + 2 * a.pad[0] < w.d[2] || x.d[3] + 2 * a.pad[1] < w.d[3] || ho < 1 || wo < 1)
            return bad("empty output");
        y.ndim = 4; y.d[0] = x.d[0]; y.d[1] = w.d[0]; y.d[2] = ho; y.d[3] = wo;
        break;
    }
    case CLG_OP_CONV3D: {
        const Shape &w = g.nodes[in[1]].shape;
        if (x.ndim != 5 || w.ndim != 5 || !f32(1)) return bad("needs x[N,C,D,H,W], w[O,C,kd,kh,kw]");
        if (a.stride_d < 1 || a.stride[0] < 1 || a.stride[1] < 1 || a.pad_d < 0 || a.pad[0] < 0 || a.pad[1] < 0)
            return bad("stride/pad");
        if (a.groups > 1 || w.d[1] != x.d[1]) return bad("channels (groups must be 1)");
        const int64_t st[3] = {a.stride_d, a.stride[0], a.stride[1]}, pd[3] = {a.pad_d, a.pad[0], a.pad[1]};
        y.ndim = 5; y.d[0] = x.d[0]; y.d[1] = w.d[0];
        for (int d = 0; d < 3; ++d) {
            if (x.d[2 + d] + 2 * pd[d] < w.d[2 + d]) return bad("empty output");
            y.d[2 + d] = (x.d[2 + d] + 2 * pd[d] - w.d[2 + d]) / st[d] + 1;
        }
        break;
    }
    case CLG_OP_MAX_POOL3D: {
        if (x.ndim != 5) return bad("needs x[N,C,D,H,W]");
        const int64_t k[3] = {a.kernel_d, a.kernel[0], a.kernel[1]}, st[3] = {a.stride_d, a.stride[0], a.stride[1]},
                      pd[3] = {a.pad_d, a.pad[0], a.pad[1]};
        y.ndim = 5; y.d[0] = x.d[0]; y.d[1] = x.d[1];
        for (int d = 0; d < 3; ++d) {
            if (k[d] < 1 || st[d] < 1 || pd[d] < 0 || 2 * pd[d] > k[d]) return bad("kernel/stride/pad");
            if (x.d[2 + d] + 2 * pd[d] < k[d]) return bad("empty output");
            y.d[2 + d] = (x.d[2 + d] + 2 * pd[d] - k[d]) / st[d] + 1;
        }
        break;
    }
    case CLG_OP_GLOBAL_AVG_POOL3D:
        if (x.ndim != 5) return bad("needs x[N,C,D,H,W]");
        y.ndim = 2; y.d[0] = x.d[0]; y.d[1] = x.d[1];
        break;
    case CLG_OP_CONV2D_TRANSPOSE: {
        const Shape &w = g.nodes[in[1]].shape;
        if (x.ndim != 4 || w.ndim != 4 || !f32(1)) return bad("needs x[N,C,H,W], w[C,O,kh,kw]");
        if (a.stride[0] < 1 || a.stride[1] < 1 || a.pad[0] < 0 || a.pad[1] < 0) return bad("stride/pad");
        if (w.d[0] != x.d[1]) return bad("channels");
        const int64_t ho = (x.d[2] - 1) * a.stride[0] - 2 * a.pad[0] + w.d[2];
        const int64_t wo = (x.d[3] - 1) * a.stride[1] - 2 * a.pad[1] + w.d[3];
        if (ho < 1 || wo < 1) return bad("empty output");
        y.ndim = 4; y.d[0] = x.d[0]; y.d[1] = w.d[1]; y.d[2] = ho; y.d[3] = wo;
        break;
    }
    case CLG_OP_DENSE: {
        const Shape &w = g.nodes[in[1]].shape;
        if (x.ndim != 2 || w.ndim != 2 || w.d[1] != x.d[1] || !f32(1)) return bad("needs x[M,K], w[U,K]");
        y.ndim = 2; y.d[0] = x.d[0]; y.d[1] = w.d[0];
        break;
    }
    case CLG_OP_BATCH_MATMUL: {
        const Shape &b = g.nodes[in[1]].shape;
        if (x.ndim != 3 || b.ndim != 3 || b.d[0] != x.d[0] || !f32(1)) return bad("needs a[B,M,K], b[B,N,K]|[B,K,N]");
        const int64_t kb = a.transpose_b ? b.d[2] : b.d[1];
        const int64_t n = a.transpose_b ? b.d[1] : b.d[2];
        if (kb != x.d[2]) return bad("inner dimension");
        y.ndim = 3; y.d[0] = x.d[0]; y.d[1] = x.d[1]; y.d[2] = n;
        break;
    }
    case CLG_OP_BIAS_ADD: {
        const Shape &b = g.nodes[in[1]].shape;
        const int ax = a.axis >= 0 ? a.axis : x.ndim + a.axis;
        if (b.ndim != 1 || ax < 0 || ax >= x.ndim || x.d[ax] != b.d[0] || !f32(1)) return bad("bias vs axis");
        y = x;
        break;
    }
    case CLG_OP_ADD:
        if (!(g.nodes[in[1]].shape == x) || !f32(1)) return bad("operands differ in shape");
        y = x;
        break;
    case CLG_OP_MUL_SCALAR: case CLG_OP_RELU: case CLG_OP_GELU: case CLG_OP_TANH:
        y = x;
        break;
    case CLG_OP_SOFTMAX:
        if (x.ndim < 1) return bad("rank");
        y = x;
        break;
    case CLG_OP_LAYER_NORM: {
        const Shape &ga = g.nodes[in[1]].shape, &be = g.nodes[in[2]].shape;
        if (x.ndim < 1 || ga.ndim != 1 || be.ndim != 1 || ga.d[0] != x.d[x.ndim - 1] ||
            be.d[0] != x.d[x.ndim - 1] || !f32(1) || !f32(2))
            return bad("gamma/beta vs last axis");
        y = x;
        break;
    }
    case CLG_OP_CONCAT: {
        const int ax = a.axis < 0 ? a.axis + x.ndim : a.axis;
        if (ax < 0 || ax >= x.ndim) return bad("axis");
        y = x;
        for (size_t i = 1; i < in.size(); ++i) {
            const Shape &s = g.nodes[in[i]].shape;
            if (!f32((int)i) || s.ndim != x.ndim) return bad("operands must be fp32 tensors of one rank");
            for (int d = 0; d < x.ndim; ++d)
                if (d != ax && s.d[d] != x.d[d]) return bad("extents differ outside the axis");
            y.d[ax] += s.d[ax];
        }
        break;
    }
    case CLG_OP_AVG_POOL2D:
    case CLG_OP_MAX_POOL2D: {
        if (x.ndim != 4) return bad("needs x[N,C,H,W]");
        if (a.kernel[0] < 1 || a.kernel[1] < 1 || a.stride[0] < 1 || a.stride[1] < 1 ||
            a.pad[0] < 0 || a.pad[1] < 0 || 2 * a.pad[0] > a.kernel[0] || 2 * a.pad[1] > a.kernel[1])
            return bad("kernel/stride/pad");
        const int64_t ho = (x.d[2] + 2 * a.pad[0] - a.kernel[0]) / a.stride[0] + 1;
        const int64_t wo = (x.d[3] + 2 * a.pad[1] - a.kernel[1]) / a.stride[1] + 1;
        if (x.d[2] + 2 * a.pad[0] < a.kernel[0] || x.d[3] + 2 * a.pad[1] < a.kernel[1]) return bad("empty output");
        y.ndim = 4; y.d[0] = x.d[0]; y.d[1] = x.d[1]; y.d[2] = ho; y.d[3] = wo;
        break;
    }
    case CLG_OP_GLOBAL_AVG_POOL2D:
        if (x.ndim != 4) return bad("needs x[N,C,H,W]");
        y.ndim = 2; y.d[0] = x.d[0]; y.d[1] = x.d[1];
        break;
    case CLG_OP_TAKE: {
        const Node &ids = g.nodes[in[1]];
        if (x.ndim != 2 || ids.shape.ndim != 1 || ids.dtype != CLG_I32) return bad("needs table[V,H], ids[L] int32");
        y.ndim = 2; y.d[0] = ids.shape.d[0]; y.d[1] = x.d[1];
        break;
    }
    case CLG_OP_RESHAPE: {
        if (a.ndims < 1 || a.ndims > CLG_MAX_DIMS) return bad("dims");
        y.ndim = a.ndims;
        for (int i = 0; i < a.ndims; ++i) {
            if (a.dims[i] < 1) return bad("dims");
            y.d[i] = a.dims[i];
        }
        if (y.numel() != x.numel()) return bad("element count changes");
        break;
    }
    case CLG_OP_TRANSPOSE: {
        if (a.ndims != x.ndim) return bad("permutation length");
        bool seen[CLG_MAX_DIMS] = {false, false, false, false, false, false};
        y.ndim = x.ndim;
        for (int i = 0; i < a.ndims; ++i) {
            if (a.dims[i] < 0 || a.dims[i] >= x.ndim || seen[a.dims[i]]) return bad("not a permutation");
            seen[a.dims[i]] = true;
            y.d[i] = x.d[a.dims[i]];
        }
        break;
    }
    default:
        return fail(CLG_INVALID_ARG, "unknown op kind %d", kind);
    }
    if (y.numel() <= 0 || y.numel() > kMaxTensorElems)
        return bad("tensor is empty or has more than 2^29 elements");
    *out = y;
    return CLG_OK;
}

// Value of a constrainable attribute of an operator node (has_attr, Sec. 3).
int64_t attr_value(const Graph &g, int32_t node, int32_t attr, bool *ok) {
    const Node &nd = g.nodes[node];
    *ok = true;
    auto weight_dim = [&](int d) -> int64_t {
        if (nd.kind == CLG_OP_MAX_POOL2D || nd.kind == CLG_OP_AVG_POOL2D) return nd.attrs.kernel[d - 2];
        if ((nd.kind == CLG_OP_CONV2D || nd.kind == CLG_OP_CONV2D_TRANSPOSE) && nd.in.size() > 1)
            return g.nodes[nd.in[1]].shape.d[d];
        *ok = false;
        return 0;
    };
    const bool spatial = nd.kind == CLG_OP_CONV2D || nd.kind == CLG_OP_CONV2D_TRANSPOSE ||
                         nd.kind == CLG_OP_MAX_POOL2D || nd.kind == CLG_OP_AVG_POOL2D;
    switch (attr) {
    case CLG_ATTR_GROUPS: return nd.attrs.groups > 0 ? nd.attrs.groups : 1;
    case CLG_ATTR_KERNEL_H: return weight_dim(2);
    case CLG_ATTR_KERNEL_W: return weight_dim(3);
    case CLG_ATTR_STRIDE_H: *ok = spatial; return nd.attrs.stride[0];
    case CLG_ATTR_STRIDE_W: *ok = spatial; return nd.attrs.stride[1];
    case CLG_ATTR_PAD_H: *ok = spatial; return nd.attrs.pad[0];
    case CLG_ATTR_PAD_W: *ok = spatial; return nd.attrs.pad[1];
    case CLG_ATTR_TRANSPOSE_B: return nd.attrs.transpose_b ? 1 : 0;
    case CLG_ATTR_AXIS: return nd.attrs.axis;
    default: *ok = false; return 0;
    }
}

void Graph::finalize() {
    if (finalized) return;
    const int n = (int)nodes.size();
    consumers.assign(n, {});
    depth.assign(n, 0);
    rank.assign(n, -1);
    is_output.assign(n, 0);
    order.clear();
    op_ids.clear();
    for (int i = 0; i < n; ++i) {
        for (int32_t j : nodes[i].in) consumers[j].push_back(i);
        if (nodes[i].is_op()) {
            int d = 0;
            for (int32_t j : nodes[i].in)
                if (nodes[j].is_op()) d = std::max(d, depth[j]);
            depth[i] = d + 1;
            order.push_back(i);
            op_ids.push_back(i);
        }
    }
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return depth[a] < depth[b]; });
    for (size_t r = 0; r < order.size(); ++r) rank[order[r]] = (int32_t)r;
    for (int32_t o : outputs) is_output[o] = 1;
    finalized = true;
}

}  // namespace clg
