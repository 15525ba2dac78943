// Lowering: a backend pattern's structure check at registration, and the
// translation of one match into one kernel call (paper Sec. 4.2: a matched
// subgraph, whether one operator or several fused ones, becomes exactly one
// low-level kernel).
//
// Every pattern the kernel families accept is a chain: an anchor operator
// whose arguments are all wildcards, followed by operators that each take the
// previous one as exactly one argument.  The anchor decides the kernel
// (contraction, row-wise reduction, elementwise, layout copy); the rest of the
// chain becomes the in-register epilogue (or, for softmax / layer norm at the
// end of the chain, the prologue).
#include <algorithm>
#include <cstdio>

#include "core.h"

namespace clg {

namespace {

bool is_elementwise(int32_t op) {
    return op == CLG_OP_BIAS_ADD || op == CLG_OP_ADD || op == CLG_OP_MUL_SCALAR ||
           op == CLG_OP_RELU || op == CLG_OP_GELU || op == CLG_OP_TANH;
}
bool is_contraction(int32_t op) {
    return op == CLG_OP_CONV2D || op == CLG_OP_CONV2D_TRANSPOSE || op == CLG_OP_DENSE ||
           op == CLG_OP_BATCH_MATMUL || op == CLG_OP_CONV3D;
}
bool is_layout(int32_t op) { return op == CLG_OP_RESHAPE || op == CLG_OP_TRANSPOSE; }
bool is_rowwise(int32_t op) { return op == CLG_OP_SOFTMAX || op == CLG_OP_LAYER_NORM; }

}  // namespace

int32_t check_pattern(const Context &ctx, Pattern *p) {
    const int n = (int)p->nodes.size();
    if (n < 1 || n > CLG_MAX_PATTERN_NODES) return fail(CLG_INVALID_ARG, "pattern has %d nodes", n);
    std::vector<int> used(n, 0);
    for (int i = 0; i < n; ++i) {
        const clg_pattern_node &pn = p->nodes[i];
        if (pn.op != CLG_WILDCARD && (pn.op < 0 || pn.op >= CLG_OP_COUNT))
            return fail(CLG_INVALID_ARG, "pattern node %d: bad op kind %d", i, pn.op);
        if (pn.n_args < 0 || pn.n_args > CLG_MAX_PATTERN_ARGS || (pn.op == CLG_WILDCARD && pn.n_args))
            return fail(CLG_INVALID_ARG, "pattern node %d: bad argument count", i);
        if (pn.n_constraints < 0 || pn.n_constraints > CLG_MAX_CONSTRAINTS)
            return fail(CLG_INVALID_ARG, "pattern node %d: bad constraint count", i);
        for (int c = 0; c < pn.n_constraints; ++c)
            if (pn.constraints[c].attr < 0 || pn.constraints[c].attr >= CLG_ATTR_COUNT)
                return fail(CLG_INVALID_ARG, "pattern node %d: bad attribute id", i);
        for (int k = 0; k < pn.n_args; ++k) {
            if (pn.args[k] < 0 || pn.args[k] >= i)
                return fail(CLG_INVALID_ARG, "pattern node %d: argument %d is not an earlier node", i, k);
            if (used[pn.args[k]]++)
                return fail(CLG_INVALID_ARG, "pattern node %d is used twice (not a tree)", pn.args[k]);
        }
    }
    for (int i = 0; i < n - 1; ++i)
        if (!used[i]) return fail(CLG_INVALID_ARG, "pattern node %d is unreachable from the root", i);
    if (p->nodes[n - 1].op == CLG_WILDCARD) return fail(CLG_INVALID_ARG, "the root is a wildcard");

    // The row-wise family also takes one tree: layer norm over the sum of two or three gathered rows.
    p->gather.clear();
    if (ctx.backends[p->backend].family == FAM_ROWWISE && p->nodes[n - 1].op == CLG_OP_LAYER_NORM && p->nodes[n - 1].n_args == 3) {
        auto is_take = [&](int i) {
            const clg_pattern_node &t = p->nodes[i];
            return t.op == CLG_OP_TAKE && t.n_args == 2 && p->nodes[t.args[0]].op == CLG_WILDCARD && p->nodes[t.args[1]].op == CLG_WILDCARD;
        };
        const clg_pattern_node &ln = p->nodes[n - 1];
        const clg_pattern_node &top = p->nodes[ln.args[0]];
        if (top.op == CLG_OP_ADD && top.n_args == 2 && p->nodes[ln.args[1]].op == CLG_WILDCARD && p->nodes[ln.args[2]].op == CLG_WILDCARD) {
            std::vector<int32_t> takes;
            const int l = top.args[0], r = top.args[1];
            auto inner = [&](int i) {                      // add(take, take)
                const clg_pattern_node &a = p->nodes[i];
                return a.op == CLG_OP_ADD && a.n_args == 2 && is_take(a.args[0]) && is_take(a.args[1]);
            };
            if (is_take(l) && is_take(r)) takes = {l, r};
            else if (inner(l) && is_take(r)) takes = {p->nodes[l].args[0], p->nodes[l].args[1], r};
            else if (is_take(l) && inner(r)) takes = {p->nodes[r].args[0], p->nodes[r].args[1], l};
            if (!takes.empty()) {
                p->gather = takes;
                p->chain = {n - 1};
                p->main_arg = {-1};
                return CLG_OK;
            }
        }
    }

    // chain view
    p->chain.clear();
    p->main_arg.clear();
    int cur = n - 1;
    for (;;) {
        const clg_pattern_node &pn = p->nodes[cur];
        int main = -1, n_ops = 0;
        for (int k = 0; k < pn.n_args; ++k)
            if (p->nodes[pn.args[k]].op != CLG_WILDCARD) {
                main = k;
                ++n_ops;
            }
        if (n_ops > 1)
            return fail(CLG_NO_KERNEL, "no kernel family fuses a pattern that branches at %s", op_name(pn.op));
        p->chain.push_back(cur);
        p->main_arg.push_back(main);
        if (n_ops == 0) break;
        cur = pn.args[main];
    }
    std::reverse(p->chain.begin(), p->chain.end());
    // main_arg[t] currently says where chain[t]'s child sits; after the reverse
    // the entry of chain[t] must describe chain[t-1]: it already does, as it was
    // pushed together with its node.
    std::reverse(p->main_arg.begin(), p->main_arg.end());

    const Backend &be = ctx.backends[p->backend];
    const int len = (int)p->chain.size();
    auto kind = [&](int t) { return p->nodes[p->chain[t]].op; };
    const int32_t k0 = kind(0), kl = kind(len - 1);
    auto tail_ok = [&](int from, int to) {   // elementwise ops taking the chain as operand 0 (add: either)
        for (int t = from; t < to; ++t) {
            const int32_t k = kind(t);
            if (k == CLG_OP_RESHAPE && t == len - 1 && to == len) continue;
            if (!is_elementwise(k)) return false;
            if (t > 0 && k == CLG_OP_BIAS_ADD && p->main_arg[t] != 0) return false;
        }
        return true;
    };
    if (len - 1 > kMaxEpi) return fail(CLG_NO_KERNEL, "pattern has more than %d fused steps", kMaxEpi);
    bool ok = false;
    switch (be.family) {
    case FAM_IGEMM:
        ok = is_contraction(k0) && tail_ok(1, len);
        // a result stored in a permuted order: dense ... reshape transpose (split into heads),
        // batch_matmul ... transpose reshape (heads merged); the exact forms are checked per match
        if (!ok && len >= 3) {
            const int32_t ka = kind(len - 2), kb = kind(len - 1);
            const bool split = k0 == CLG_OP_DENSE && ka == CLG_OP_RESHAPE && kb == CLG_OP_TRANSPOSE;
            const bool merge = k0 == CLG_OP_BATCH_MATMUL && ka == CLG_OP_TRANSPOSE && kb == CLG_OP_RESHAPE;
            ok = (split || merge) && tail_ok(1, len - 2);
            for (int t = 1; t < len - 2; ++t) ok = ok && kind(t) != CLG_OP_RESHAPE;
        }
        break;
    case FAM_ATTENTION: {
        // batch_matmul [mul_scalar] softmax batch_matmul [transpose reshape]; the probabilities are the
        // first operand of the second product
        int t = 0;
        ok = kind(t++) == CLG_OP_BATCH_MATMUL;
        if (ok && t < len && kind(t) == CLG_OP_MUL_SCALAR) ++t;
        ok = ok && t + 1 < len && kind(t) == CLG_OP_SOFTMAX && kind(t + 1) == CLG_OP_BATCH_MATMUL && p->main_arg[t + 1] == 0;
        t += 2;
        ok = ok && (t == len || (t + 2 == len && kind(t) == CLG_OP_TRANSPOSE && kind(t + 1) == CLG_OP_RESHAPE));
        break;
    }
    case FAM_SEPCONV: {
        // [relu] conv2d [conv2d] tail: a depthwise + 1x1 pair, or a 1x1 convolution behind a relu;
        // which convolution is which is checked per match
        int t = 0;
        const bool pro = k0 == CLG_OP_RELU;
        if (pro) ++t;
        int convs = 0;
        while (t < len && kind(t) == CLG_OP_CONV2D && convs < 2) {
            if (t > 0 && p->main_arg[t] != 0) break;
            ++t;
            ++convs;
        }
        ok = convs >= 1 && (pro || convs == 2) && tail_ok(t, len) && kl != CLG_OP_RESHAPE;
        break;
    }
    case FAM_DIRECT:
        ok = ((k0 == CLG_OP_CONV2D || k0 == CLG_OP_CONV2D_TRANSPOSE || k0 == CLG_OP_MAX_POOL2D || k0 == CLG_OP_AVG_POOL2D || k0 == CLG_OP_MAX_POOL3D) &&
              tail_ok(1, len) && kl != CLG_OP_RESHAPE) ||
             (len == 1 && (k0 == CLG_OP_GLOBAL_AVG_POOL2D || k0 == CLG_OP_GLOBAL_AVG_POOL3D));
        break;
    case FAM_ROWWISE:
        ok = is_rowwise(kl) && (len == 1 || (p->main_arg[len - 1] == 0 && is_elementwise(k0) &&
                                             tail_ok(1, len - 1)));
        break;
    case FAM_ELTWISE: {
        if (is_layout(k0)) {
            int n_tr = 0;
            ok = true;
            for (int t = 0; t < len; ++t) {
                ok = ok && is_layout(kind(t));
                n_tr += kind(t) == CLG_OP_TRANSPOSE;
            }
            ok = ok && n_tr <= 1;
        } else if (k0 == CLG_OP_CONCAT) {
            ok = len == 1;
        } else {
            ok = (is_elementwise(k0) || k0 == CLG_OP_TAKE) && tail_ok(1, len) &&
                 kl != CLG_OP_RESHAPE;
        }
        break;
    }
    default:
        break;
    }
    if (!ok) {
        std::string s;
        for (int t = 0; t < len; ++t) s += std::string(t ? "+" : "") + op_name(kind(t));
        return fail(CLG_NO_KERNEL, "backend %s has no kernel for the fused kind %s", be.name.c_str(), s.c_str());
    }
    return CLG_OK;
}

namespace {

struct ChainView {
    const Graph &g;
    const Pattern &p;
    const MatchRec &m;
    int len() const { return (int)p.chain.size(); }
    int32_t op(int t) const { return p.nodes[p.chain[t]].op; }
    int32_t node(int t) const { return m.wild[p.chain[t]]; }                 // graph node of chain[t]
    int32_t arg(int t, int k) const { return m.wild[p.nodes[p.chain[t]].args[k]]; }  // graph value of its k-th pattern arg
    int32_t other(int t) const { return arg(t, 1 - p.main_arg[t]); }          // binary op: the non-chain operand
};

// Appends the step of elementwise chain op t to `e`.  `as_anchor`: the op's
// own operand 0 is the running value.
int32_t add_step(const ChainView &cv, int t, bool as_anchor, Epilogue *e, int32_t *epi_nodes) {
    const int32_t k = cv.op(t);
    if (k == CLG_OP_RESHAPE) return CLG_OK;
    if (e->n >= kMaxEpi) return fail(CLG_NO_KERNEL, "too many fused steps");
    EpiStep &s = e->s[e->n];
    s.scalar = 0.f;
    s.ptr = nullptr;
    int32_t operand = -1;
    const Node &nd = cv.g.nodes[cv.node(t)];
    switch (k) {
    case CLG_OP_BIAS_ADD: {
        s.op = EPI_BIAS;
        operand = cv.arg(t, 1);
        const Shape &xs = nd.shape;
        const int ax = nd.attrs.axis >= 0 ? nd.attrs.axis : xs.ndim + nd.attrs.axis;
        int64_t inner = 1;
        for (int d = ax + 1; d < xs.ndim; ++d) inner *= xs.d[d];
        const int64_t c = xs.d[ax];
        if (e->bias_c && (e->bias_c != c || e->bias_inner != inner))
            return fail(CLG_NO_KERNEL, "bias_add steps with different channel layouts in one kernel");
        e->bias_c = (int32_t)c;
        e->bias_inner = (int32_t)inner;
        break;
    }
    case CLG_OP_ADD:
        s.op = EPI_ADD;
        operand = as_anchor ? cv.arg(t, 1) : cv.other(t);
        break;
    case CLG_OP_MUL_SCALAR:
        s.op = EPI_SCALE;
        s.scalar = (float)nd.attrs.scalar;
        break;
    case CLG_OP_RELU: s.op = EPI_RELU; break;
    case CLG_OP_GELU: s.op = EPI_GELU; break;
    case CLG_OP_TANH: s.op = EPI_TANH; break;
    default:
        return fail(CLG_NO_KERNEL, "%s cannot be a fused step", op_name(k));
    }
    epi_nodes[e->n] = operand;
    ++e->n;
    return CLG_OK;
}

std::string shape_key(const Graph &g, int32_t v) { return g.nodes[v].shape.str(); }

}  // namespace

int32_t lower_match(const Context &ctx, const Graph &g, int32_t match_id, KernelCall *out) {
    if (match_id < 0 || match_id >= (int32_t)g.matches.size())
        return fail(CLG_UNKNOWN_ID, "match id %d", match_id);
    const MatchRec &m = g.matches[match_id];
    const Pattern &p = ctx.patterns[m.pattern];
    const Backend &be = ctx.backends[p.backend];
    const ChainView cv{g, p, m};
    const int len = cv.len();
    KernelCall c;
    c.match = match_id;
    c.out_node = m.sink;
    const Shape &out_shape = g.nodes[m.sink].shape;
    const int32_t k0 = cv.op(0);
    const Node &anchor = g.nodes[cv.node(0)];
    const int rfw = be.rf_waves ? -be.rf_waves : 0;          // the backend's bound on K-waves per workgroup

    // operands counted once each for the algorithmic byte count
    std::vector<int32_t> ext;
    auto use = [&](int32_t v) {
        if (v >= 0 && std::find(ext.begin(), ext.end(), v) == ext.end()) ext.push_back(v);
    };
    std::string kinds;
    for (int t = 0; t < len; ++t) kinds += std::string(t ? "+" : "") + op_name(cv.op(t));
    if (!p.gather.empty()) kinds = "take*" + std::to_string(p.gather.size()) + "+add+layer_norm";
    char abuf[160];
    std::snprintf(abuf, sizeof abuf, "s%dx%d,p%dx%d,g%d,tb%d,k%dx%d,d%d.%d.%d,ax%d", anchor.attrs.stride[0], anchor.attrs.stride[1],
                  anchor.attrs.pad[0], anchor.attrs.pad[1], anchor.attrs.groups > 0 ? anchor.attrs.groups : 1,
                  anchor.attrs.transpose_b ? 1 : 0, anchor.attrs.kernel[0], anchor.attrs.kernel[1],
                  anchor.attrs.stride_d, anchor.attrs.pad_d, anchor.attrs.kernel_d, anchor.attrs.axis);

    Epilogue epi{};
    int32_t rc = CLG_OK;
    bool gathered = false;
    if (!p.gather.empty()) {
        // layer_norm(add(add(take, take), take), gamma, beta): tables in the pointer slots 0..2 of the fused
        // steps, ids in 3..5
        RowwiseArgs &a = c.row;
        const Node &root = g.nodes[m.sink];
        a.mode = 1;
        a.len = (int)root.shape.d[root.shape.ndim - 1];
        a.rows = (int)(root.shape.numel() / a.len);
        a.eps = (float)root.attrs.eps;
        a.n_gather = (int32_t)p.gather.size();
        for (size_t k = 0; k < p.gather.size(); ++k) {
            const clg_pattern_node &tk = p.nodes[p.gather[k]];
            const int32_t tab = m.wild[tk.args[0]], ids = m.wild[tk.args[1]];
            const Shape &ts = g.nodes[tab].shape, &is = g.nodes[ids].shape;
            if (ts.ndim != 2 || ts.d[1] != a.len || is.numel() != a.rows || g.nodes[ids].dtype != CLG_I32)
                return fail(CLG_NO_KERNEL, "embedding layer norm: every table must be [rows, %d] and every id list hold %d ids", a.len, a.rows);
            a.tab_rows[k] = (int32_t)ts.d[0];
            c.epi_nodes[k] = tab;
            c.epi_nodes[3 + k] = ids;
            use(ids);
        }
        if (a.len % 4 || a.len < 64 || a.len > 2048)
            return fail(CLG_NO_KERNEL, "embedding layer norm: row length must be a multiple of 4 in 64..2048");
        const clg_pattern_node &ln = p.nodes[p.nodes.size() - 1];
        c.a_node = c.epi_nodes[0];
        c.b_node = m.wild[ln.args[1]];
        c.c_node = m.wild[ln.args[2]];
        use(c.b_node);
        use(c.c_node);
        c.kind = CALL_ROWWISE;
        c.name = "embed" + std::to_string(a.n_gather) + "_layer_norm";
        gathered = true;
    } else if (be.family == FAM_ATTENTION) {
        AttentionArgs &a = c.att;
        int t = 1;
        a.scale = 1.f;
        if (cv.op(t) == CLG_OP_MUL_SCALAR) a.scale = (float)g.nodes[cv.node(t++)].attrs.scalar;
        const int t_pv = t + 1;
        const Node &qk = g.nodes[cv.node(0)], &pv = g.nodes[cv.node(t_pv)];
        const int32_t q = cv.arg(0, 0), k = cv.arg(0, 1), v = cv.arg(t_pv, 1);
        const Shape &qs = g.nodes[q].shape, &ks = g.nodes[k].shape, &vs = g.nodes[v].shape;
        if (!qk.attrs.transpose_b || pv.attrs.transpose_b)
            return fail(CLG_NO_KERNEL, "attention needs q k^T with k as [B, Sk, d] and p v with v as [B, Sk, d]");
        if (qs.ndim != 3 || ks.ndim != 3 || vs.ndim != 3 || vs.d[2] != qs.d[2] || vs.d[1] != ks.d[1])
            return fail(CLG_NO_KERNEL, "attention: q, k, v must be [B, S, d] with one head size");
        a.B = (int)qs.d[0]; a.Sq = (int)qs.d[1]; a.Sk = (int)ks.d[1]; a.d = (int)qs.d[2];
        if (!attention_shape_ok(a)) return fail(CLG_NO_KERNEL, "attention kernel takes head sizes 32 / 64 / 128 and up to 512 keys");
        a.merge = 0;
        if (t_pv + 1 < len) {                                // [B, Sq, d] -> transpose (1, 0, 2) -> reshape [Sq, B*d]
            const Node &tr = g.nodes[cv.node(t_pv + 1)], &rs = g.nodes[cv.node(t_pv + 2)];
            if (tr.attrs.ndims != 3 || tr.attrs.dims[0] != 1 || tr.attrs.dims[1] != 0 || tr.attrs.dims[2] != 2 ||
                rs.shape.ndim != 2 || rs.shape.d[0] != a.Sq || rs.shape.d[1] != (int64_t)a.B * a.d)
                return fail(CLG_NO_KERNEL, "attention stores only the head merge [B, S, d] -> [S, B*d] permuted");
            a.merge = 1;
        }
        c.kind = CALL_ATTENTION;
        c.a_node = q; c.b_node = k; c.c_node = v;
        use(q); use(k); use(v);
        c.flops = 2.0 * a.B * a.Sq * (double)a.Sk * a.d * 2.0;
        c.bound = 0;
        c.name = std::string("attention_d") + std::to_string(a.d) + (a.merge ? "_merge" : "");
    } else if (be.family == FAM_SEPCONV) {
        int t = 0;
        SepConvArgs &a = c.sep;
        a.pro_relu = k0 == CLG_OP_RELU ? 1 : 0;
        if (a.pro_relu) ++t;
        const int32_t xa = cv.arg(0, 0);
        const Shape &xs = g.nodes[xa].shape;
        const int t_first = t;
        int t_pw = t;
        if (t + 1 < len && cv.op(t + 1) == CLG_OP_CONV2D) t_pw = t + 1;
        const Node &pwn = g.nodes[cv.node(t_pw)];
        const int32_t wp = cv.arg(t_pw, 1);
        const Shape &wps = g.nodes[wp].shape;
        if (xs.ndim != 4) return fail(CLG_NO_KERNEL, "sepconv needs x[N,C,H,W]");
        a.N = (int)xs.d[0]; a.C = (int)xs.d[1]; a.H = (int)xs.d[2]; a.W = (int)xs.d[3];
        const Node &first = g.nodes[cv.node(t_first)];
        a.sh = first.attrs.stride[0]; a.sw = first.attrs.stride[1];
        a.ph = first.attrs.pad[0]; a.pw = first.attrs.pad[1];
        a.KH = a.KW = 1;
        double macs = 0;
        if (t_pw != t_first) {                             // depthwise stage
            const int32_t wd = cv.arg(t_first, 1);
            const Shape &wds = g.nodes[wd].shape;
            const int G = first.attrs.groups > 0 ? first.attrs.groups : 1;
            if (G != a.C || wds.d[0] != a.C || wds.d[1] != 1 || g.nodes[wd].kind != NODE_CONST)
                return fail(CLG_NO_KERNEL, "the first convolution of a separable pair must be depthwise with constant weights");
            a.KH = (int)wds.d[2]; a.KW = (int)wds.d[3];
            a.has_dw = 1;
            if (pwn.attrs.stride[0] != 1 || pwn.attrs.stride[1] != 1)
                return fail(CLG_NO_KERNEL, "the 1x1 convolution of a separable pair must have stride 1");
            c.c_node = wd;
            use(wd);
            macs += (double)first.shape.numel() * a.KH * a.KW;
        }
        const int Gp = pwn.attrs.groups > 0 ? pwn.attrs.groups : 1;
        if (t_pw == t_first && a.pro_relu && Gp == a.C && wps.d[0] == a.C && wps.d[1] == 1) {
            // relu -> depthwise convolution -> tail: the depthwise kernel of the direct family, with the relu as its prologue
            DirectConvArgs &dc = c.dconv;
            dc.N = a.N; dc.C = a.C; dc.H = a.H; dc.W = a.W; dc.O = a.C; dc.G = a.C;
            dc.KH = (int)wps.d[2]; dc.KW = (int)wps.d[3];
            dc.sh = a.sh; dc.sw = a.sw; dc.ph = pwn.attrs.pad[0]; dc.pw = pwn.attrs.pad[1];
            dc.HO = (int)pwn.shape.d[2]; dc.WO = (int)pwn.shape.d[3];
            dc.pro_relu = 1;
            if (!depthwise_fast_ok(dc)) return fail(CLG_NO_KERNEL, "relu + depthwise convolution: the kernel takes 3x3, 5x5 and 7x7 filters");
            for (int u = t_pw + 1; u < len; ++u)
                if ((rc = add_step(cv, u, false, &epi, c.epi_nodes)) != CLG_OK) return rc;
            if (epi.bias_c && (epi.bias_inner != (int64_t)dc.HO * dc.WO || epi.bias_c != dc.O))
                return fail(CLG_NO_KERNEL, "bias_add axis does not match the kernel's channel dimension");
            for (int s = 0; s < epi.n; ++s) use(c.epi_nodes[s]);
            dc.epi = epi;
            c.kind = CALL_DIRECT_CONV;
            c.a_node = xa;
            c.b_node = wp;
            use(xa);
            use(wp);
            c.flops = 2.0 * (double)pwn.shape.numel() * dc.KH * dc.KW;
            c.bound = 1;
            c.name = "relu_dwconv" + std::to_string(dc.KH) + (epi.n ? "_epi" + std::to_string(epi.n) : std::string());
        } else {
        // relu -> 1x1 convolution -> tail: the register-fed 1x1 kernel with the relu on its operand, if it takes the shape
        bool on_rf = false;
        if (t_pw == t_first && a.pro_relu && Gp == 1 && wps.ndim == 4 && wps.d[2] == 1 && wps.d[3] == 1 &&
            pwn.attrs.pad[0] == 0 && pwn.attrs.pad[1] == 0 && wps.d[1] == a.C && g.nodes[wp].kind == NODE_CONST) {
            Epilogue e2{};
            int32_t nodes2[kMaxEpi];
            for (auto &n2 : nodes2) n2 = -1;
            bool ok2 = true;
            for (int u = t_pw + 1; u < len && ok2; ++u) ok2 = add_step(cv, u, false, &e2, nodes2) == CLG_OK;
            GemmArgs ga{};
            ga.tile = TILE_R16;
            ga.batch = 1;
            ga.epi = e2;
            ga.Nimg = a.N; ga.Cin = a.C; ga.H = a.H; ga.W = a.W;
            ga.Cout = (int)wps.d[0]; ga.KH = ga.KW = 1; ga.sh = a.sh; ga.sw = a.sw; ga.ph = ga.pw = 0;
            ga.HO = (int)pwn.shape.d[2]; ga.WO = (int)pwn.shape.d[3];
            ga.c_numel = pwn.shape.numel();
            ga.bias_on_row = 1;
            ga.mode = GM_CONV;
            ga.M = ga.Cout; ga.N = ga.Nimg * ga.HO * ga.WO; ga.K = ga.Cin;
            ga.lda = ga.K;
            ga.rf_groups = 1;
            if (ok2 && (!e2.bias_c || (e2.bias_inner == (int64_t)ga.HO * ga.WO && e2.bias_c == ga.Cout)) &&
                rf_resolve(&ga, 16, epi_fast_flags(e2), ctx.n_cus, rfw) && ga.rf_tapk == 1) {
                ga.rf_prelu = 1;
                c.gemm = ga;
                for (int s2 = 0; s2 < e2.n; ++s2) {
                    c.epi_nodes[s2] = nodes2[s2];
                    use(nodes2[s2]);
                }
                epi = e2;
                c.kind = CALL_GEMM;
                c.gemm_swap = true;
                c.a_node = xa;
                c.b_node = wp;
                use(xa);
                use(wp);
                c.pack_bytes = rf_pack_bytes(ga);
                c.scratch_bytes = gemm_scratch_bytes(ga);
                c.flops = 2.0 * (double)ga.M * ga.N * ga.K;
                c.bound = 0;
                c.name = "relu_conv_rf16_t1_w" + std::to_string(ga.rf_wgk);
                on_rf = true;
            }
        }
        if (!on_rf) {
        if (Gp != 1 || wps.d[2] != 1 || wps.d[3] != 1 || pwn.attrs.pad[0] != 0 || pwn.attrs.pad[1] != 0 ||
            wps.d[1] != a.C || g.nodes[wp].kind != NODE_CONST)
            return fail(CLG_NO_KERNEL, "sepconv ends in an ungrouped 1x1 convolution without padding and with constant weights");
        a.Cout = (int)wps.d[0];
        a.HO = (int)pwn.shape.d[2]; a.WO = (int)pwn.shape.d[3];
        if ((int64_t)a.N * a.HO * a.WO > ((int64_t)1 << 30)) return fail(CLG_NO_KERNEL, "sepconv: too many pixels");
        for (int u = t_pw + 1; u < len; ++u)
            if ((rc = add_step(cv, u, false, &epi, c.epi_nodes)) != CLG_OK) return rc;
        if (epi.bias_c && (epi.bias_inner != (int64_t)a.HO * a.WO || epi.bias_c != a.Cout))
            return fail(CLG_NO_KERNEL, "bias_add axis does not match the kernel's channel dimension");
        for (int s = 0; s < epi.n; ++s) use(c.epi_nodes[s]);
        a.epi = epi;
        sepconv_resolve(&a);
        if (sepconv_lds_bytes(a) > 160 * 1024) return fail(CLG_NO_KERNEL, "sepconv: %d input channels do not fit in LDS", a.C);
        c.pack_bytes = sepconv_pack_bytes(a);
        c.kind = CALL_SEPCONV;
        c.a_node = xa;
        c.b_node = wp;
        use(xa);
        use(wp);
        macs += (double)pwn.shape.numel() * a.C;
        c.flops = 2.0 * macs;
        c.bound = 0;
        c.name = std::string(a.pro_relu ? "relu_" : "") + (c.c_node >= 0 ? "sepconv" + std::to_string(a.KH) : std::string("pwconv")) +
                 "_w" + std::to_string(a.nwaves) + "m" + std::to_string(a.mt_per_wg) + (epi.n ? "_epi" + std::to_string(epi.n) : std::string());
        }
        }
    } else if (is_contraction(k0)) {
        const int32_t xa = cv.arg(0, 0), wb = cv.arg(0, 1);
        const Shape &xs = g.nodes[xa].shape, &ws = g.nodes[wb].shape, &ys = anchor.shape;
        use(xa);
        use(wb);
        // trailing reshape + transpose (or transpose + reshape): the result is stored permuted
        const bool permuted = len >= 3 && is_layout(cv.op(len - 1)) && is_layout(cv.op(len - 2));
        const int n_tail = permuted ? len - 2 : len;
        for (int t = 1; t < n_tail; ++t) {
            if ((rc = add_step(cv, t, false, &epi, c.epi_nodes)) != CLG_OK) return rc;
        }
        if (permuted)
            for (int s = 0; s < epi.n; ++s)
                if (epi.s[s].op == EPI_ADD)
                    return fail(CLG_NO_KERNEL, "a residual add cannot be fused in front of a permuted store");
        for (int s = 0; s < epi.n; ++s) use(c.epi_nodes[s]);
        // where the channel of a bias step lives
        const bool conv_like = (k0 == CLG_OP_CONV2D || k0 == CLG_OP_CONV2D_TRANSPOSE || k0 == CLG_OP_CONV3D);
        if (epi.bias_c) {
            const int64_t want_inner = k0 == CLG_OP_CONV3D ? ys.d[2] * ys.d[3] * ys.d[4] : (conv_like ? ys.d[2] * ys.d[3] : 1);
            const int64_t want_c = conv_like ? ys.d[1] : ys.d[ys.ndim - 1];
            if (k0 == CLG_OP_BATCH_MATMUL || epi.bias_inner != want_inner || epi.bias_c != want_c)
                return fail(CLG_NO_KERNEL, "bias_add axis does not match the kernel's channel dimension");
        }
        double macs = 0;
        if (be.family == FAM_DIRECT) {
            if (k0 != CLG_OP_CONV2D && k0 != CLG_OP_CONV2D_TRANSPOSE)
                return fail(CLG_NO_KERNEL, "direct backend runs conv2d and conv2d_transpose only");
            DirectConvArgs &a = c.dconv;
            a.transposed = k0 == CLG_OP_CONV2D_TRANSPOSE;
            a.N = (int)xs.d[0]; a.C = (int)xs.d[1]; a.H = (int)xs.d[2]; a.W = (int)xs.d[3];
            a.O = (int)ws.d[a.transposed ? 1 : 0]; a.KH = (int)ws.d[2]; a.KW = (int)ws.d[3];
            a.sh = anchor.attrs.stride[0]; a.sw = anchor.attrs.stride[1];
            a.ph = anchor.attrs.pad[0]; a.pw = anchor.attrs.pad[1];
            a.G = (!a.transposed && anchor.attrs.groups > 0) ? anchor.attrs.groups : 1;
            a.HO = (int)ys.d[2]; a.WO = (int)ys.d[3];
            if (a.transposed && (a.O > 65535 || a.N > 65535))
                return fail(CLG_NO_KERNEL, "the direct transposed convolution takes up to 65535 output channels and images");
            a.epi = epi;
            c.kind = CALL_DIRECT_CONV;
            c.name = a.transposed ? "direct_convt" : "direct_conv";
            macs = a.transposed ? (double)xs.numel() * a.O * a.KH * a.KW : (double)ys.numel() * (a.C / a.G) * a.KH * a.KW;
            c.bound = 1;
        } else {
            GemmArgs &a = c.gemm;
            a.tile = be.tile;
            const bool want_rf = a.tile == TILE_R32 || a.tile == TILE_R16 || a.tile == TILE_R16X2;
            bool rf = false;
            a.batch = 1;
            a.epi = epi;
            a.c_numel = ys.numel();
            if (k0 == CLG_OP_DENSE) {
                a.mode = GM_NT;
                a.M = (int)xs.d[0]; a.K = (int)xs.d[1]; a.N = (int)ws.d[0];
                a.lda = a.K; a.ldb = a.K; a.ldc = a.N;
                a.bias_on_row = 0;
                c.name = "gemm_nt";
                if (permuted) {
                    // [M, H*D] -> reshape [M, H, D] -> transpose (1, 0, 2) -> [H, M, D]
                    const Node &rs = g.nodes[cv.node(len - 2)], &tr = g.nodes[cv.node(len - 1)];
                    if (rs.shape.ndim != 3 || rs.shape.d[0] != a.M || rs.shape.d[1] * rs.shape.d[2] != a.N ||
                        tr.attrs.dims[0] != 1 || tr.attrs.dims[1] != 0 || tr.attrs.dims[2] != 2)
                        return fail(CLG_NO_KERNEL, "dense stores only the head split [M, H*D] -> [H, M, D] permuted");
                    a.ldc = (int)rs.shape.d[2];
                    a.cs_len = (int)rs.shape.d[2];
                    a.cs_stride = (int64_t)a.M * rs.shape.d[2];
                }
                if (want_rf && g.nodes[wb].kind == NODE_CONST)
                    rf = rf_resolve_dense(&a, a.tile == TILE_R32 ? 32 : 16, epi_fast_flags(epi), ctx.n_cus, rfw,
                                           a.tile == TILE_R16X2 ? 2 : 1);
                if (rf) c.pack_bytes = rf_pack_bytes(a);
            } else if (k0 == CLG_OP_BATCH_MATMUL) {
                const bool tb = anchor.attrs.transpose_b != 0;
                a.mode = tb ? GM_NT : GM_NN;
                a.batch = (int)xs.d[0];
                a.M = (int)xs.d[1]; a.K = (int)xs.d[2]; a.N = (int)ys.d[2];
                a.lda = a.K; a.ldb = tb ? a.K : a.N; a.ldc = a.N;
                a.strideA = (int64_t)a.M * a.K; a.strideB = (int64_t)a.N * a.K; a.strideC = (int64_t)a.M * a.N;
                c.name = tb ? "bmm_nt" : "bmm_nn";
                if (permuted) {
                    // [B, M, N] -> transpose (1, 0, 2) -> [M, B, N] -> reshape [M, B*N]
                    const Node &tr = g.nodes[cv.node(len - 2)], &rs = g.nodes[cv.node(len - 1)];
                    if (tr.attrs.dims[0] != 1 || tr.attrs.dims[1] != 0 || tr.attrs.dims[2] != 2 || rs.shape.ndim != 2 ||
                        rs.shape.d[0] != a.M || rs.shape.d[1] != (int64_t)a.batch * a.N)
                        return fail(CLG_NO_KERNEL, "batch_matmul stores only the head merge [B, M, N] -> [M, B*N] permuted");
                    a.ldc = a.batch * a.N;
                    a.strideC = a.N;
                    c.name += "_merge";
                }
            } else if (k0 == CLG_OP_CONV3D) {
                // only the register-fed kernels run it: one grid slice per output depth, depth taps folded
                // into the channel index
                if (!want_rf || g.nodes[wb].kind != NODE_CONST)
                    return fail(CLG_NO_KERNEL, "conv3d runs on the register-fed kernels with constant weights only");
                a.Nimg = (int)xs.d[0]; a.Cin = (int)xs.d[1]; a.D = (int)xs.d[2]; a.H = (int)xs.d[3]; a.W = (int)xs.d[4];
                a.Cout = (int)ws.d[0]; a.KD = (int)ws.d[2]; a.KH = (int)ws.d[3]; a.KW = (int)ws.d[4];
                a.sd = anchor.attrs.stride_d; a.sh = anchor.attrs.stride[0]; a.sw = anchor.attrs.stride[1];
                a.pd = anchor.attrs.pad_d; a.ph = anchor.attrs.pad[0]; a.pw = anchor.attrs.pad[1];
                a.DO = (int)ys.d[2]; a.HO = (int)ys.d[3]; a.WO = (int)ys.d[4];
                a.bias_on_row = 1;
                c.gemm_swap = true;
                a.mode = GM_CONV;
                a.M = a.Cout; a.N = a.Nimg * a.DO * a.HO * a.WO; a.K = a.Cin * a.KD * a.KH * a.KW;
                a.lda = a.K;
                a.rf_groups = 1;
                if ((int64_t)a.Nimg * a.DO > 65535) return fail(CLG_NO_KERNEL, "conv3d: too many (image, depth) slices");
                if (a.KD == 1 && a.pd != 0) return fail(CLG_NO_KERNEL, "conv3d: depth padding needs more than one depth tap");
                rf = rf_resolve(&a, a.tile == TILE_R32 ? 32 : 16, epi_fast_flags(epi), ctx.n_cus, rfw, !be.no_split);
                if (!rf) return fail(CLG_NO_KERNEL, "conv3d: the register-fed kernel does not take this shape or tail");
                c.pack_bytes = rf_pack_bytes(a);
                c.name = "conv3d";
            } else if (k0 == CLG_OP_CONV2D) {
                const int G = anchor.attrs.groups > 0 ? anchor.attrs.groups : 1;
                if (G != 1 && !want_rf)
                    return fail(CLG_NO_KERNEL, "the LDS-tiled implicit-GEMM conv needs groups = 1 (got %d)", G);
                a.Nimg = (int)xs.d[0]; a.Cin = (int)xs.d[1]; a.H = (int)xs.d[2]; a.W = (int)xs.d[3];
                a.Cout = (int)ws.d[0]; a.KH = (int)ws.d[2]; a.KW = (int)ws.d[3];
                a.sh = anchor.attrs.stride[0]; a.sw = anchor.attrs.stride[1];
                a.ph = anchor.attrs.pad[0]; a.pw = anchor.attrs.pad[1];
                a.HO = (int)ys.d[2]; a.WO = (int)ys.d[3];
                a.bias_on_row = 1;
                c.gemm_swap = true;
                // register-fed kernel: needs constant weights (re-packed once) and a common-form tail
                if (want_rf && g.nodes[wb].kind == NODE_CONST) {
                    a.mode = GM_CONV;
                    a.M = a.Cout; a.N = a.Nimg * a.HO * a.WO; a.K = a.Cin * a.KH * a.KW;
                    a.lda = a.K;
                    a.rf_groups = G;
                    rf = rf_resolve(&a, a.tile == TILE_R32 ? 32 : 16, epi_fast_flags(epi), ctx.n_cus, rfw, !be.no_split);
                }
                if (G != 1 && !rf)
                    return fail(CLG_NO_KERNEL, "the register-fed conv runs %d groups only with constant weights, a common-form "
                                "tail and channels per group that divide, or are a multiple of, the tile edge", G);
                if (rf) {
                    c.pack_bytes = rf_pack_bytes(a);
                } else if (a.KH == 1 && a.KW == 1 && a.sh == 1 && a.sw == 1 && a.ph == 0 && a.pw == 0) {
                    // 1x1 stride-1 convolution is a plain GEMM per image: W[Cout,Cin] * X[Cin,H*W]
                    a.mode = GM_NN;
                    a.batch = a.Nimg;
                    a.M = a.Cout; a.N = a.H * a.W; a.K = a.Cin;
                    a.lda = a.K; a.ldb = a.N; a.ldc = a.N;
                    a.strideA = 0; a.strideB = (int64_t)a.Cin * a.N; a.strideC = (int64_t)a.Cout * a.N;
                } else {
                    a.mode = GM_CONV;
                    a.M = a.Cout; a.N = a.Nimg * a.HO * a.WO; a.K = a.Cin * a.KH * a.KW;
                    a.lda = a.K;
                }
                c.name = "conv_igemm";
            } else {
                a.mode = GM_CONVT;
                a.Nimg = (int)xs.d[0]; a.Cin = (int)xs.d[1]; a.H = (int)xs.d[2]; a.W = (int)xs.d[3];
                a.Cout = (int)ws.d[1]; a.KH = (int)ws.d[2]; a.KW = (int)ws.d[3];
                a.sh = anchor.attrs.stride[0]; a.sw = anchor.attrs.stride[1];
                a.ph = anchor.attrs.pad[0]; a.pw = anchor.attrs.pad[1];
                a.HO = (int)ys.d[2]; a.WO = (int)ys.d[3];
                if (a.KH % a.sh || a.KW % a.sw || a.HO % a.sh || a.WO % a.sw)
                    return fail(CLG_NO_KERNEL, "transposed conv kernel needs kernel and output sizes divisible by the stride");
                a.batch = a.sh * a.sw;                       // sub-pixel phases
                a.M = a.Cout; a.N = a.Nimg * (a.HO / a.sh) * (a.WO / a.sw);
                a.K = a.Cin * (a.KH / a.sh) * (a.KW / a.sw);
                a.bias_on_row = 1;
                c.gemm_swap = true;
                c.name = "convt_igemm";
                if (want_rf && g.nodes[wb].kind == NODE_CONST)
                    rf = rf_resolve_convt(&a, a.tile == TILE_R32 ? 32 : 16, epi_fast_flags(epi), ctx.n_cus, rfw);
                if (rf) c.pack_bytes = rf_pack_bytes(a);
            }
            macs = (double)a.batch * a.M * a.N * a.K;
            if (rf && a.rf_groups > 1) macs /= a.rf_groups;
            if ((double)a.M * a.N > 2.0e9 || a.K < 1) return fail(CLG_NO_KERNEL, "GEMM dimensions out of range");
            c.kind = CALL_GEMM;
            c.bound = 0;
            if (rf) {
                c.scratch_bytes = gemm_scratch_bytes(a);
                c.name = (a.rf_tapk == -1 ? "dense_rf" + std::to_string(a.rf_ts) + (a.rf_nb == 2 ? "x2" : "")
                                          : std::string((a.rf_convt || a.rf_d2s) ? "convt_rf" : (a.D > 1 ? "conv3d_rf" : "conv_rf")) + std::to_string(a.rf_ts) + "_t" +
                                                std::to_string(a.rf_tapk)) +
                         "_w" + std::to_string(a.rf_wgk) + (a.cs_len ? "_split" : "") + (a.splitk > 1 ? "_k" + std::to_string(a.splitk) : "");
            } else {
                if (want_rf) a.tile = TILE_S8;           // what the register-fed kernels do not run goes to the LDS-tiled ones
                gemm_resolve(&a, ctx.n_cus);
                if (be.no_split) a.splitk = 1;
                if (k0 == CLG_OP_DENSE && gemv_shape_ok(a, epi_fast_flags(epi))) {
                    a.gemv = 1;                          // a handful of rows: the weights are streamed once, a wave per column
                    a.splitk = 1;
                    c.bound = 1;
                    c.name = "gemv_nt";
                }
                if (a.cs_len) {
                    // only the lean kernel's K-wave tiles place columns block by block, and the
                    // split-K reduction derives a bias channel from the plain offset
                    a.splitk = 1;
                    if (!lean_mm_shape_ok(a, epi_fast_flags(epi)) || a.tile == TILE_M || a.tile == TILE_L)
                        return fail(CLG_NO_KERNEL, "this tile does not store a head-split result");
                    c.name += "_split";
                }
                c.scratch_bytes = gemm_scratch_bytes(a);
                static const char *tn[] = {"auto", "s", "m", "l", "s8", "s16"};
                if (!a.gemv) c.name += std::string("_") + tn[a.tile] + (a.splitk > 1 ? "_k" + std::to_string(a.splitk) : "");
            }
        }
        c.a_node = xa;
        c.b_node = wb;
        c.flops = 2.0 * macs;
    } else if (k0 == CLG_OP_CONCAT) {
        // the operands go into the call's eight pointer slots for fused-step operands
        ConcatArgs &a = c.cat;
        const int ax = anchor.attrs.axis < 0 ? anchor.attrs.axis + out_shape.ndim : anchor.attrs.axis;
        a.n = (int32_t)anchor.in.size();
        a.outer = 1;
        for (int d = 0; d < ax; ++d) a.outer *= out_shape.d[d];
        a.row = out_shape.numel() / a.outer;
        for (int i = 0; i < a.n; ++i) {
            const int32_t v = cv.arg(0, i);
            a.chunk[i] = g.nodes[v].shape.numel() / a.outer;
            c.epi_nodes[i] = v;
            use(v);
        }
        c.kind = CALL_CONCAT;
        c.name = "concat" + std::to_string(a.n);
        c.a_node = cv.arg(0, 0);
    } else if (k0 == CLG_OP_MAX_POOL3D || k0 == CLG_OP_GLOBAL_AVG_POOL3D) {
        const int32_t xa = cv.arg(0, 0);
        const Shape &xs = g.nodes[xa].shape;
        use(xa);
        PoolArgs &a = c.pool;
        a.NC = (int)(xs.d[0] * xs.d[1]);
        if (k0 == CLG_OP_MAX_POOL3D) {
            a.mode = 0;
            a.D = (int)xs.d[2]; a.H = (int)xs.d[3]; a.W = (int)xs.d[4];
            a.KD = anchor.attrs.kernel_d; a.KH = anchor.attrs.kernel[0]; a.KW = anchor.attrs.kernel[1];
            a.sd = anchor.attrs.stride_d; a.sh = anchor.attrs.stride[0]; a.sw = anchor.attrs.stride[1];
            a.pd = anchor.attrs.pad_d; a.ph = anchor.attrs.pad[0]; a.pw = anchor.attrs.pad[1];
            a.DO = (int)anchor.shape.d[2]; a.HO = (int)anchor.shape.d[3]; a.WO = (int)anchor.shape.d[4];
            for (int t = 1; t < len; ++t)
                if ((rc = add_step(cv, t, false, &epi, c.epi_nodes)) != CLG_OK) return rc;
            for (int s = 0; s < epi.n; ++s) use(c.epi_nodes[s]);
            a.epi = epi;
            c.name = "max_pool3d" + (epi.n ? "_epi" + std::to_string(epi.n) : std::string());
        } else {
            a.mode = 1;                                        // the mean over D*H*W values per (n, c)
            a.H = (int)(xs.d[2] * xs.d[3]); a.W = (int)xs.d[4];
            a.D = a.KD = a.sd = a.DO = 1;
            a.HO = a.WO = 1;
            c.name = "global_avg_pool3d";
        }
        c.kind = CALL_POOL;
        c.a_node = xa;
    } else if (k0 == CLG_OP_MAX_POOL2D || k0 == CLG_OP_AVG_POOL2D || k0 == CLG_OP_GLOBAL_AVG_POOL2D) {
        const int32_t xa = cv.arg(0, 0);
        const Shape &xs = g.nodes[xa].shape;
        use(xa);
        PoolArgs &a = c.pool;
        a.NC = (int)(xs.d[0] * xs.d[1]); a.H = (int)xs.d[2]; a.W = (int)xs.d[3];
        a.D = a.KD = a.sd = a.DO = 1;
        if (k0 != CLG_OP_GLOBAL_AVG_POOL2D) {
            a.mode = k0 == CLG_OP_MAX_POOL2D ? 0 : 2;
            a.KH = anchor.attrs.kernel[0]; a.KW = anchor.attrs.kernel[1];
            a.sh = anchor.attrs.stride[0]; a.sw = anchor.attrs.stride[1];
            a.ph = anchor.attrs.pad[0]; a.pw = anchor.attrs.pad[1];
            a.HO = (int)anchor.shape.d[2]; a.WO = (int)anchor.shape.d[3];
            for (int t = 1; t < len; ++t)
                if ((rc = add_step(cv, t, false, &epi, c.epi_nodes)) != CLG_OK) return rc;
            for (int s = 0; s < epi.n; ++s) use(c.epi_nodes[s]);
            a.epi = epi;
            c.name = (a.mode == 0 ? "max_pool" : "avg_pool") + (epi.n ? "_epi" + std::to_string(epi.n) : std::string());
        } else {
            a.mode = 1;
            a.HO = a.WO = 1;
            c.name = "global_avg_pool";
        }
        c.kind = CALL_POOL;
        c.a_node = xa;
    } else if (is_rowwise(cv.op(len - 1))) {
        RowwiseArgs &a = c.row;
        const Node &root = g.nodes[cv.node(len - 1)];
        const Shape &xs = root.shape;
        a.len = (int)xs.d[xs.ndim - 1];
        a.rows = (int)(xs.numel() / a.len);
        int32_t xa;
        if (len == 1) {
            xa = cv.arg(0, 0);
        } else {
            xa = cv.arg(0, 0);
            for (int t = 0; t < len - 1; ++t)
                if ((rc = add_step(cv, t, t == 0, &epi, c.epi_nodes)) != CLG_OK) return rc;
            if (epi.bias_c && (epi.bias_inner != 1 || epi.bias_c != a.len))
                return fail(CLG_NO_KERNEL, "row-wise prologue bias must run along the last axis");
        }
        use(xa);
        for (int s = 0; s < epi.n; ++s) use(c.epi_nodes[s]);
        a.pro = epi;
        if (cv.op(len - 1) == CLG_OP_SOFTMAX) {
            a.mode = 0;
            c.name = "softmax";
        } else {
            a.mode = 1;
            a.eps = (float)root.attrs.eps;
            c.b_node = cv.arg(len - 1, 1);
            c.c_node = cv.arg(len - 1, 2);
            use(c.b_node);
            use(c.c_node);
            c.name = "layer_norm";
        }
        if (epi.n) c.name += "_pro" + std::to_string(epi.n);
        c.kind = CALL_ROWWISE;
        c.a_node = xa;
    } else if (is_layout(k0)) {
        LayoutArgs &a = c.layout;
        const int32_t xa = cv.arg(0, 0);
        use(xa);
        a.numel = out_shape.numel();
        a.ndim = 1;
        a.out_dims[0] = a.numel;
        a.in_strides[0] = 1;
        for (int t = 0; t < len; ++t) {
            if (cv.op(t) != CLG_OP_TRANSPOSE) continue;
            const Node &tr = g.nodes[cv.node(t)];
            const Shape &src = g.nodes[tr.in[0]].shape;     // contiguous view being permuted
            int64_t st[CLG_MAX_DIMS];
            int64_t acc = 1;
            for (int d = src.ndim - 1; d >= 0; --d) {
                st[d] = acc;
                acc *= src.d[d];
            }
            a.ndim = src.ndim;
            for (int d = 0; d < src.ndim; ++d) {
                a.out_dims[d] = tr.shape.d[d];
                a.in_strides[d] = st[tr.attrs.dims[d]];
            }
        }
        c.kind = CALL_LAYOUT;
        c.name = a.ndim == 1 ? "copy" : "permute_copy";
        c.a_node = xa;
    } else if (is_elementwise(k0) || k0 == CLG_OP_TAKE) {
        EltwiseArgs &a = c.elt;
        a.numel = out_shape.numel();
        const int32_t xa = cv.arg(0, 0);
        int start = 0;
        if (k0 == CLG_OP_TAKE) {
            c.b_node = cv.arg(0, 1);
            a.row_len = (int)g.nodes[xa].shape.d[1];
            a.table_rows = (int)g.nodes[xa].shape.d[0];
            start = 1;
            c.name = "take";
        } else {
            c.name = "eltwise";
            use(xa);
        }
        for (int t = start; t < len; ++t)
            if ((rc = add_step(cv, t, t == 0, &epi, c.epi_nodes)) != CLG_OK) return rc;
        for (int s = 0; s < epi.n; ++s) use(c.epi_nodes[s]);
        if (c.b_node >= 0) use(c.b_node);
        a.epi = epi;
        c.name += std::to_string(epi.n);
        c.kind = CALL_ELTWISE;
        c.a_node = xa;
    } else {
        return fail(CLG_NO_KERNEL, "no kernel for a pattern anchored at %s", op_name(k0));
    }

    // algorithmic bytes: every distinct operand and the output once
    double bytes = 4.0 * (double)out_shape.numel();
    for (int32_t v : ext) bytes += 4.0 * (double)g.nodes[v].shape.numel();
    if (k0 == CLG_OP_TAKE) bytes += 4.0 * (double)out_shape.numel();   // the gathered rows, not the table
    if (gathered) bytes += 4.0 * (double)out_shape.numel() * (double)p.gather.size();
    c.bytes = bytes;

    std::string key = be.name + "|" + kinds + "|" + abuf + "|";
    key += shape_key(g, c.a_node);
    for (int32_t v : ext)
        if (v != c.a_node) key += shape_key(g, v);
    key += "->" + out_shape.str();
    for (int s = 0; s < epi.n; ++s)
        if (epi.s[s].op == EPI_SCALE) {
            char sb[32];
            std::snprintf(sb, sizeof sb, "|x%.9g", (double)epi.s[s].scalar);
            key += sb;
        }
    c.key = key;
    *out = c;
    return CLG_OK;
}

}  // namespace clg
