"""GPU parity on seeded random single operators at odd shapes: ragged tiles,
non-square images and filters, unequal strides, pads up to the filter size,
grouped and depthwise convolutions, every fused tail, each as ONE kernel under
every kernel-variant backend that takes it, against the oracle at the
per-operator bar.  The fixed cases of the other files cover the shapes of the
workloads; these cover what nobody thought of.
"""
import numpy as np
import pytest

import workloads as wl
from workloads.patterns import P, W
from parity_util import run_group
from test_gpu_real_shapes import conv_graph, BR, BAR, B_, BT

pytestmark = pytest.mark.gpu

TAILS = [(), B_, BR, BAR, ("relu",), BT]
DENSE_TAILS = [(), ("bias_add",), ("bias_add", "relu"), ("bias_add", "gelu"), ("bias_add", "add"), ("bias_add", "tanh")]
CASES_PER_SEED = 6


def _backends():
    import bench
    return tuple(bench.VARIANTS) + ("direct",)


def _run(d, pat, what, backends=None, tol=1e-4):
    import paper_2111_00655_amd as clg
    ref, ran = None, 0
    for be in backends or _backends():
        try:
            name, ref = run_group(d, be, pat, ref=ref, tol=tol, what=what)
        except clg.ClgError as e:                       # the backend has no kernel for this fused kind at all
            assert e.status == "NO_KERNEL", (what, be, str(e))
            continue
        ran += name is not None
    assert ran >= 1, (what, "no backend ran it")


def random_conv2d(r, scale):
    g = int(r.choice([1, 1, 1, 2, 3, 4, 8]))
    cin, cout = g * int(r.integers(1, 24 * scale)), g * int(r.integers(1, 24 * scale))
    if r.random() < 0.15:
        g = cin = cout = int(r.integers(2, 40))         # depthwise
    h, w = int(r.integers(1, 34 * min(scale, 2))), int(r.integers(1, 34 * min(scale, 2)))
    kh, kw = (int(r.choice([1, 2, 3, 5, 7])),) * 2 if r.random() < 0.7 else (int(r.integers(1, 6)), int(r.integers(1, 6)))
    sh, sw = (int(r.integers(1, 4)),) * 2 if r.random() < 0.8 else (int(r.integers(1, 4)), int(r.integers(1, 4)))
    ph, pw = int(r.integers(0, kh)), int(r.integers(0, kw))
    if h + 2 * ph < kh or w + 2 * pw < kw:
        h, w = h + kh, w + kw
    n = int(r.choice([1, 1, 2, 3]))
    tail = TAILS[int(r.integers(len(TAILS)))]
    return ("conv2d", n, cin, cout, h, w, kh, kw, sh, sw, ph, pw, g, tail), \
        conv_graph("conv2d", r, n, cin, cout, (h, w), (kh, kw), (sh, sw), (ph, pw), tail, groups=g)


def random_conv2d_transpose(r, scale):
    cin, cout = int(r.integers(1, 40 * scale)), int(r.integers(1, 40 * scale))
    h, w = int(r.integers(1, 18)), int(r.integers(1, 18))
    k, s, p = [(4, 2, 1), (6, 3, 0), (2, 2, 0), (3, 1, 1), (4, 1, 0), (3, 2, 1), (5, 2, 2), (4, 4, 0)][int(r.integers(8))]
    if (min(h, w) - 1) * s - 2 * p + k < 1:
        h, w = h + 2, w + 2
    n = int(r.choice([1, 2, 5]))
    tail = TAILS[int(r.integers(len(TAILS)))]
    return ("conv2d_transpose", n, cin, cout, h, w, k, s, p, tail), \
        conv_graph("conv2d_transpose", r, n, cin, cout, (h, w), (k, k), (s, s), (p, p), tail, wscale=0.1)


def random_conv3d(r, scale):
    cin, cout = int(r.integers(1, 20 * scale)), int(r.integers(1, 20 * scale))
    k = tuple(int(x) for x in r.choice([1, 3], 3))
    sp = tuple(int(x) + kk - 1 for x, kk in zip(r.integers(1, 12, 3), k))
    s = tuple(int(x) for x in r.integers(1, 3, 3))
    p = tuple(int(r.integers(0, kk)) for kk in k)
    tail = TAILS[int(r.integers(len(TAILS) - 1))]
    return ("conv3d", cin, cout, sp, k, s, p, tail), conv_graph("conv3d", r, 1, cin, cout, sp, k, s, p, tail)


def random_dense(r, scale):
    m, n = int(r.integers(1, 150 * scale)), int(r.integers(1, 150 * scale))
    k = int(r.integers(1, 80 * scale)) * int(r.choice([1, 1, 4, 16]))
    tail = DENSE_TAILS[int(r.integers(len(DENSE_TAILS)))]
    d = wl.GraphDesc("dense")
    x = d.input(r.standard_normal((m, k)).astype(np.float32))
    y = d.op("dense", [x, d.const((r.standard_normal((n, k)) * k ** -0.5).astype(np.float32))])
    pat = P("dense", W, W)
    for op in tail:
        if op == "bias_add":
            y = d.op("bias_add", [y, d.const(r.standard_normal(n).astype(np.float32))], axis=-1)
            pat = P("bias_add", pat, W)
        elif op == "add":
            y = d.op("add", [y, d.input(r.standard_normal((m, n)).astype(np.float32))])
            pat = P("add", pat, W)
        else:
            y = d.op(op, [y])
            pat = P(op, pat)
    d.mark_output(y)
    return ("dense", m, k, n, tail), (d, pat)


MAKERS = (random_conv2d, random_conv2d, random_dense, random_conv2d_transpose, random_conv3d, random_dense)


@pytest.mark.parametrize("scale", [1, 6])
@pytest.mark.parametrize("seed", range(16))
def test_random_single_operators_under_every_backend(seed, scale):
    for i in range(CASES_PER_SEED):
        r = np.random.default_rng([2111, scale, seed, i])
        what, (d, pat) = MAKERS[i % len(MAKERS)](r, scale)
        _run(d, pat, what)


@pytest.mark.parametrize("seed", range(24))
def test_random_graphs_under_searched_and_random_placements(seed):
    """Search-then-compile-then-run on random DAGs (chains, branches, diamonds, values with several consumers):
    the op-level search's optimum under several seeded cost tables and a handful of other covers of the match
    list, executed and compared with the oracle; every placement of one graph must give the same outputs."""
    import paper_2111_00655_amd as clg
    from oracle.graph import Graph, norm_err
    from oracle.match import enumerate_matches
    from oracle import search
    d = wl.random_dag(seed, n_ops=6 + seed % 9, ch=(4, 16, 20, 33)[seed % 4], image=(6, 9, 14)[seed % 3])
    reg = wl.default_registry(("igemm", "igemm_s8_nk", "igemm_r16", "igemm_r32_w4"))
    s = clg.Session(d, reg, device=0)
    ms = s.match()
    g = Graph(d)
    ref = g.run()
    placements = []
    for cs in range(3):
        costs = wl.synthetic_costs(len(ms), 131 * seed + cs, ties=(cs == 1))
        placements.append(s.search(costs, 0)[1])
    oms = enumerate_matches(g, reg)
    assert len(oms) == len(ms)
    r = np.random.default_rng([7, seed])
    for cs in range(4):                                 # covers the search would not pick: optimum of a random table in the oracle
        costs = [int(c) for c in r.integers(1, 1000, len(oms))]
        placements.append(search.dp(g, reg, oms, costs, 0)[1])
    ran = 0
    for ids in placements:
        plan = s.compile(ids)
        got = plan.run()
        ran += 1
        for a, b in zip(got, ref):
            assert a.shape == b.shape
            assert norm_err(a, b) <= 1e-3, (seed, ids, plan.kernels())
        plan.destroy()
    assert ran == len(placements)
    s.close()


# ---- the other kernel families ------------------------------------------------------------------------------
def _f32(r, *shape, scale=1.0):
    return (r.standard_normal(shape) * scale).astype(np.float32)


def random_batch_matmul(r):
    b, m, n, k = int(r.integers(1, 7)), int(r.integers(1, 150)), int(r.integers(1, 150)), int(r.integers(1, 150))
    tb, sc = bool(r.integers(2)), bool(r.integers(2))
    d = wl.GraphDesc("bmm")
    y = d.op("batch_matmul", [d.input(_f32(r, b, m, k)), d.input(_f32(r, b, n, k) if tb else _f32(r, b, k, n))], transpose_b=tb)
    pat = P("batch_matmul", W, W)
    if sc:
        y, pat = d.op("mul_scalar", [y], scalar=0.125), P("mul_scalar", pat)
    d.mark_output(y)
    return ("batch_matmul", b, m, n, k, tb, sc), d, pat, None, 1e-4


def random_softmax(r):
    nd = int(r.integers(1, 4))
    shape = tuple(int(x) for x in r.integers(1, 12, nd - 1)) + (int(r.choice([r.integers(1, 70), r.integers(1, 3000)])),)
    d = wl.GraphDesc("softmax")
    if r.integers(2):
        d.mark_output(d.op("softmax", [d.input(_f32(r, *shape, scale=3.0))]))
        pat = P("softmax", W)
    else:
        d.mark_output(d.op("softmax", [d.op("mul_scalar", [d.input(_f32(r, *shape, scale=9.0))], scalar=0.125)]))
        pat = P("softmax", P("mul_scalar", W))
    return ("softmax", shape), d, pat, ("rowwise",), 1e-5


def random_layer_norm(r):
    # rows of 8 values and more: over two or three values the result is +-1 however close they are, which no
    # fp32 mean resolves to 1e-4 of the oracle's fp64 one
    rows, L = int(r.integers(1, 200)), int(r.choice([r.integers(8, 70), r.integers(8, 3000), 4 * r.integers(16, 512)]))
    shape = (rows, L) if r.integers(2) else (int(r.integers(1, 4)), rows, L)
    g, b = (1 + 0.02 * r.standard_normal(L)).astype(np.float32), _f32(r, L, scale=0.02)
    d = wl.GraphDesc("layer_norm")
    v = int(r.integers(3))
    if v == 0:
        y, pat = d.input(_f32(r, *shape) + np.float32(0.5)), W
    elif v == 1:
        y, pat = d.op("add", [d.input(_f32(r, *shape)), d.input(_f32(r, *shape))]), P("add", W, W)
    else:
        y = d.op("bias_add", [d.input(_f32(r, *shape)), d.const(_f32(r, L))], axis=-1)
        y, pat = d.op("add", [y, d.input(_f32(r, *shape))]), P("add", P("bias_add", W, W), W)
    d.mark_output(d.op("layer_norm", [y, d.const(g), d.const(b)], eps=1e-12))
    return ("layer_norm", shape, v), d, P("layer_norm", pat, W, W), ("rowwise",), 5e-5


def random_attention(r):
    heads, sq, sk, dd = int(r.integers(1, 7)), int(r.integers(1, 200)), int(r.integers(1, 513)), int(r.choice([32, 64, 128]))
    scaled, merged = bool(r.integers(2)), bool(r.integers(2))
    d = wl.GraphDesc("attention")
    q, k, v = d.input(_f32(r, heads, sq, dd)), d.input(_f32(r, heads, sk, dd)), d.input(_f32(r, heads, sk, dd))
    y, pat = d.op("batch_matmul", [q, k], transpose_b=True), P("batch_matmul", W, W)
    if scaled:
        y, pat = d.op("mul_scalar", [y], scalar=float(1.0 / np.sqrt(dd))), P("mul_scalar", pat)
    y = d.op("batch_matmul", [d.op("softmax", [y]), v], transpose_b=False)
    pat = P("batch_matmul", P("softmax", pat), W)
    if merged:
        y = d.op("reshape", [d.op("transpose", [y], dims=(1, 0, 2))], dims=(sq, heads * dd))
        pat = P("reshape", P("transpose", pat))
    d.mark_output(y)
    return ("attention", heads, sq, sk, dd, scaled, merged), d, pat, ("attention",), 1e-4


def random_pool(r):
    k = (int(r.integers(1, 6)), int(r.integers(1, 6))) if r.random() < 0.3 else (int(r.integers(1, 6)),) * 2
    s = (int(r.integers(1, 4)), int(r.integers(1, 4))) if r.random() < 0.3 else (int(r.integers(1, 4)),) * 2
    p = (int(r.integers(0, k[0] // 2 + 1)), int(r.integers(0, k[1] // 2 + 1)))
    shape = (int(r.integers(1, 4)), int(r.integers(1, 50)), int(r.integers(k[0], 40)), int(r.integers(k[1], 40)))
    kind = ["max_pool2d", "avg_pool2d", "global_avg_pool2d"][int(r.integers(3))]
    d = wl.GraphDesc("pool")
    x = d.input(_f32(r, *shape))
    if kind == "global_avg_pool2d":
        d.mark_output(d.op(kind, [x]))
        return (kind, shape), d, P(kind, W), ("direct",), 1e-5
    y, pat = d.op(kind, [x], kernel=k, stride=s, pad=p), P(kind, W)
    if r.integers(2):
        ho, wo = (shape[2] + 2 * p[0] - k[0]) // s[0] + 1, (shape[3] + 2 * p[1] - k[1]) // s[1] + 1
        other = d.input(_f32(r, shape[0], shape[1], ho, wo))
        y, pat = d.op("add", [other, y] if r.integers(2) else [y, other]), P("add", pat, W)
    d.mark_output(y)
    return (kind, k, s, p, shape), d, pat, ("direct",), 1e-5


def random_concat(r):
    n, nd = int(r.integers(2, 9)), int(r.integers(1, 5))
    base = [int(x) for x in r.integers(1, 9, nd)]
    axis = int(r.integers(-nd, nd))
    shapes = []
    for _ in range(n):
        sh = list(base)
        sh[axis] = int(r.integers(1, 12))
        shapes.append(tuple(sh))
    d = wl.GraphDesc("concat")
    d.mark_output(d.op("concat", [d.input(_f32(r, *s)) for s in shapes], axis=axis))
    return ("concat", shapes, axis), d, P("concat", *([W] * n)), ("eltwise",), 0.0


def random_elementwise_chain(r):
    nd = int(r.integers(2, 5))
    shape = tuple(int(x) for x in r.integers(1, 20, nd))
    d = wl.GraphDesc("elementwise")
    y, pat, ops = d.input(_f32(r, *shape)), W, []
    for _ in range(int(r.integers(1, 6))):
        op = ["relu", "gelu", "tanh", "mul_scalar", "add", "bias_add"][int(r.integers(6))]
        ops.append(op)
        if op == "add":
            o = d.input(_f32(r, *shape))
            first = bool(r.integers(2)) or pat is W
            y, pat = d.op("add", [y, o] if first else [o, y]), (P("add", pat, W) if first else P("add", W, pat))
        elif op == "bias_add":
            ax = 1 if (nd == 4 and r.integers(2)) else -1
            y, pat = d.op("bias_add", [y, d.const(_f32(r, shape[ax]))], axis=ax), P("bias_add", pat, W)
        elif op == "mul_scalar":
            y, pat = d.op("mul_scalar", [y], scalar=0.37), P("mul_scalar", pat)
        else:
            y, pat = d.op(op, [y]), P(op, pat)
    d.mark_output(y)
    return ("elementwise", shape, ops), d, pat, ("eltwise",), 1e-5


def random_embedding_layer_norm(r):
    vocab, L, H, nt = int(r.integers(2, 500)), int(r.integers(1, 150)), 4 * int(r.integers(16, 513)), int(r.integers(2, 4))
    d = wl.GraphDesc("embedding")
    e, pat = d.op("take", [d.const(_f32(r, vocab, H, scale=0.02)), d.input(r.integers(0, vocab, L).astype(np.int32))]), P("take", W, W)
    e = d.op("add", [e, d.op("take", [d.const(_f32(r, L + 3, H, scale=0.02)), d.const(np.arange(L, dtype=np.int32))])])
    pat = P("add", pat, P("take", W, W))
    if nt == 3:
        e = d.op("add", [e, d.op("take", [d.const(_f32(r, 2, H, scale=0.02)), d.const(np.zeros(L, dtype=np.int32))])])
        pat = P("add", pat, P("take", W, W))
    g, b = (1 + 0.02 * r.standard_normal(H)).astype(np.float32), _f32(r, H, scale=0.02)
    d.mark_output(d.op("layer_norm", [e, d.const(g), d.const(b)], eps=1e-12))
    return ("embedding", vocab, L, H, nt), d, P("layer_norm", pat, W, W), ("rowwise",), 5e-5


def random_layout(r):
    nd = int(r.integers(2, 5))
    shape, perm = tuple(int(x) for x in r.integers(1, 12, nd)), tuple(int(x) for x in r.permutation(nd))
    d = wl.GraphDesc("transpose")
    d.mark_output(d.op("transpose", [d.input(_f32(r, *shape))], dims=perm))
    return ("transpose", shape, perm), d, P("transpose", W), ("eltwise",), 0.0


def random_separable_conv(r):
    c = int(r.integers(1, 100))
    cout = c if r.integers(2) else int(r.integers(1, 100))
    k, s = int(r.choice([0, 3, 5, 7])), int(r.integers(1, 3))
    h, w = int(r.integers(max(k, 1), 40)), int(r.integers(max(k, 1), 40))
    pre = bool(r.integers(2)) or k == 0
    n = int(r.choice([1, 1, 2, 3]))
    tail = [(), ("bias_add",), ("bias_add", "relu"), ("bias_add", "add"), ("bias_add", "add", "relu")][int(r.integers(5))]
    d = wl.GraphDesc("separable")
    y, pat = d.input(_f32(r, n, c, h, w)), W
    if pre:
        y, pat = d.op("relu", [y]), P("relu", pat)
    if k:
        y = d.op("conv2d", [y, d.const(_f32(r, c, 1, k, k, scale=1.0 / k))], stride=(s, s), pad=(k // 2, k // 2), groups=c)
        y = d.op("conv2d", [y, d.const(_f32(r, cout, c, 1, 1, scale=c ** -0.5))], stride=(1, 1), pad=(0, 0), groups=1)
        pat = P("conv2d", P("conv2d", pat, W), W)
    else:
        y = d.op("conv2d", [y, d.const(_f32(r, cout, c, 1, 1, scale=c ** -0.5))], stride=(s, s), pad=(0, 0), groups=1)
        pat = P("conv2d", pat, W)
    ho, wo = (h + 2 * (k // 2) - max(k, 1)) // s + 1, (w + 2 * (k // 2) - max(k, 1)) // s + 1
    for op in tail:
        if op == "bias_add":
            y, pat = d.op("bias_add", [y, d.const(_f32(r, cout, scale=0.1))], axis=1), P("bias_add", pat, W)
        elif op == "add":
            y, pat = d.op("add", [y, d.input(_f32(r, n, cout, ho, wo))]), P("add", pat, W)
        else:
            y, pat = d.op(op, [y]), P(op, pat)
    d.mark_output(y)
    return ("separable", n, c, cout, h, w, k, s, pre, tail), d, pat, ("sepconv",), 1e-4


OTHER_FAMILIES = (random_batch_matmul, random_softmax, random_layer_norm, random_attention, random_pool, random_concat,
                  random_elementwise_chain, random_embedding_layer_norm, random_layout, random_separable_conv)


@pytest.mark.parametrize("family", OTHER_FAMILIES, ids=lambda f: f.__name__)
def test_random_cases_of_the_other_kernel_families(family):
    for i in range(24):
        r = np.random.default_rng([2111, OTHER_FAMILIES.index(family), i])
        what, d, pat, backends, tol = family(r)
        _run(d, pat, what, backends=backends, tol=tol)
