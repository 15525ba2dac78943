"""GPU parity per fused operator at the benchmark's own layer shapes.

Every distinct convolution of ResNet-50 v1.5 with its real fused tail, the
grouped 3x3 convolutions of ResNeXt-50 32x4d, DCGAN's four transposed
convolutions at batch 1 and 64, and 3D-ResNet50's stem and 3x3x3 shape, each
as ONE kernel under every kernel-variant backend the benchmark registers that
runs it, against the oracle at the per-operator bar (1e-4, tensor-normalised
and element-wise).  The shape lists are written out here; CPU tests check them
against the model builders.
"""
import numpy as np
import pytest

import workloads as wl
from workloads.patterns import P, W
from parity_util import run_group

BR, BAR, B_, BT = ("bias_add", "relu"), ("bias_add", "add", "relu"), ("bias_add",), ("bias_add", "tanh")

# cin, cout, input height = width, filter, stride, pad, fused tail.  The residual add + relu of a block with a
# projection shortcut can ride on either of its two producers, so projections appear with both tails.
RESNET50_CONVS = [
    (3, 64, 224, 7, 2, 3, BR),                                       # stem
    (64, 64, 56, 1, 1, 0, BR), (64, 64, 56, 3, 1, 1, BR), (64, 256, 56, 1, 1, 0, BAR), (64, 256, 56, 1, 1, 0, B_),
    (256, 64, 56, 1, 1, 0, BR),
    (256, 128, 56, 1, 1, 0, BR), (128, 128, 56, 3, 2, 1, BR), (128, 512, 28, 1, 1, 0, BAR), (256, 512, 56, 1, 2, 0, B_), (256, 512, 56, 1, 2, 0, BAR),
    (512, 128, 28, 1, 1, 0, BR), (128, 128, 28, 3, 1, 1, BR),
    (512, 256, 28, 1, 1, 0, BR), (256, 256, 28, 3, 2, 1, BR), (256, 1024, 14, 1, 1, 0, BAR), (512, 1024, 28, 1, 2, 0, B_), (512, 1024, 28, 1, 2, 0, BAR),
    (1024, 256, 14, 1, 1, 0, BR), (256, 256, 14, 3, 1, 1, BR),
    (1024, 512, 14, 1, 1, 0, BR), (512, 512, 14, 3, 2, 1, BR), (512, 2048, 7, 1, 1, 0, BAR), (1024, 2048, 14, 1, 2, 0, B_), (1024, 2048, 14, 1, 2, 0, BAR),
    (2048, 512, 7, 1, 1, 0, BR), (512, 512, 7, 3, 1, 1, BR),
]
# channels (in = out), input size, stride; 32 groups, 3x3, pad 1, bias + relu
RESNEXT50_GROUPED = [(128, 56, 1), (256, 56, 2), (256, 28, 1), (512, 28, 2), (512, 14, 1), (1024, 14, 2), (1024, 7, 1)]
# cin, cout, input size, tail; 4x4 filter, stride 2, pad 1
DCGAN_CONVT = [(512, 256, 4, BR), (256, 128, 8, BR), (128, 64, 16, BR), (64, 3, 32, BT)]
# cin, cout, (d, h, w), filter, stride, pad, tail
RESNET3D_CONVS = [(3, 64, (16, 112, 112), (7, 7, 7), (1, 2, 2), (3, 3, 3), BR),
                  (64, 64, (8, 28, 28), (3, 3, 3), (1, 1, 1), (1, 1, 1), BR),
                  (128, 128, (8, 28, 28), (3, 3, 3), (2, 2, 2), (1, 1, 1), BR)]


def tail_pattern(anchor, tail):
    p = anchor
    for op in tail:
        p = P(op, p, W) if op in ("bias_add", "add") else P(op, p)
    return p


def _f32(r, *shape, scale=1.0):
    return (r.standard_normal(shape) * scale).astype(np.float32)


def conv_graph(kind, r, batch, cin, cout, spatial, k, s, p, tail, groups=1, wscale=None):
    """One convolution of `kind` with its fused tail as a graph of its own; He-normal weights unless
    wscale is given."""
    d = wl.GraphDesc(f"{kind}_{cin}_{cout}_{spatial[-1]}")
    x = d.input(_f32(r, batch, cin, *spatial))
    if kind == "conv2d_transpose":
        w = d.const(_f32(r, cin, cout, *k, scale=wscale))
        y = d.op(kind, [x, w], stride=s, pad=p)
        out_sp = tuple((n - 1) * ss - 2 * pp + kk for n, ss, pp, kk in zip(spatial, s, p, k))
    else:
        fan = cin // groups * int(np.prod(k))
        w = d.const(_f32(r, cout, cin // groups, *k, scale=wscale or (2.0 / fan) ** 0.5))
        y = d.op(kind, [x, w], stride=s, pad=p, **({"groups": groups} if kind == "conv2d" else {}))
        out_sp = tuple((n + 2 * pp - kk) // ss + 1 for n, ss, pp, kk in zip(spatial, s, p, k))
    for op in tail:
        if op == "bias_add":
            y = d.op("bias_add", [y, d.const(r.uniform(-0.1, 0.1, cout).astype(np.float32))], axis=1)
        elif op == "add":
            y = d.op("add", [y, d.input(_f32(r, batch, cout, *out_sp))])
        else:
            y = d.op(op, [y])
    d.mark_output(y)
    return d, tail_pattern(P(kind, W, W), tail)


def under_every_variant(d, pat, what, must_run, extra=()):
    """Runs the single group under each backend of the benchmark's registry; returns {backend: kernel name}."""
    import bench
    ref, names = None, {}
    for be in tuple(bench.VARIANTS) + tuple(extra):
        name, ref = run_group(d, be, pat, ref=ref, what=what)
        if name is not None:
            names[be] = name
    for be in must_run:
        assert be in names, (what, be, "refused the shape")
    return names


@pytest.mark.gpu
@pytest.mark.parametrize("ci", range(len(RESNET50_CONVS)))
def test_resnet50_convolutions_at_their_real_shapes(ci):
    cin, cout, h, k, s, p, tail = RESNET50_CONVS[ci]
    r = np.random.default_rng([101, ci])
    d, pat = conv_graph("conv2d", r, 1, cin, cout, (h, h), (k, k), (s, s), (p, p), tail)
    import bench
    names = under_every_variant(d, pat, RESNET50_CONVS[ci], must_run=bench.VARIANTS, extra=("direct",))
    assert names["igemm_r32"].startswith("conv_rf32") and names["igemm_r16"].startswith("conv_rf16"), names
    # the three never-split variants stay in one launch: no split-K suffix
    for be in ("igemm_s_nk", "igemm_s8_nk", "igemm_s16_nk"):
        assert "_k" not in names[be].replace("_kw", ""), names


@pytest.mark.gpu
@pytest.mark.parametrize("ci", range(len(RESNEXT50_GROUPED)))
def test_resnext50_grouped_convolutions_at_their_real_shapes(ci):
    c, h, s = RESNEXT50_GROUPED[ci]
    r = np.random.default_rng([102, ci])
    d, pat = conv_graph("conv2d", r, 1, c, c, (h, h), (3, 3), (s, s), (1, 1), BR, groups=32)
    names = under_every_variant(d, pat, RESNEXT50_GROUPED[ci], must_run=("igemm_r32", "igemm_r16"), extra=("direct",))
    import bench
    register_fed = {b for b in bench.VARIANTS if b.startswith("igemm_r")}
    assert set(names) == register_fed | {"direct"}, names        # the LDS-tiled kernels take one group only


@pytest.mark.gpu
@pytest.mark.parametrize("batch", [1, 64])
@pytest.mark.parametrize("ci", range(len(DCGAN_CONVT)))
def test_dcgan_transposed_convolutions_at_their_real_shapes(ci, batch):
    cin, cout, h, tail = DCGAN_CONVT[ci]
    r = np.random.default_rng([103, ci, batch])
    d, pat = conv_graph("conv2d_transpose", r, batch, cin, cout, (h, h), (4, 4), (2, 2), (1, 1), tail, wscale=0.02)
    import bench
    names = under_every_variant(d, pat, (DCGAN_CONVT[ci], batch), must_run=bench.VARIANTS)
    assert names["igemm_r32"].startswith("convt_rf32") and names["igemm_r16"].startswith("convt_rf16"), names


@pytest.mark.gpu
@pytest.mark.parametrize("ci", range(len(RESNET3D_CONVS)))
def test_resnet3d_convolutions_at_their_real_shapes(ci):
    cin, cout, sp, k, s, p, tail = RESNET3D_CONVS[ci]
    r = np.random.default_rng([104, ci])
    d, pat = conv_graph("conv3d", r, 1, cin, cout, sp, k, s, p, tail)
    names = under_every_variant(d, pat, RESNET3D_CONVS[ci], must_run=("igemm_r32", "igemm_r16"))
    assert all(n.startswith("conv3d_rf") for n in names.values()), names


# ---- the lists above against the model builders (no GPU) ---------------------------------------------------
def _convs_of(desc, kind):
    """Every `kind` node of a model with its shapes and its elementwise tail (followed while the
    value has one consumer and that consumer is bias_add / add / relu / tanh taking it)."""
    from oracle.graph import Graph
    import paper_2111_00655_amd as clg
    from paper_2111_00655_amd import binding as B
    s = clg.Session(desc, [], device=None)
    g = Graph(desc)
    found = set()
    for v, nd in enumerate(desc.nodes):
        if nd["kind"] != kind:
            continue
        xs = B.clg_graph_node_shape(s.graph, nd["inputs"][0])[1]
        ws = B.clg_graph_node_shape(s.graph, nd["inputs"][1])[1]
        tail, cur = [], v
        while len(g.consumers[cur]) == 1 and desc.nodes[g.consumers[cur][0]]["kind"] in ("bias_add", "add", "relu", "tanh") \
                and cur not in desc.outputs:
            cur = g.consumers[cur][0]
            tail.append(desc.nodes[cur]["kind"])
        found.add((xs, ws, tuple(nd["attrs"]["stride"]), tuple(nd["attrs"]["pad"]), nd["attrs"].get("groups", 1), tuple(tail)))
    s.close()
    return found


def test_the_resnet50_list_is_every_distinct_convolution_of_the_model():
    got = _convs_of(wl.resnet50(0), "conv2d")      # with each convolution's longest tail
    want = {((1, cin, h, h), (cout, cin, k, k), (s, s), (p, p), 1, tail) for cin, cout, h, k, s, p, tail in RESNET50_CONVS}
    assert got <= want
    assert {c[:5] for c in got} == {c[:5] for c in want} and len({c[:5] for c in want}) == 23      # 23 distinct shapes
    longest = {c[:5]: c[5] for c in got}
    assert all(c[5] == longest[c[:5]][:len(c[5])] for c in want)       # the shorter tails are prefixes of the real one


def test_the_resnext50_list_is_every_grouped_convolution_of_the_model():
    got = {c for c in _convs_of(wl.resnext50(0), "conv2d") if c[4] > 1}
    want = {((1, c, h, h), (c, c // 32, 3, 3), (s, s), (1, 1), 32, BR) for c, h, s in RESNEXT50_GROUPED}
    assert got == want


def test_the_dcgan_and_resnet3d_lists_come_from_the_models():
    for batch in (1, 64):
        got = _convs_of(wl.dcgan(0, batch=batch), "conv2d_transpose")
        want = {((batch, cin, h, h), (cin, cout, 4, 4), (2, 2), (1, 1), 1, tail) for cin, cout, h, tail in DCGAN_CONVT}
        assert got == want
    got = _convs_of(wl.resnet3d_50(0), "conv3d")
    for cin, cout, sp, k, s, p, tail in RESNET3D_CONVS:
        assert ((1, cin) + sp, (cout, cin) + k, s, p, 1, tail) in got
