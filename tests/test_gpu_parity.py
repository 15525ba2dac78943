"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Bars (fp32): max|gpu - ref| / max|ref| <= 1e-4 per
fused op and <= 1e-3 on a network's final outputs; placements bit-exact.
"""
import numpy as np
import pytest

import workloads as wl
from workloads.patterns import P, W
import paper_2111_00655_amd as clg
from paper_2111_00655_amd import binding as B
from oracle.graph import Graph, norm_err
from oracle.match import enumerate_matches
from oracle import search

pytestmark = pytest.mark.gpu

OP_TOL = 1e-4
NET_TOL = 1e-3
IGEMM = ("igemm", "igemm_s", "igemm_s8", "igemm_s16", "igemm_m", "igemm_l")
RF = ("igemm_r32", "igemm_r16")          # register-fed convolution kernels (packed weights)
RFW = ("igemm_r32_w4", "igemm_r16_w8")   # the same with a bound on the K-waves per workgroup (several chunks per wave)
RFD = RF + RFW + ("igemm_r16x2_w4", "igemm_r16x2_w8")     # ... and the dense kernels with two tiles per wave


def rng_for(*key):
    return np.random.default_rng([int(k) for k in key])


def f32(r, *shape, scale=1.0):
    return (r.standard_normal(shape) * scale).astype(np.float32)


def run_single_group(desc, backend, pattern, tol=OP_TOL, extra=()):
    """The graph's operators form exactly one match of `pattern`: run it as one
    kernel of `backend` and compare with the oracle."""
    reg = [(backend, pattern)] + list(extra)
    s = clg.Session(desc, reg, device=0)
    ms = s.match()
    full = [i for i, m in enumerate(ms) if m.pattern == 0 and m.n_nodes == len(desc.op_nodes())]
    assert len(full) == 1, [(m.pattern, m.n_nodes) for m in ms]
    plan = s.compile(full)
    assert plan.n_kernels == 1
    got = plan.run()
    ref = Graph(desc).run()
    err = max(norm_err(a, b) for a, b in zip(got, ref))
    again = plan.run()
    assert all(np.array_equal(a, b) for a, b in zip(got, again)), "not deterministic"
    name = plan.kernels()[0]["name"]
    plan.destroy()
    s.close()
    assert err <= tol, (name, err)
    return name, err


def tail_pattern(anchor, tail):
    p = anchor
    for op in tail:
        p = P(op, p, W) if op in ("bias_add", "add") else P(op, p)
    return p


# ------------------------------------------------------------------ convolution
CONV_CASES = [
    # cin, cout, h, w, k, stride, pad, tail
    (3, 16, 32, 32, 3, 1, 1, ("bias_add", "relu")),            # tiny-CNN layer 1 (K = 27)
    (16, 32, 32, 32, 3, 1, 1, ("bias_add", "add", "relu")),
    (3, 64, 56, 56, 7, 2, 3, ("bias_add", "relu")),            # stem shape class (K = 147), reduced image
    (64, 64, 28, 28, 1, 1, 0, ("bias_add", "relu")),           # 1x1: plain GEMM path
    (64, 96, 14, 14, 1, 2, 0, ("bias_add",)),                  # 1x1 stride 2 projection
    (32, 48, 28, 28, 3, 2, 1, ("bias_add", "relu")),           # 3x3 stride 2
    (40, 72, 9, 7, 3, 1, 1, ()),                               # ragged M, N, K; no epilogue
    (128, 130, 7, 7, 3, 1, 1, ("bias_add", "add")),            # N = 49 < one tile
    (512, 64, 7, 7, 1, 1, 0, ("bias_add", "add", "relu")),     # long K, small M*N: split-K
    (256, 40, 14, 14, 3, 2, 1, ("bias_add", "relu")),          # long K 3x3 stride 2: sixteen K-waves, several chunks each
    (5, 10, 8, 8, 5, 1, 2, ("bias_add", "tanh")),              # odd channel count, 5x5 filter
    (1024, 48, 6, 6, 1, 1, 0, ("bias_add",)),                  # 1x1 with K = 1024: two chunks per wave
]


def conv_desc(case, seed, batch=1, groups=1):
    cin, cout, h, w, k, s, p, tail = case
    r = rng_for(seed, cin, cout, h, k)
    d = wl.GraphDesc("conv_case")
    x = d.input(f32(r, batch, cin, h, w))
    wt = d.const(f32(r, cout, cin // groups, k, k, scale=(2.0 / (cin // groups * k * k)) ** 0.5))
    y = d.op("conv2d", [x, wt], stride=(s, s), pad=(p, p), groups=groups)
    ho, wo = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
    for op in tail:
        if op == "bias_add":
            y = d.op("bias_add", [y, d.const(f32(r, cout))], axis=1)
        elif op == "add":
            y = d.op("add", [y, d.input(f32(r, batch, cout, ho, wo))])
        else:
            y = d.op(op, [y])
    d.mark_output(y)
    return d, tail_pattern(P("conv2d", W, W), tail)


@pytest.mark.parametrize("backend", IGEMM + RF + RFW + ("direct",))
@pytest.mark.parametrize("ci", range(len(CONV_CASES)))
def test_conv2d_fused(ci, backend):
    d, pat = conv_desc(CONV_CASES[ci], 10 + ci)
    name, _ = run_single_group(d, backend, pat)
    if backend in RF + RFW:
        assert name.startswith("conv_rf"), name


def test_conv2d_batched_igemm():
    d, pat = conv_desc((8, 24, 12, 10, 3, 1, 1, ("bias_add", "relu")), 77, batch=3)
    run_single_group(d, "igemm", pat)
    d, pat = conv_desc((16, 24, 10, 10, 1, 1, 0, ("bias_add", "relu")), 78, batch=3)
    run_single_group(d, "igemm_m", pat)


@pytest.mark.parametrize("backend", RF)
def test_conv2d_batched_register_fed(backend):
    for seed, case in enumerate([(8, 24, 12, 10, 3, 1, 1, ("bias_add", "relu")), (16, 24, 10, 10, 1, 2, 0, ("bias_add", "add")),
                                 (3, 20, 17, 13, 7, 2, 3, ("bias_add", "relu"))]):
        d, pat = conv_desc(case, 80 + seed, batch=3)
        run_single_group(d, backend, pat)


@pytest.mark.parametrize("case", [(128, 128, 28, 28, 3, 1, 1, 32), (256, 256, 14, 14, 3, 2, 1, 32),
                                  (64, 64, 9, 9, 3, 1, 1, 16), (12, 18, 8, 8, 3, 1, 1, 6)])
def test_grouped_conv_direct(case):
    cin, cout, h, w, k, s, p, g = case
    d, pat = conv_desc((cin, cout, h, w, k, s, p, ("bias_add", "relu")), 5, groups=g)
    run_single_group(d, "direct", pat)


@pytest.mark.parametrize("backend", RF)
@pytest.mark.parametrize("case", [(128, 128, 28, 28, 3, 1, 1, 32), (256, 256, 14, 14, 3, 2, 1, 32), (512, 512, 7, 7, 3, 1, 1, 32),
                                  (64, 64, 9, 9, 3, 1, 1, 16), (24, 48, 8, 8, 3, 1, 1, 6), (32, 32, 6, 6, 1, 1, 0, 2),
                                  (64, 128, 7, 7, 5, 1, 2, 2)])
def test_grouped_conv_register_fed(case, backend):
    """Grouped convolution on the MFMA kernels: m-tiles that span several groups
    (4 channels per group), exactly one, or a part of one (64 output channels per group)."""
    cin, cout, h, w, k, s, p, g = case
    d, pat = conv_desc((cin, cout, h, w, k, s, p, ("bias_add", "relu")), 6, groups=g, batch=2 if cin == 24 else 1)
    name, _ = run_single_group(d, backend, pat)
    assert name.startswith("conv_rf"), name


@pytest.mark.parametrize("backend", ("direct",) + RF)
@pytest.mark.parametrize("case", [(44, 44, 28, 28, 3, 1, 1, 44), (44, 44, 28, 28, 5, 2, 2, 44), (22, 22, 15, 15, 7, 2, 3, 22),
                                  (176, 176, 7, 7, 5, 1, 2, 176), (11, 11, 56, 56, 7, 2, 3, 11)])
def test_depthwise_conv(case, backend):
    """One input channel per group (the depthwise half of a separable convolution), NasNet-A's sizes."""
    cin, cout, h, w, k, s, p, g = case
    d, pat = conv_desc((cin, cout, h, w, k, s, p, ()), 8, groups=g)
    run_single_group(d, backend, pat)


CONV3D_CASES = [
    # batch, cin, cout, d, h, w, kernel, stride, pad, tail
    (1, 16, 32, 4, 9, 9, (3, 3, 3), (1, 1, 1), (1, 1, 1), ("bias_add", "relu")),
    (1, 16, 24, 6, 10, 8, (3, 3, 3), (2, 2, 2), (1, 1, 1), ("bias_add", "add", "relu")),
    (2, 8, 40, 5, 7, 7, (3, 3, 3), (1, 1, 1), (1, 1, 1), ("bias_add",)),           # batch 2, ragged pixels
    (1, 3, 16, 6, 20, 20, (7, 7, 7), (1, 2, 2), (3, 3, 3), ("bias_add", "relu")),     # the stem's shape class
    (1, 64, 48, 4, 7, 7, (1, 1, 1), (1, 1, 1), (0, 0, 0), ("bias_add", "relu")),      # 1x1x1
    (1, 64, 128, 8, 14, 14, (1, 1, 1), (2, 2, 2), (0, 0, 0), ("bias_add",)),          # strided 1x1x1 projection
    (2, 32, 16, 3, 6, 5, (1, 1, 1), (1, 1, 1), (0, 0, 0), ("bias_add", "add", "relu")),
    (1, 6, 10, 4, 6, 6, (3, 1, 1), (1, 1, 1), (1, 0, 0), ()),                          # depth taps only
    (1, 8, 12, 5, 8, 8, (1, 3, 3), (2, 1, 1), (0, 1, 1), ("bias_add",)),               # one depth tap, depth stride 2
    (1, 5, 7, 4, 6, 6, (2, 3, 2), (1, 2, 1), (1, 1, 0), ()),                           # odd everything
]


@pytest.mark.parametrize("backend", RF)
@pytest.mark.parametrize("case", CONV3D_CASES)
def test_conv3d_register_fed(case, backend):
    """3-D convolution (3D-ResNet50, paper Sec. 5.1): one grid slice per output depth, depth taps folded
    into the channel index of the 2-D kernels."""
    batch, cin, cout, dd, h, w, k, s, p, tail = case
    r = rng_for(31, cin, cout, dd, h)
    d = wl.GraphDesc("conv3d_case")
    x = d.input(f32(r, batch, cin, dd, h, w))
    wt = d.const(f32(r, cout, cin, *k, scale=1.0 / np.sqrt(cin * k[0] * k[1] * k[2])))
    y = d.op("conv3d", [x, wt], stride=s, pad=p)
    od = [(n + 2 * pp - kk) // ss + 1 for n, pp, kk, ss in zip((dd, h, w), p, k, s)]
    for op in tail:
        if op == "bias_add":
            y = d.op("bias_add", [y, d.const(f32(r, cout))], axis=1)
        elif op == "add":
            y = d.op("add", [y, d.input(f32(r, batch, cout, *od))])
        else:
            y = d.op(op, [y])
    d.mark_output(y)
    name, _ = run_single_group(d, backend, tail_pattern(P("conv3d", W, W), tail))
    assert name.startswith("conv3d_rf"), name


RF_SPLIT = ("igemm_r16_sk", "igemm_r16_sk_w4", "igemm_r32_sk")
SPLIT_K_CASES = [
    # kind, batch, cin, cout, spatial, kernel, stride, pad, tail: long reductions over few output tiles
    ("conv3d", 1, 512, 64, (2, 4, 4), (3, 3, 3), (1, 1, 1), (1, 1, 1), ("bias_add", "relu")),        # 3D-ResNet50's last stage, narrower
    ("conv3d", 1, 96, 40, (3, 7, 7), (3, 3, 3), (2, 2, 2), (1, 1, 1), ("bias_add", "add", "relu")),
    ("conv2d", 1, 512, 96, (7, 7), (3, 3), (1, 1), (1, 1), ("bias_add", "relu")),
    ("conv2d", 2, 1024, 48, (4, 4), (1, 1), (1, 1), (0, 0), ("bias_add", "add")),
    ("conv2d", 1, 200, 24, (5, 6), (5, 5), (1, 1), (2, 2), ("bias_add",)),                           # any-filter path
    ("conv2d", 1, 64, 64, (56, 56), (3, 3), (1, 1), (1, 1), ("bias_add", "relu")),                   # a full grid: no split
]


@pytest.mark.parametrize("backend", RF_SPLIT)
@pytest.mark.parametrize("ci", range(len(SPLIT_K_CASES)))
def test_register_fed_convolution_with_k_split_across_workgroups(ci, backend):
    """The register-fed kernels with the reduction cut across workgroups where the grid would otherwise leave most
    of the chip idle: partial tiles in scratch memory, added in slice order by the reduction kernel with the tail."""
    from test_gpu_real_shapes import conv_graph
    from parity_util import run_group
    kind, batch, cin, cout, sp, k, st, pd, tail = SPLIT_K_CASES[ci]
    r = rng_for(33, ci)
    d, pat = conv_graph(kind, r, batch, cin, cout, sp, k, st, pd, tail)
    name, _ = run_group(d, backend, pat, what=(SPLIT_K_CASES[ci], backend))
    assert "_rf" in name, name
    split = "_k" in name.split("_w")[-1]
    assert not (split and ci == 5), name
    assert split or ci == 5 or backend != "igemm_r16_sk_w4", name      # with four K-waves every long reduction here is split


def test_pools_3d():
    r = rng_for(32)
    d = wl.GraphDesc("maxpool3d")
    d.mark_output(d.op("max_pool3d", [d.input(f32(r, 2, 5, 6, 15, 13))], kernel=(3, 3, 3), stride=(2, 2, 2), pad=(1, 1, 1)))
    run_single_group(d, "direct", P("max_pool3d", W), tol=0.0)
    d = wl.GraphDesc("maxpool3d_b")
    d.mark_output(d.op("max_pool3d", [d.input(f32(r, 1, 3, 4, 7, 6))], kernel=(1, 3, 2), stride=(1, 2, 2), pad=(0, 1, 0)))
    run_single_group(d, "direct", P("max_pool3d", W), tol=0.0)
    d = wl.GraphDesc("gap3d")
    d.mark_output(d.op("global_avg_pool3d", [d.input(f32(r, 2, 37, 2, 4, 4))]))
    run_single_group(d, "direct", P("global_avg_pool3d", W), tol=1e-6)


def test_resnet3d_whole_path():
    """3D-ResNet50 at reduced size through profile, search, compile, execute."""
    desc = wl.resnet3d_50(0, frames=4, image=32, width=16, blocks=(2, 1, 1), classes=10)
    reg = wl.default_registry(("igemm_s8", "igemm_r32", "igemm_r16"))
    s, g, oms = _session_and_oracle(desc, reg)
    costs = s.profile(B.ProfileOpts(warmup=2, batches=2, min_batch_us=30, max_launches=30))
    got_search = s.search(costs, 0)
    assert got_search == search.dp(g, reg, oms, costs, 0)
    plan = s.compile(got_search[1])
    got = plan.run()
    ref = g.run()
    assert got[0].shape == (1, 10)
    assert max(norm_err(a, b) for a, b in zip(got, ref)) <= NET_TOL
    plan.destroy()
    s.close()


ATT_CASES = [
    # heads, Sq, Sk, d, scale?, merged store?
    (12, 128, 128, 64, True, True),        # BERT-base
    (3, 50, 70, 32, False, False),         # ragged rows and keys, no scale, heads kept apart
    (2, 16, 512, 128, True, True),         # the most keys and the largest head the kernel takes
    (1, 1, 5, 32, True, False),            # a single query
    (5, 33, 17, 64, True, True),
    (2, 200, 129, 32, True, False),
]


@pytest.mark.parametrize("case", ATT_CASES)
def test_attention_in_one_kernel(case):
    """softmax(scale q k^T) v per head as one kernel against the oracle's operator-by-operator result."""
    heads, sq, sk, dd, scaled, merged = case
    r = rng_for(41, heads, sq, sk, dd)
    d = wl.GraphDesc("attention_case")
    q, k, v = d.input(f32(r, heads, sq, dd)), d.input(f32(r, heads, sk, dd)), d.input(f32(r, heads, sk, dd))
    y = d.op("batch_matmul", [q, k], transpose_b=True)
    pat = P("batch_matmul", W, W)
    if scaled:
        y = d.op("mul_scalar", [y], scalar=float(1.0 / np.sqrt(dd)))
        pat = P("mul_scalar", pat)
    y = d.op("softmax", [y])
    y = d.op("batch_matmul", [y, v], transpose_b=False)
    pat = P("batch_matmul", P("softmax", pat), W)
    if merged:
        y = d.op("transpose", [y], dims=(1, 0, 2))
        y = d.op("reshape", [y], dims=(sq, heads * dd))
        pat = P("reshape", P("transpose", pat))
    d.mark_output(y)
    name, _ = run_single_group(d, "attention", pat)
    assert name == f"attention_d{dd}" + ("_merge" if merged else ""), name


def test_attention_refuses_what_it_cannot_run():
    r = rng_for(42)
    d = wl.GraphDesc("att_small_head")
    q, k, v = d.input(f32(r, 2, 8, 8)), d.input(f32(r, 2, 8, 8)), d.input(f32(r, 2, 8, 8))
    y = d.op("batch_matmul", [d.op("softmax", [d.op("batch_matmul", [q, k], transpose_b=True)]), v], transpose_b=False)
    d.mark_output(y)
    s = clg.Session(d, [("attention", P("batch_matmul", P("softmax", P("batch_matmul", W, W)), W))], device=0)
    assert len(s.match()) == 1
    assert B.clg_profile_match(s.ctx, s.graph, 0) >= B.COST_INF      # head size 8
    with pytest.raises(clg.ClgError) as e:
        s.compile([0])
    assert e.value.status == "NO_KERNEL"
    s.close()
    with pytest.raises(clg.ClgError):                                  # a lone product is not this family's
        clg.Session(d, [("attention", P("batch_matmul", W, W))], device=0)


SEP_CASES = [
    # batch, c, cout, h, w, k (0 = no depthwise stage), stride, pre-relu, tail
    (1, 44, 44, 28, 28, 3, 1, True, ("bias_add",)),
    (1, 44, 44, 28, 28, 5, 2, True, ("bias_add", "relu")),
    (1, 22, 22, 15, 13, 7, 2, True, ("bias_add", "add")),
    (1, 176, 176, 7, 7, 5, 1, True, ("bias_add", "add", "relu")),
    (1, 11, 11, 56, 56, 7, 2, False, ("bias_add",)),
    (2, 88, 88, 14, 14, 3, 1, True, ()),
    (3, 20, 50, 9, 9, 3, 1, False, ("bias_add",)),            # Cout != C, ragged everything, batch 3
    (1, 1056, 176, 7, 7, 0, 1, True, ("bias_add",)),          # relu + 1x1 over 1056 channels (LDS > 64 KB)
    (1, 264, 88, 28, 28, 0, 2, True, ("bias_add",)),          # relu + strided 1x1
    (1, 32, 11, 112, 112, 0, 1, True, ("bias_add", "relu")),  # many pixels, one m-tile
    (2, 7, 5, 6, 5, 0, 1, True, ()),
]


@pytest.mark.parametrize("case", SEP_CASES)
def test_separable_conv_in_one_kernel(case):
    """[relu] -> depthwise -> 1x1 -> tail (or relu -> 1x1 -> tail) as one kernel against the oracle's
    operator-by-operator result."""
    batch, c, cout, h, w, k, s, pre, tail = case
    r = rng_for(21, c, cout, h, k)
    d = wl.GraphDesc("sep_case")
    x = d.input(f32(r, batch, c, h, w))
    y = d.op("relu", [x]) if pre else x
    pat = P("relu", W) if pre else W
    if k:
        wd = d.const(f32(r, c, 1, k, k, scale=1.0 / k))
        y = d.op("conv2d", [y, wd], stride=(s, s), pad=(k // 2, k // 2), groups=c)
        pat = P("conv2d", pat, W)
    wp = d.const(f32(r, cout, c, 1, 1, scale=1.0 / np.sqrt(c)))
    y = d.op("conv2d", [y, wp], stride=(1, 1) if k else (s, s), pad=(0, 0), groups=1)
    pat = P("conv2d", pat, W)
    for op in tail:
        if op == "bias_add":
            y = d.op("bias_add", [y, d.const(f32(r, cout))], axis=1)
        elif op == "add":
            ho, wo = ((h + 2 * (k // 2) - k) // s + 1, (w + 2 * (k // 2) - k) // s + 1) if k else ((h - 1) // s + 1, (w - 1) // s + 1)
            y = d.op("add", [y, d.input(f32(r, batch, cout, ho, wo))])
        else:
            y = d.op(op, [y])
    d.mark_output(y)
    name, _ = run_single_group(d, "sepconv", tail_pattern(pat, tail))
    assert ("sepconv" in name) == bool(k) and name.startswith("relu_") == pre, name


@pytest.mark.parametrize("case", [(1, 44, 28, 28, 3, 1, ()), (1, 22, 15, 13, 7, 2, ("bias_add",)), (2, 176, 7, 7, 5, 1, ("bias_add", "add")),
                                  (1, 11, 56, 56, 5, 2, ("bias_add", "relu")), (3, 5, 9, 6, 3, 1, ("tanh",))])
def test_relu_then_depthwise_conv(case):
    """relu -> depthwise convolution -> tail as one launch of the depthwise kernel (the first half of a
    separable convolution where the search keeps its 1x1 half on another kernel)."""
    batch, c, h, w, k, s, tail = case
    r = rng_for(23, c, h, k)
    d = wl.GraphDesc("relu_dw")
    x = d.input(f32(r, batch, c, h, w))
    y = d.op("conv2d", [d.op("relu", [x]), d.const(f32(r, c, 1, k, k, scale=1.0 / k))], stride=(s, s), pad=(k // 2, k // 2), groups=c)
    ho, wo = (h + 2 * (k // 2) - k) // s + 1, (w + 2 * (k // 2) - k) // s + 1
    for op in tail:
        if op == "bias_add":
            y = d.op("bias_add", [y, d.const(f32(r, c))], axis=1)
        elif op == "add":
            y = d.op("add", [y, d.input(f32(r, batch, c, ho, wo))])
        else:
            y = d.op(op, [y])
    d.mark_output(y)
    name, _ = run_single_group(d, "sepconv", tail_pattern(P("conv2d", P("relu", W), W), tail))
    assert name.startswith(f"relu_dwconv{k}"), name


def test_sepconv_refuses_what_it_cannot_run():
    r = rng_for(22)
    d = wl.GraphDesc("not_sep")
    x = d.input(f32(r, 1, 8, 6, 6))
    y = d.op("conv2d", [d.op("relu", [x]), d.const(f32(r, 8, 8, 3, 3))], stride=(1, 1), pad=(1, 1), groups=1)
    d.mark_output(y)
    s = clg.Session(d, [("sepconv", P("conv2d", P("relu", W), W))], device=0)
    assert len(s.match()) == 1
    assert B.clg_profile_match(s.ctx, s.graph, 0) >= B.COST_INF      # a 3x3 convolution is not the 1x1 stage
    with pytest.raises(clg.ClgError) as e:
        s.compile([0])
    assert e.value.status == "NO_KERNEL"
    s.close()
    with pytest.raises(clg.ClgError):                                  # a lone convolution is not this family's
        clg.Session(d, [("sepconv", P("conv2d", W, W))], device=0)


def test_grouped_conv_is_refused_by_igemm():
    d, pat = conv_desc((8, 8, 6, 6, 3, 1, 1, ()), 5, groups=2)
    s = clg.Session(d, [("igemm", pat)], device=0)
    ms = s.match()
    assert len(ms) == 1
    assert B.clg_profile_match(s.ctx, s.graph, 0) >= B.COST_INF
    with pytest.raises(clg.ClgError) as e:
        s.compile([0])
    assert e.value.status == "NO_KERNEL"
    s.close()


# ------------------------------------------------------- transposed convolution
def convt_desc(case, k=4, stride=2, pad=1):
    batch, cin, cout, h, tail = case
    r = rng_for(3, cin, cout, h, k)
    d = wl.GraphDesc("convt_case")
    x = d.input(f32(r, batch, cin, h, h))
    wt = d.const(f32(r, cin, cout, k, k, scale=0.05))
    y = d.op("conv2d_transpose", [x, wt], stride=(stride, stride), pad=(pad, pad))
    for op in tail:
        y = d.op("bias_add", [y, d.const(f32(r, cout))], axis=1) if op == "bias_add" else d.op(op, [y])
    d.mark_output(y)
    return d, tail_pattern(P("conv2d_transpose", W, W), tail)


@pytest.mark.parametrize("backend", IGEMM + RF)
@pytest.mark.parametrize("case", [(1, 64, 32, 4, ("bias_add", "relu")), (2, 32, 16, 8, ("bias_add", "relu")),
                                  (3, 16, 3, 16, ("bias_add", "tanh")), (1, 24, 40, 5, ()),
                                  (2, 7, 5, 6, ("bias_add", "relu")),
                                  # few output channels: the layer as one 3x3 convolution with (channel, phase) rows
                                  (2, 8, 4, 5, ("bias_add", "relu")), (1, 12, 1, 7, ()), (5, 64, 2, 9, ("bias_add", "tanh"))])
def test_conv2d_transpose_fused(case, backend):
    d, pat = convt_desc(case)
    name, _ = run_single_group(d, backend, pat)
    if backend in RF:
        assert name.startswith("convt_rf"), name


@pytest.mark.parametrize("backend", RF)
@pytest.mark.parametrize("geom", [(6, 3, 0), (2, 2, 0), (3, 1, 1), (4, 1, 0)])
def test_conv2d_transpose_other_geometries(geom, backend):
    """Kernel sizes, strides and paddings other than k4 s2 p1: three phases per axis,
    2x2 without overlap, stride 1 (a single phase with flipped taps)."""
    k, s, p = geom
    d, pat = convt_desc((2, 8, 12, 5, ("bias_add", "relu")), k=k, stride=s, pad=p)
    name, _ = run_single_group(d, backend, pat)
    assert name.startswith("convt_rf"), name


@pytest.mark.parametrize("geom", [(3, 2, 1), (5, 2, 2), (3, 3, 0), (5, 3, 1), (4, 2, 1), (1, 2, 0), (7, 4, 3)])
@pytest.mark.parametrize("case", [(2, 8, 12, 5, ("bias_add", "relu")), (1, 33, 3, 9, ("bias_add", "tanh")), (3, 5, 70, 4, ())])
def test_conv2d_transpose_of_any_geometry_in_the_direct_kernel(case, geom):
    """Filter sizes the stride does not divide have no phase decomposition: the MFMA backends refuse
    them and the direct kernel runs them (and every other geometry)."""
    k, s, p = geom
    d, pat = convt_desc(case, k=k, stride=s, pad=p)
    name, ref = run_single_group(d, "direct", pat)
    assert name == "direct_convt", name
    if k % s:
        for backend in ("igemm", "igemm_r16"):
            s_ = clg.Session(d, [(backend, pat)], device=0)
            with pytest.raises(clg.ClgError) as e:
                s_.compile([i for i, m in enumerate(s_.match()) if m.n_nodes == len(d.op_nodes())])
            assert e.value.status == "NO_KERNEL"
            s_.close()


# ------------------------------------------------------------- dense / bmm
DENSE_CASES =[(128, 768, 768, ("bias_add",)), (128, 768, 3072, ("bias_add", "gelu")),
               (128, 3072, 768, ("bias_add", "add")), (1, 2048, 1000, ("bias_add",)),
               (1, 32, 10, ("bias_add",)), (5, 100, 130, ("bias_add", "relu")), (130, 27, 70, ()),
               (70, 4096, 50, ("bias_add", "relu")), (33, 48, 40, ("bias_add", "tanh")),
               (8, 2100, 37, ("bias_add", "add")), (3, 100, 8192, ("bias_add", "relu"))]
# which of them the register-fed dense kernel takes (K a multiple of 16); the others fall back to the LDS-tiled kernel
DENSE_RF = {0, 1, 2, 3, 4, 7, 8}          # (K = 2100 and K = 100 are not multiples of 8 / 16)


@pytest.mark.parametrize("backend", IGEMM + RFD)
@pytest.mark.parametrize("ci", range(len(DENSE_CASES)))
def test_dense_fused(ci, backend):
    m, k, n, tail = DENSE_CASES[ci]
    r = rng_for(4, m, k, n)
    d = wl.GraphDesc("dense_case")
    x = d.input(f32(r, m, k))
    y = d.op("dense", [x, d.const(f32(r, n, k, scale=k ** -0.5))])
    for op in tail:
        if op == "bias_add":
            y = d.op("bias_add", [y, d.const(f32(r, n))], axis=-1)
        elif op == "add":
            y = d.op("add", [y, d.input(f32(r, m, n))])
        else:
            y = d.op(op, [y])
    d.mark_output(y)
    name, _ = run_single_group(d, backend, tail_pattern(P("dense", W, W), tail))
    if backend in RFD:
        assert name.startswith("dense_rf") == (ci in DENSE_RF), name
        assert ("x2" in name) == (backend.startswith("igemm_r16x2") and ci in DENSE_RF), name
    else:
        assert (name == "gemv_nt") == (m <= 8 and k % 4 == 0 and k >= 512), name


@pytest.mark.parametrize("backend", ("igemm", "igemm_s", "igemm_s8", "igemm_s16") + RFD)
@pytest.mark.parametrize("case", [(128, 768, 12, 64), (70, 64, 3, 32), (5, 128, 2, 16), (33, 256, 5, 48)])
def test_dense_stored_split_into_heads(case, backend):
    """transpose(reshape(bias_add(dense))) as one kernel: [M, H*D] is stored as [H, M, D]."""
    m, k, h, dd = case
    r = rng_for(14, m, k, h)
    d = wl.GraphDesc("dense_split")
    y = d.op("dense", [d.input(f32(r, m, k)), d.const(f32(r, h * dd, k, scale=k ** -0.5))])
    y = d.op("bias_add", [y, d.const(f32(r, h * dd))], axis=-1)
    y = d.op("reshape", [y], dims=(m, h, dd))
    y = d.op("transpose", [y], dims=(1, 0, 2))
    d.mark_output(y)
    name, _ = run_single_group(d, backend, P("transpose", P("reshape", P("bias_add", P("dense", W, W), W))))
    assert "_split" in name, name


@pytest.mark.parametrize("backend", IGEMM)
@pytest.mark.parametrize("case", [(12, 128, 128, 64), (3, 70, 33, 20), (2, 33, 64, 8)])
def test_batch_matmul_stored_with_heads_merged(case, backend):
    """reshape(transpose(batch_matmul)) as one kernel: [B, M, N] is stored as [M, B*N]."""
    b, m, k, n = case
    r = rng_for(15, b, m, k, n)
    d = wl.GraphDesc("bmm_merge")
    y = d.op("batch_matmul", [d.input(f32(r, b, m, k)), d.input(f32(r, b, k, n))], transpose_b=False)
    y = d.op("transpose", [y], dims=(1, 0, 2))
    y = d.op("reshape", [y], dims=(m, b * n))
    d.mark_output(y)
    name, _ = run_single_group(d, backend, P("reshape", P("transpose", P("batch_matmul", W, W))))
    assert name.endswith("_merge") or "_merge_" in name, name


def test_permuted_store_refuses_other_layouts():
    r = rng_for(16)
    d = wl.GraphDesc("dense_bad_split")
    y = d.op("dense", [d.input(f32(r, 8, 64)), d.const(f32(r, 64, 64))])
    y = d.op("bias_add", [y, d.const(f32(r, 64))], axis=-1)
    y = d.op("reshape", [y], dims=(8, 4, 16))
    y = d.op("transpose", [y], dims=(0, 2, 1))
    d.mark_output(y)
    s = clg.Session(d, [("igemm_s", P("transpose", P("reshape", P("bias_add", P("dense", W, W), W))))], device=0)
    assert len(s.match()) == 1
    assert B.clg_profile_match(s.ctx, s.graph, 0) >= B.COST_INF
    s.close()


def test_dense_bias_relu_reshape():
    r = rng_for(8)
    d = wl.GraphDesc("dense_rs")
    y = d.op("dense", [d.input(f32(r, 2, 20)), d.const(f32(r, 64, 20))])
    y = d.op("bias_add", [y, d.const(f32(r, 64))], axis=-1)
    y = d.op("relu", [y])
    y = d.op("reshape", [y], dims=(2, 4, 4, 4))
    d.mark_output(y)
    run_single_group(d, "igemm", P("reshape", P("relu", P("bias_add", P("dense", W, W), W))))


@pytest.mark.parametrize("backend", IGEMM)
@pytest.mark.parametrize("case", [(12, 128, 128, 64, True, True), (12, 128, 64, 128, False, False),
                                  (3, 70, 33, 50, True, False), (2, 33, 70, 21, False, True)])
def test_batch_matmul(case, backend):
    b, m, n, k, tb, scale = case
    r = rng_for(6, b, m, n, k)
    d = wl.GraphDesc("bmm_case")
    a = d.input(f32(r, b, m, k))
    bm = d.input(f32(r, b, n, k) if tb else f32(r, b, k, n))
    y = d.op("batch_matmul", [a, bm], transpose_b=tb)
    pat = P("batch_matmul", W, W)
    if scale:
        y = d.op("mul_scalar", [y], scalar=0.125)
        pat = P("mul_scalar", pat)
    d.mark_output(y)
    run_single_group(d, backend, pat)


# --------------------------------------------------------------- row-wise
@pytest.mark.parametrize("shape", [(12, 128, 128), (1, 1000), (1, 10), (3, 7, 65), (2, 2100), (5, 300), (2, 2048), (3, 700)])
def test_softmax(shape):
    r = rng_for(7, *shape)
    d = wl.GraphDesc("softmax_case")
    d.mark_output(d.op("softmax", [d.input(f32(r, *shape, scale=3.0))]))
    run_single_group(d, "rowwise", P("softmax", W), tol=1e-5)
    d = wl.GraphDesc("softmax_scaled")
    y = d.op("mul_scalar", [d.input(f32(r, *shape, scale=9.0))], scalar=0.125)
    d.mark_output(d.op("softmax", [y]))
    run_single_group(d, "rowwise", P("softmax", P("mul_scalar", W)), tol=1e-5)


@pytest.mark.parametrize("shape", [(128, 768), (4, 48), (3, 2100), (1, 64), (7, 65), (2, 2048), (9, 700), (5, 257)])
def test_layer_norm(shape):
    r = rng_for(9, *shape)
    L = shape[-1]
    g, b = (1 + 0.02 * r.standard_normal(L)).astype(np.float32), f32(r, L, scale=0.02)
    d = wl.GraphDesc("ln_case")
    d.mark_output(d.op("layer_norm", [d.input(f32(r, *shape) + np.float32(0.5)), d.const(g), d.const(b)], eps=1e-12))
    run_single_group(d, "rowwise", P("layer_norm", W, W, W), tol=2e-5)
    d = wl.GraphDesc("ln_res")
    y = d.op("bias_add", [d.input(f32(r, *shape)), d.const(f32(r, L))], axis=-1)
    y = d.op("add", [y, d.input(f32(r, *shape))])
    d.mark_output(d.op("layer_norm", [y, d.const(g), d.const(b)], eps=1e-12))
    run_single_group(d, "rowwise", P("layer_norm", P("add", P("bias_add", W, W), W), W, W), tol=2e-5)


# ---------------------------------------------------------- elementwise / glue
def test_elementwise_chains():
    r = rng_for(11)
    shape = (2, 6, 5, 7)                     # numel not a multiple of 4
    for sh in (shape, (1, 8, 4, 4)):
        d = wl.GraphDesc("ew")
        y = d.op("bias_add", [d.input(f32(r, *sh)), d.const(f32(r, sh[1]))], axis=1)
        y = d.op("add", [y, d.input(f32(r, *sh))])
        d.mark_output(d.op("relu", [y]))
        run_single_group(d, "eltwise", P("relu", P("add", P("bias_add", W, W), W)), tol=1e-6)
    for op in ("relu", "gelu", "tanh"):
        d = wl.GraphDesc(op)
        d.mark_output(d.op(op, [d.input(f32(r, 128, 3072 if op == "gelu" else 33, scale=2.0))]))
        run_single_group(d, "eltwise", P(op, W), tol=1e-6)
    d = wl.GraphDesc("add_first_operand_is_residual")
    a = d.input(f32(r, 3, 50))
    y = d.op("relu", [d.op("add", [a, d.op("mul_scalar", [d.input(f32(r, 3, 50))], scalar=0.5)])])
    d.mark_output(y)
    run_single_group(d, "eltwise", P("relu", P("add", P("mul_scalar", W), W)), tol=1e-6)
    d = wl.GraphDesc("bias_last_axis")
    d.mark_output(d.op("gelu", [d.op("bias_add", [d.input(f32(r, 9, 50)), d.const(f32(r, 50))], axis=-1)]))
    run_single_group(d, "eltwise", P("gelu", P("bias_add", W, W)), tol=1e-6)


def test_take_and_embedding_sum():
    r = rng_for(12)
    tab = f32(r, 100, 24)
    ids = r.integers(0, 100, 17).astype(np.int32)
    d = wl.GraphDesc("take")
    d.mark_output(d.op("take", [d.const(tab), d.input(ids)]))
    run_single_group(d, "eltwise", P("take", W, W), tol=0.0)
    d = wl.GraphDesc("take_sum")
    e = d.op("take", [d.const(tab), d.input(ids)])
    e = d.op("add", [e, d.input(f32(r, 17, 24))])
    d.mark_output(d.op("add", [e, d.input(f32(r, 17, 24))]))
    run_single_group(d, "eltwise", P("add", P("add", P("take", W, W), W), W), tol=1e-6)


@pytest.mark.parametrize("case", [(1000, 128, 768, 3), (100, 17, 64, 3), (50, 5, 2048, 2), (300, 33, 700, 3)])
def test_embedding_layer_norm_in_one_kernel(case):
    """layer_norm(add(add(take, take), take)): the rows of three tables gathered, summed and normalised by one
    kernel (BERT's embedding: word + position + type), and the two-table form."""
    vocab, L, H, n_tab = case
    r = rng_for(18, vocab, L, H)
    d = wl.GraphDesc("embed_ln")
    ids = d.input(r.integers(0, vocab, L).astype(np.int32))
    e = d.op("take", [d.const(f32(r, vocab, H, scale=0.02)), ids])
    pat = P("take", W, W)
    e = d.op("add", [e, d.op("take", [d.const(f32(r, L + 3, H, scale=0.02)), d.const(np.arange(L, dtype=np.int32))])])
    pat = P("add", pat, P("take", W, W))
    if n_tab == 3:
        e = d.op("add", [e, d.op("take", [d.const(f32(r, 2, H, scale=0.02)), d.const(np.zeros(L, dtype=np.int32))])])
        pat = P("add", pat, P("take", W, W))
    g_, b_ = (1 + 0.02 * r.standard_normal(H)).astype(np.float32), f32(r, H, scale=0.02)
    d.mark_output(d.op("layer_norm", [e, d.const(g_), d.const(b_)], eps=1e-12))
    name, _ = run_single_group(d, "rowwise", P("layer_norm", pat, W, W), tol=2e-5)
    assert name == f"embed{n_tab}_layer_norm", name


def test_layout_copies():
    r = rng_for(13)
    x = f32(r, 16, 96)
    d = wl.GraphDesc("split_heads")
    d.mark_output(d.op("transpose", [d.op("reshape", [d.input(x)], dims=(16, 12, 8))], dims=(1, 0, 2)))
    run_single_group(d, "eltwise", P("transpose", P("reshape", W)), tol=0.0)
    d = wl.GraphDesc("merge_heads")
    d.mark_output(d.op("reshape", [d.op("transpose", [d.input(f32(r, 12, 16, 8))], dims=(1, 0, 2))], dims=(16, 96)))
    run_single_group(d, "eltwise", P("reshape", P("transpose", W)), tol=0.0)
    d = wl.GraphDesc("perm4")
    d.mark_output(d.op("transpose", [d.input(f32(r, 2, 3, 5, 7))], dims=(0, 3, 1, 2)))
    run_single_group(d, "eltwise", P("transpose", W), tol=0.0)
    d = wl.GraphDesc("reshape")
    d.mark_output(d.op("reshape", [d.input(f32(r, 6, 35))], dims=(2, 3, 5, 7)))
    run_single_group(d, "eltwise", P("reshape", W), tol=0.0)


def test_pools():
    r = rng_for(14)
    d = wl.GraphDesc("maxpool")
    d.mark_output(d.op("max_pool2d", [d.input(f32(r, 2, 5, 15, 13))], kernel=(3, 3), stride=(2, 2), pad=(1, 1)))
    run_single_group(d, "direct", P("max_pool2d", W), tol=0.0)
    d = wl.GraphDesc("gap")
    d.mark_output(d.op("global_avg_pool2d", [d.input(f32(r, 2, 37, 7, 7))]))
    run_single_group(d, "direct", P("global_avg_pool2d", W), tol=1e-6)


@pytest.mark.parametrize("k,s,p,shape", [(3, 1, 1, (2, 5, 15, 13)), (3, 2, 1, (1, 44, 28, 28)), (2, 2, 0, (3, 7, 8, 10)),
                                         (5, 1, 2, (1, 3, 9, 9))])
def test_avg_pool_and_pools_with_a_fused_add(k, s, p, shape):
    r = rng_for(15)
    d = wl.GraphDesc("avgpool")
    d.mark_output(d.op("avg_pool2d", [d.input(f32(r, *shape))], kernel=(k, k), stride=(s, s), pad=(p, p)))
    run_single_group(d, "direct", P("avg_pool2d", W), tol=1e-6)
    for kind in ("avg_pool2d", "max_pool2d"):
        d = wl.GraphDesc(kind + "_add")
        x = d.input(f32(r, *shape))
        y = d.op(kind, [x], kernel=(k, k), stride=(s, s), pad=(p, p))
        ho, wo = (shape[2] + 2 * p - k) // s + 1, (shape[3] + 2 * p - k) // s + 1
        other = d.input(f32(r, shape[0], shape[1], ho, wo))
        # the pool may be either operand of the add
        d.mark_output(d.op("add", [other, y] if kind == "max_pool2d" else [y, other]))
        run_single_group(d, "direct", P("add", P(kind, W), W), tol=1e-6)


@pytest.mark.parametrize("shapes,axis", [([(1, 44, 7, 7)] * 6, 1), ([(2, 3, 5, 4), (2, 1, 5, 4), (2, 6, 5, 4)], 1),
                                         ([(3, 5), (3, 2)], -1), ([(2, 4, 3), (5, 4, 3), (1, 4, 3), (1, 4, 3)], 0),
                                         ([(1, 8, 4, 4)] * 8, 1)])
def test_concat(shapes, axis):
    r = rng_for(16)
    d = wl.GraphDesc("concat")
    d.mark_output(d.op("concat", [d.input(f32(r, *s)) for s in shapes], axis=axis))
    run_single_group(d, "eltwise", P("concat", *([W] * len(shapes))), tol=0.0)


# ---------------------------------------------------------- whole graphs
def _session_and_oracle(desc, reg):
    s = clg.Session(desc, reg, device=0)
    g = Graph(desc)
    oms = enumerate_matches(g, reg)
    lms = s.match()
    assert [(m.pattern, m.first) for m in lms] == [(m.pattern, m.first) for m in oms]
    return s, g, oms


def test_tiny_cnn_every_placement_matches_the_oracle():
    desc = wl.tiny_cnn(0)
    reg = wl.default_registry()
    s, g, oms = _session_and_oracle(desc, reg)
    ref = g.run()
    placements = list(search.all_placements(g, oms))
    assert len(placements) == 2048
    worst = 0.0
    for pi in range(len(placements)):                   # every one of them
        plan = s.compile(placements[pi])
        got = plan.run()
        plan.destroy()
        worst = max(worst, max(norm_err(a, b) for a, b in zip(got, ref)))
    assert worst <= NET_TOL, worst
    s.close()


def _variants():
    return wl.default_registry(("igemm", "igemm_s", "igemm_m", "igemm_l", "igemm_r32", "igemm_r16"))


@pytest.mark.parametrize("name", ["tiny_cnn", "resnet50", "resnext50", "bert_base", "dcgan_b1", "dcgan_b64"])
def test_model_under_searched_placement(name):
    """Profile every candidate subgraph, search, compile, execute; compare the
    network outputs with the oracle and the placement with the oracle's DP on
    the same cost table."""
    desc = wl.MODEL_BUILDERS[name](0)
    reg = _variants()
    s, g, oms = _session_and_oracle(desc, reg)
    opts = B.ProfileOpts(warmup=3, batches=3, min_batch_us=50, max_launches=50)
    costs = s.profile(opts)
    assert np.all(costs > 0)
    got_search = s.search(costs, 0)
    assert got_search == search.dp(g, reg, oms, costs, 0)          # bit-exact placement
    plan = s.compile(got_search[1])
    got = plan.run()
    ref = g.run()
    errs = [norm_err(a, b) for a, b in zip(got, ref)]
    print(name, "kernels", plan.n_kernels, "errors", errs, "cost_ns", got_search[0])
    assert max(errs) <= NET_TOL, errs
    # the all-single-operator placement computes the same thing
    singles = [i for i, m in enumerate(oms) if len(m.nodes) == 1]
    first_single = {}
    for i in singles:
        first_single.setdefault(oms[i].nodes[0], i)
    plan1 = s.compile(sorted(first_single.values()))
    got1 = plan1.run()
    assert max(norm_err(a, b) for a, b in zip(got1, ref)) <= NET_TOL
    plan.destroy()
    plan1.destroy()
    s.close()


@pytest.mark.parametrize("name", ["tiny_cnn", "resnet50", "resnext50", "bert_base", "dcgan_b1", "dcgan_b64", "nasnet_a", "resnet3d_50"])
def test_model_in_the_benchmark_s_configuration(name):
    """Full size, the registry and measurer options bench.py uses (all kernel variants and the
    one-kernel separable convolution family)."""
    import bench
    desc = wl.MODEL_BUILDERS[name](0)
    reg = wl.default_registry(bench.VARIANTS, sepconv=True, attention=True)
    s, g, oms = _session_and_oracle(desc, reg)
    costs = s.profile(B.ProfileOpts(warmup=10, batches=5, min_batch_us=200, max_launches=500))
    got_search = s.search(costs, 0)
    assert got_search == search.dp(g, reg, oms, costs, 0)
    plan = s.compile(got_search[1])
    got = plan.run()
    ref = g.run()
    errs = [norm_err(a, b) for a, b in zip(got, ref)]
    print(name, "kernels", plan.n_kernels, "errors", errs)
    assert max(errs) <= NET_TOL, errs
    # Every kernel of this plan once more, alone: the same match cut out of the model (same shapes, same
    # weights, same backend, hence the same kernel instantiation) against the oracle at the per-operator bar.
    from parity_util import cut_out, run_group
    seen = set()
    for k in plan.kernels():
        if k["name"].endswith("_alias"):
            continue
        m = s.matches[k["match"]]
        key = B.clg_match_key(s.ctx, s.graph, k["match"])
        if key in seen:
            continue
        seen.add(key)
        backend, pattern = reg[m.pattern]
        sub = cut_out(desc, lambda v: B.clg_graph_node_shape(s.graph, v)[1], list(m.nodes[:m.n_nodes]), 9)
        tol = 2e-5 if k["name"].startswith(("softmax", "layer_norm")) else OP_TOL
        alone, _ = run_group(sub, backend, pattern, tol=tol, what=(name, k["name"]))
        assert alone == k["name"], (alone, k["name"])
    print(name, "distinct kernels checked alone:", len(seen))
    plan.destroy()
    s.close()


@pytest.mark.parametrize("name", ["tiny_cnn", "resnet50", "bert_base", "dcgan_b1"])
def test_model_under_a_rule_generated_registry(name):
    """The registry comes from pattern rules (the generator walks this graph) plus the
    few patterns no rule covers; matches and placement equal the oracle's over the
    same registry, the outputs equal the oracle's."""
    from workloads import patterns as wp
    desc = wl.MODEL_BUILDERS[name](0)
    explicit, rules = wp.rule_registry(("igemm_s8", "igemm_r16"))
    s = clg.Session(desc, explicit, device=0, rules=rules)
    assert s.generated > 0
    reg = s.full_registry()
    g = Graph(desc)
    oms = enumerate_matches(g, reg)
    lms = s.match()
    assert [(m.pattern, m.first) for m in lms] == [(m.pattern, m.first) for m in oms]
    costs = s.profile(B.ProfileOpts(warmup=3, batches=3, min_batch_us=50, max_launches=50))
    got_search = s.search(costs, 0)
    assert got_search == search.dp(g, reg, oms, costs, 0)
    plan = s.compile(got_search[1])
    got = plan.run()
    ref = g.run()
    errs = [norm_err(a, b) for a, b in zip(got, ref)]
    print(name, "generated patterns", s.generated, "kernels", plan.n_kernels, "errors", errs)
    assert max(errs) <= NET_TOL, errs
    plan.destroy()
    s.close()


@pytest.mark.parametrize("batch", [2, 5])
def test_resnext_at_larger_batch(batch):
    """The paper also varies the batch size (its Fig. 8, ResNeXt-50): the whole path at
    batch > 1 on a reduced ResNeXt (grouped 3x3, strided projection, residual adds)."""
    desc = wl.resnext50(0, image=64, width=32, blocks=(2, 1), groups=8, classes=20, batch=batch)
    reg = wl.default_registry(("igemm_s8", "igemm_r32", "igemm_r16"))
    s, g, oms = _session_and_oracle(desc, reg)
    costs = s.profile(B.ProfileOpts(warmup=3, batches=3, min_batch_us=50, max_launches=50))
    got_search = s.search(costs, 0)
    assert got_search == search.dp(g, reg, oms, costs, 0)
    plan = s.compile(got_search[1])
    got = plan.run()
    ref = g.run()
    assert got[0].shape == (batch, 20)
    assert max(norm_err(a, b) for a, b in zip(got, ref)) <= NET_TOL
    plan.destroy()
    s.close()


def test_nasnet_cells_whole_path():
    """NasNet-A (paper Sec. 5.1) at reduced size: separable convolutions (depthwise + 1x1), average and
    max pools, identities, adds and six-way concats in many parallel branches; channel counts that
    are no multiple of a tile (2, 4, 8 channels; 48-channel concats)."""
    desc = wl.nasnet_a(0, image=32, stem=8, filters=8, cells=1, classes=10)
    reg = wl.default_registry(("igemm_s8", "igemm_r16"), sepconv=True)
    s, g, oms = _session_and_oracle(desc, reg)
    costs = s.profile(B.ProfileOpts(warmup=2, batches=2, min_batch_us=30, max_launches=30))
    got_search = s.search(costs, 0)
    assert got_search == search.dp(g, reg, oms, costs, 0)
    plan = s.compile(got_search[1])
    got = plan.run()
    ref = g.run()
    assert max(norm_err(a, b) for a, b in zip(got, ref)) <= NET_TOL
    # a second placement: every operator alone, on whatever backend lists it first
    first = {}
    for i, m in enumerate(oms):
        if len(m.nodes) == 1 and costs[i] < B.COST_INF:
            first.setdefault(m.nodes[0], i)
    plan2 = s.compile(sorted(first.values()))
    assert plan2.n_kernels == len(g.op_ids)
    got2 = plan2.run()
    assert max(norm_err(a, b) for a, b in zip(got2, ref)) <= NET_TOL
    plan.destroy()
    plan2.destroy()
    s.close()


def test_profiler_is_repeatable_and_cached():
    desc = wl.resnet50(0, image=64, blocks=(1,))
    reg = wl.default_registry()
    s = clg.Session(desc, reg, device=0)
    ms = s.match()
    conv = [i for i, m in enumerate(ms) if m.n_nodes == 3 and reg[m.pattern][0] == "igemm"][0]
    nocache = B.ProfileOpts(no_cache=1)
    a = sorted(B.clg_profile_match(s.ctx, s.graph, conv, nocache) for _ in range(7))
    # The paper reports < 3 % spread for its measurements (Sec. 5.2).  Here about one measurement in thirty is
    # inflated as a whole (clocks), so: five of seven within 8 % of the smallest (typically 1 - 2 %).
    assert a[4] <= 1.08 * a[0], a
    assert B.clg_cost_log_size(s.ctx) == 0
    c1 = B.clg_profile_match(s.ctx, s.graph, conv)
    assert B.clg_cost_log_size(s.ctx) == 1
    assert B.clg_profile_match(s.ctx, s.graph, conv) == c1            # served from the log
    assert c1 <= 1.5 * a[0] and a[0] <= 1.5 * c1, (c1, a)
    assert B.clg_profile_empty(s.ctx) > 0
    s.close()


def test_execute_argument_errors():
    desc = wl.tiny_cnn(0)
    reg = wl.default_registry()
    s = clg.Session(desc, reg, device=0)
    ms = s.match()
    _, ids = s.search(wl.synthetic_costs(len(ms), 0), 0)
    plan = s.compile(ids).bind()
    ins, outs, ws, nbytes, stream = plan._args()
    with pytest.raises(clg.ClgError) as e:
        B.clg_execute(plan.h, ins, outs, ws, plan.ws_bytes - 1, stream)
    assert e.value.status == "WORKSPACE_TOO_SMALL"
    with pytest.raises(clg.ClgError) as e:
        B.clg_execute(plan.h, ins, outs, ws + 4, nbytes, stream)
    assert e.value.status == "INVALID_ARG"
    with pytest.raises(clg.ClgError) as e:
        B.clg_execute(plan.h, [0], outs, ws, nbytes, stream)
    assert e.value.status == "INVALID_ARG"
    ns = plan.execute_timed()
    assert len(ns) == plan.n_kernels and np.all(ns > 0)
    plan.destroy()
    s.close()


# ------------------------------------------------------------------- graph-level search
def _rand_u32(seed, n=200000):
    return np.random.default_rng(seed).integers(0, 2 ** 32, n, dtype=np.uint64).tolist()


# ------------------------------------------------------------------- regions
def _per_operator_plan(desc, backend="igemm_r16"):
    """Every operator group on `backend` where it runs it (cost table: the register-fed kernels are cheap)."""
    reg = wl.default_registry(("igemm_s8", backend), attention=True)
    s = clg.Session(desc, reg, device=0)
    ms = s.match()
    costs = []
    for i, m in enumerate(ms):
        try:
            clg.clg_match_key(s.ctx, s.graph, i)
            costs.append((10 if reg[m.pattern][0] == backend else 1000) * m.n_nodes)
        except clg.ClgError:
            costs.append(B.COST_INF)
    _, ids = s.search(costs, 0)
    return s, s.compile(ids).bind()


def _dense_branch(d, r, x, k, n, tail, heads=0):
    y = d.op("dense", [x, d.const(f32(r, n, k, scale=k ** -0.5))])
    y = d.op("bias_add", [y, d.const(f32(r, n))], axis=-1)
    for op in tail:
        if op == "add":                                    # a residual operand of its own
            y = d.op("add", [y, d.input(f32(r, d.nodes[x]["shape"][0], n))])
        else:
            y = d.op(op, [y])
    if heads:
        m = d.nodes[x]["shape"][0]
        y = d.op("transpose", [d.op("reshape", [y], dims=(m, heads, n // heads))], dims=(1, 0, 2))
    return y


REGION_DENSE_CASES = {
    "qkv": [(0, 768, 768, (), 12)] * 3,                                     # BERT's projections: one input, equal shapes
    "mixed": [(0, 768, 768, (), 12), (0, 768, 3072, ("gelu",), 0), (1, 256, 48, ("relu",), 0), (0, 768, 100, (), 0)],
    "two_inputs": [(0, 768, 64, ("relu",), 0), (1, 256, 768, (), 0)],
    "with_residual": [(0, 768, 768, ("add",), 0), (1, 256, 96, ("add",), 0), (0, 768, 256, (), 0)],
}


@pytest.mark.parametrize("backend", RF + ("igemm_r16_w4", "igemm_r16x2_w4"))
@pytest.mark.parametrize("case", sorted(REGION_DENSE_CASES))
def test_region_of_sibling_dense_layers(case, backend):
    """Independent dense layers as one launch (graph-level backend, Sec. 4.3): every subset of the region
    handed over gives the oracle's values at the per-operator bar."""
    from parity_util import check_outputs
    r = rng_for(71, len(case))
    d = wl.GraphDesc("region_dense_" + case)
    xs = [d.input(f32(r, 128, 768)), d.input(f32(r, 70, 256))]
    for which, k, n, tail, heads in REGION_DENSE_CASES[case]:
        d.mark_output(_dense_branch(d, r, xs[which], k, n, tail, heads))
    s, plan = _per_operator_plan(d, backend)
    n = plan.n_kernels
    rg = plan.regions()
    assert n == len(REGION_DENSE_CASES[case]) and rg == [0] * n, (rg, [k["name"] for k in plan.kernels()])
    ref = Graph(d).run()
    for digits in ([1] * n, [1, 1] + [0] * (n - 2), [0] * (n - 2) + [1, 1], [1] + [0] * (n - 1)):
        plan.set_handover(digits, lanes=1)
        assert plan.n_launches == n - max(sum(digits) - 1, 0)
        got = plan.run()
        check_outputs(got, ref, OP_TOL, (case, backend, digits))
        assert all(np.array_equal(a, b) for a, b in zip(got, plan.run()))          # deterministic
    ns = plan.execute_timed()
    assert (ns > 0).sum() == plan.n_launches
    s.close()


REGION_CONV_CASES = [
    # cin, h, [(cout, stride, tail)...]: members read the same input
    (256, 56, [(512, 2, ("bias_add",)), (128, 1, ("bias_add", "relu"))]),          # ResNet-50 stage 2: projection + c1
    (1024, 14, [(2048, 2, ("bias_add",)), (512, 1, ("bias_add", "relu"))]),        # stage 4
    (64, 56, [(256, 1, ("bias_add",)), (64, 1, ("bias_add", "relu"))]),            # stage 1: equal strides
    (40, 9, [(24, 1, ()), (70, 2, ("bias_add", "relu")), (16, 1, ("bias_add",)), (33, 3, ("bias_add", "relu"))]),   # ragged, four members
]


@pytest.mark.parametrize("backend", RF)
@pytest.mark.parametrize("ci", range(len(REGION_CONV_CASES)))
def test_region_of_sibling_1x1_convolutions(ci, backend):
    from parity_util import check_outputs
    cin, h, branches = REGION_CONV_CASES[ci]
    r = rng_for(72, ci)
    d = wl.GraphDesc("region_conv")
    x = d.input(f32(r, 1, cin, h, h))
    for cout, stride, tail in branches:
        y = d.op("conv2d", [x, d.const(f32(r, cout, cin, 1, 1, scale=(2.0 / cin) ** 0.5))], stride=(stride, stride), pad=(0, 0), groups=1)
        for op in tail:
            y = d.op("bias_add", [y, d.const(f32(r, cout))], axis=1) if op == "bias_add" else d.op(op, [y])
        d.mark_output(y)
    s, plan = _per_operator_plan(d, backend)
    n = plan.n_kernels
    assert n == len(branches) and plan.regions() == [0] * n, (plan.regions(), [k["name"] for k in plan.kernels()])
    ref = Graph(d).run()
    for digits in ([1] * n, [0] * n, [1, 1] + [0] * (n - 2)):
        plan.set_handover(digits, lanes=1)
        assert plan.n_launches == n - max(sum(digits) - 1, 0)
        check_outputs(plan.run(), ref, OP_TOL, (ci, backend, digits))
    s.close()


PLANE_REGION_CASES = [
    # batch, channels, height, width, branches: (kind, filter, stride, relu in front, tail)
    (1, 44, 28, 28, [("dw", 3, 1, True, ("bias_add",)), ("dw", 5, 1, True, ("bias_add",)), ("avg", 3, 1, False, ()), ("max", 3, 1, False, ("add",)),
                     ("dw", 7, 1, False, ("bias_add", "add")), ("avg", 3, 1, False, ("add",))]),          # a cell's first stage: two regions
    (2, 22, 15, 13, [("dw", 5, 2, True, ()), ("max", 3, 2, False, ()), ("dw", 3, 2, False, ("bias_add",))]),   # strided, ragged, batch 2
    (1, 7, 9, 9, [("avg", 2, 1, False, ()), ("dw", 3, 1, True, ("bias_add", "add"))]),
]


@pytest.mark.parametrize("ci", range(len(PLANE_REGION_CASES)))
def test_region_of_sibling_depthwise_convolutions_and_pools(ci):
    """The thread-per-output kernels of a cell's branches (depthwise convolutions with and without a relu in front,
    window pools with and without a fused add) that read the same tensor run as one launch per region; the outputs are
    those of the kernels run one by one, bit for bit."""
    from parity_util import check_outputs
    n_img, c, h, w, branches = PLANE_REGION_CASES[ci]
    r = rng_for(73, ci)
    d = wl.GraphDesc("region_plane")
    x = d.input(f32(r, n_img, c, h, w))
    for kind, k, stride, pre, tail in branches:
        ho, wo = (h + 2 * (k // 2) - k) // stride + 1, (w + 2 * (k // 2) - k) // stride + 1
        if kind == "dw":
            y = d.op("relu", [x]) if pre else x
            y = d.op("conv2d", [y, d.const(f32(r, c, 1, k, k, scale=1.0 / k))], stride=(stride, stride), pad=(k // 2, k // 2), groups=c)
        else:
            y = d.op("avg_pool2d" if kind == "avg" else "max_pool2d", [x], kernel=(k, k), stride=(stride, stride), pad=(k // 2, k // 2))
        for op in tail:
            y = d.op("bias_add", [y, d.const(f32(r, c))], axis=1) if op == "bias_add" else d.op("add", [y, d.input(f32(r, n_img, c, ho, wo))])
        d.mark_output(y)
    tails = [(), ("bias_add",), ("bias_add", "add")]
    reg = [("sepconv", tail_pattern(P("conv2d", P("relu", W), W), t)) for t in tails]
    reg += [("direct", tail_pattern(P("conv2d", W, W), t)) for t in tails]
    reg += [("direct", P(k, W)) for k in ("avg_pool2d", "max_pool2d")] + [("direct", P("add", P(k, W), W)) for k in ("avg_pool2d", "max_pool2d")]
    reg += [("eltwise", P("relu", W)), ("eltwise", P("add", W, W)), ("eltwise", P("bias_add", W, W))]
    s = clg.Session(d, reg, device=0)
    ms = s.match()
    _, ids = s.search([100] * len(ms), 0)                   # fewest kernels: every branch is one kernel
    plan = s.compile(ids).bind()
    n = plan.n_kernels
    assert n == len(branches), [k["name"] for k in plan.kernels()]
    regions = plan.regions()
    assert all(g >= 0 for g in regions[:4 * (n // 4) + (n % 4 if n % 4 > 1 else 0)]), regions
    n_regions = max(regions) + 1
    ref = Graph(d).run()
    plan.set_handover([0] * n, lanes=1)
    one_by_one = plan.run()
    check_outputs(one_by_one, ref, OP_TOL, (ci, "one by one"))
    for digits in ([1] * n, [i % 2 for i in range(n)], [1, 1] + [0] * (n - 2), [1] * n):
        plan.set_handover(digits, lanes=1)
        fused_members = sum(max(sum(dg for dg, g in zip(digits, regions) if g == q) - 1, 0) for q in range(n_regions))
        assert plan.n_launches == n - fused_members, (digits, regions, plan.n_launches)
        got = plan.run()
        assert all(np.array_equal(a, b) for a, b in zip(got, one_by_one)), (ci, digits)
    s.close()


SEP_REGION_CASES = [
    # batch, channels, height, width, branches: (filter, stride, relu in front, output channels, tail)
    (1, 44, 28, 28, [(3, 1, True, 44, ("bias_add",)), (3, 1, True, 44, ("bias_add", "add")), (3, 1, False, 44, ("bias_add",)), (5, 1, True, 44, ("bias_add",)),
                     (5, 1, True, 44, ("bias_add", "relu"))]),       # three 3x3 share a launch, two 5x5 another
    (2, 20, 9, 9, [(3, 2, True, 50, ()), (3, 2, True, 20, ("bias_add",))]),              # strided, ragged, batch 2, unequal output channels
    (1, 176, 7, 7, [(7, 1, True, 176, ("bias_add",)), (7, 1, False, 176, ("bias_add", "add")), (3, 1, True, 176, ())]),
]


@pytest.mark.parametrize("ci", range(len(SEP_REGION_CASES)))
def test_region_of_sibling_separable_convolutions(ci):
    """One-kernel separable convolutions of a cell's branches that read the same tensor and share the kernel shape
    (filter size, waves per workgroup) run as one launch; outputs are those of the kernels run one by one, bit for bit."""
    from parity_util import check_outputs
    n_img, c, h, w, branches = SEP_REGION_CASES[ci]
    r = rng_for(74, ci)
    d = wl.GraphDesc("region_sep")
    x = d.input(f32(r, n_img, c, h, w))
    for k, stride, pre, cout, tail in branches:
        ho, wo = (h + 2 * (k // 2) - k) // stride + 1, (w + 2 * (k // 2) - k) // stride + 1
        y = d.op("relu", [x]) if pre else x
        y = d.op("conv2d", [y, d.const(f32(r, c, 1, k, k, scale=1.0 / k))], stride=(stride, stride), pad=(k // 2, k // 2), groups=c)
        y = d.op("conv2d", [y, d.const(f32(r, cout, c, 1, 1, scale=c ** -0.5))], stride=(1, 1), pad=(0, 0), groups=1)
        for op in tail:
            if op == "bias_add":
                y = d.op("bias_add", [y, d.const(f32(r, cout))], axis=1)
            elif op == "add":
                y = d.op("add", [y, d.input(f32(r, n_img, cout, ho, wo))])
            else:
                y = d.op(op, [y])
        d.mark_output(y)
    tails = [(), ("bias_add",), ("bias_add", "add"), ("bias_add", "relu")]
    reg = [("sepconv", tail_pattern(P("conv2d", P("conv2d", P("relu", W), W), W), t)) for t in tails]
    reg += [("sepconv", tail_pattern(P("conv2d", P("conv2d", W, W), W), t)) for t in tails]
    reg += wl.default_registry(("igemm_s8",))
    s = clg.Session(d, reg, device=0)
    ms = s.match()
    _, ids = s.search([100 if reg[m.pattern][0] == "sepconv" else 1000 * m.n_nodes for m in ms], 0)
    plan = s.compile(ids).bind()
    n = plan.n_kernels
    names = [k["name"] for k in plan.kernels()]
    assert n == len(branches) and all("sepconv" in nm for nm in names), names
    regions = plan.regions()
    n_regions = max(regions) + 1
    assert n_regions >= 1, (regions, names)
    ref = Graph(d).run()
    plan.set_handover([0] * n, lanes=1)
    one_by_one = plan.run()
    check_outputs(one_by_one, ref, OP_TOL, (ci, "one by one"))
    for digits in ([1] * n, [i % 2 for i in range(n)], [1, 1] + [0] * (n - 2), [1] * n):
        plan.set_handover(digits, lanes=1)
        fused_members = sum(max(sum(dg for dg, g in zip(digits, regions) if g == q) - 1, 0) for q in range(n_regions))
        assert plan.n_launches == n - fused_members, (digits, regions, plan.n_launches)
        got = plan.run()
        assert all(np.array_equal(a, b) for a, b in zip(got, one_by_one)), (ci, digits)
    s.close()


def _random_sibling_graph(seed):
    """A random DAG over [1, C, 12, 12] tensors in which 1x1 convolutions (with bias / relu / residual tails, some
    strided), 3x3 convolutions, adds and relus read any earlier value of a fitting shape: many kernels that do not
    depend on each other, in an order that makes the region finder move members past unrelated kernels."""
    r = rng_for(91, seed)
    d = wl.GraphDesc(f"siblings_{seed}")
    vals = {}                                  # (channels, size) -> values of that shape

    def put(v, c, h):
        vals.setdefault((c, h), []).append(v)
        return v
    x = put(d.input(f32(r, 1, 8, 12, 12)), 8, 12)
    used = set()
    for step in range(int(r.integers(8, 15))):
        (c, h), pool = list(vals.items())[int(r.integers(0, len(vals)))]
        src = pool[int(r.integers(0, len(pool)))]
        kind = r.random()
        if kind < 0.6:                         # 1x1 convolution, the fusable kind
            cout = int(r.choice([8, 16, 24, 40]))
            stride = 2 if (r.random() < 0.3 and h % 2 == 0) else 1
            y = d.op("conv2d", [src, d.const(f32(r, cout, c, 1, 1, scale=(2.0 / c) ** 0.5))], stride=(stride, stride), pad=(0, 0), groups=1)
            ho = (h - 1) // stride + 1
            if r.random() < 0.7:
                y = d.op("bias_add", [y, d.const(f32(r, cout))], axis=1)
                if r.random() < 0.4 and (cout, ho) in vals:
                    other = vals[(cout, ho)][int(r.integers(0, len(vals[(cout, ho)])))]
                    y = d.op("add", [y, other])
                    used.add(other)
                if r.random() < 0.6:
                    y = d.op("relu", [y])
            put(y, cout, ho)
        elif kind < 0.75:
            y = d.op("conv2d", [src, d.const(f32(r, c, c, 3, 3, scale=(2.0 / (9 * c)) ** 0.5))], stride=(1, 1), pad=(1, 1), groups=1)
            put(d.op("relu", [d.op("bias_add", [y, d.const(f32(r, c))], axis=1)]), c, h)
        elif kind < 0.9 and len(pool) > 1:
            other = pool[int(r.integers(0, len(pool)))]
            put(d.op("add", [src, other]), c, h)
            used.add(other)
        else:
            put(d.op("relu", [src]), c, h)
        used.add(src)
    for pool in vals.values():
        for v in pool:
            if v not in used and d.nodes[v]["kind"] != "input":
                d.mark_output(v)
    if not d.outputs:
        d.mark_output(list(vals.values())[-1][-1])
    return d


@pytest.mark.parametrize("seed", range(12))
def test_regions_on_random_graphs_of_sibling_kernels(seed):
    """Whatever the topology: with every kernel handed over (regions fused, members moved next to each other, one
    workspace for all digit strings), with none, and with every other one, the outputs equal the oracle's."""
    from parity_util import check_outputs
    d = _random_sibling_graph(seed)
    s, plan = _per_operator_plan(d, "igemm_r16" if seed % 2 else "igemm_r32")
    ref = Graph(d).run()
    n = plan.n_kernels
    n_regions = max(plan.regions() + [-1]) + 1
    for digits in ([1] * n, [0] * n, [i % 2 for i in range(n)], [1] * n):
        plan.set_handover(digits, lanes=1)
        check_outputs(plan.run(), ref, OP_TOL * 4, (seed, digits))      # a few fused operators deep
    print("seed", seed, "kernels", n, "regions", n_regions, "launches all-ones", plan.n_launches)
    s.close()


@pytest.mark.parametrize("name", ["resnet50", "bert_base", "resnext50", "resnet3d_50", "nasnet_a"])
def test_model_with_every_region_fused(name):
    """Full size, the benchmark's registry: the searched op-level plan, then every kernel handed over so that
    each region runs as one launch; outputs against the oracle."""
    import bench
    desc = wl.MODEL_BUILDERS[name](0)
    reg = wl.default_registry(bench.VARIANTS, sepconv=True, attention=True)
    s = clg.Session(desc, reg, device=0)
    s.match()
    costs = s.profile(B.ProfileOpts(warmup=5, batches=3, min_batch_us=100, max_launches=200))
    _, ids = s.search(costs, 0)
    plan = s.compile(ids).bind()
    before = plan.n_launches
    plan.set_handover([1] * plan.n_kernels, lanes=1)
    after = plan.n_launches
    n_regions = max(plan.regions()) + 1
    print(name, "launches", before, "->", after, "regions", n_regions)
    # which kernels are siblings of one kind depends on the measured placement
    assert n_regions >= (6 if name == "bert_base" else 0) and after <= before - n_regions
    ref = Graph(desc).run()
    for _ in range(2):
        got = plan.run()
        assert max(norm_err(a, b) for a, b in zip(got, ref)) <= NET_TOL
    plan.set_handover([0] * plan.n_kernels, lanes=1)
    assert plan.n_launches == before
    assert max(norm_err(a, b) for a, b in zip(plan.run(), ref)) <= NET_TOL
    s.close()


SMALL_CELL_NETS = [dict(image=24, stem=4, filters=4, cells=1, classes=5), dict(image=40, stem=8, filters=11, cells=2, classes=7),
                   dict(image=33, stem=6, filters=20, cells=1, classes=3, batch=2), dict(image=56, stem=16, filters=44, cells=1, classes=10)]


@pytest.mark.parametrize("prefer", ["one_kernel", "split"])
@pytest.mark.parametrize("ci", range(len(SMALL_CELL_NETS)))
def test_regions_of_every_kind_on_small_cell_networks(ci, prefer):
    """Small NasNet-A-like networks (odd sizes, batch 2) under two placements - separable convolutions as one kernel
    each, or split into depthwise + 1x1 kernels - with all regions fused, none, and every other kernel handed over:
    each string's outputs against the oracle, and all-zero against all-one strings to the rounding of the register-fed
    members' common tile shape."""
    desc = wl.nasnet_a(ci, **SMALL_CELL_NETS[ci])
    reg = wl.default_registry(("igemm_s8", "igemm_r16"), sepconv=True)
    s = clg.Session(desc, reg, device=0)
    ms = s.match()
    costs = []
    for i, m in enumerate(ms):
        try:
            clg.clg_match_key(s.ctx, s.graph, i)
        except clg.ClgError:
            costs.append(B.COST_INF)
            continue
        be = reg[m.pattern][0]
        base = {"sepconv": 30 if prefer == "one_kernel" else 3000, "igemm_r16": 40, "direct": 50}.get(be, 100)
        costs.append(base * m.n_nodes if be != "sepconv" else base)
    _, ids = s.search(costs, 0)
    plan = s.compile(ids).bind()
    n = plan.n_kernels
    regions = plan.regions()
    names = [k["name"] for k in plan.kernels()]
    kinds = {("sep" if "sepconv" in names[i] else "plane" if names[i].split("_epi")[0] in
              ("avg_pool", "max_pool", "direct_conv", "relu_dwconv3", "relu_dwconv5", "relu_dwconv7") else "mfma")
             for i in range(n) if regions[i] >= 0}
    assert "mfma" in kinds and ("sep" if prefer == "one_kernel" else "plane") in kinds, (kinds, sorted(set(names)))
    ref = Graph(desc).run()
    for digits in ([1] * n, [0] * n, [i % 2 for i in range(n)], [(i // 3) % 2 for i in range(n)], [1] * n):
        plan.set_handover(digits, lanes=1)
        got = plan.run()
        assert max(norm_err(a, b) for a, b in zip(got, ref)) <= NET_TOL, (ci, prefer, digits[:8])
    s.close()


@pytest.mark.parametrize("name", ["resnet50", "bert_base"])
def test_a_plan_never_reads_the_weights_it_has_packed(name):
    """What clg_plan_reads_constant reports as not read can be overwritten after clg_compile: the plan's outputs do
    not change (the model's hot set is the packed copies, not both)."""
    import torch
    desc = wl.resnet50(0, image=64, width=16, blocks=(2, 1), classes=10) if name == "resnet50" else \
        wl.bert_base(0, layers=2, seq=32, hidden=128, heads=2, ffn=256, vocab=60, max_pos=32)
    s, plan = _per_operator_plan(desc, "igemm_r16")
    before = plan.run()
    gone = plan.constants_not_read()
    assert len(gone) >= 4
    for nid in gone:
        s.const_tensors[nid].fill_(float("nan"))
    torch.cuda.synchronize()
    plan.set_handover([1] * plan.n_kernels, lanes=1)        # the region kernels read packed copies too
    fused = plan.run()
    plan.set_handover([0] * plan.n_kernels, lanes=1)
    after = plan.run()
    assert all(np.array_equal(a, b) for a, b in zip(before, after))
    assert max(norm_err(a, b) for a, b in zip(fused, before)) <= 1e-5
    s.close()


@pytest.mark.parametrize("lanes", [1, 3])
@pytest.mark.parametrize("name", ["resnet_small", "tiny_cnn"])
def test_graph_level_search_keeps_outputs_and_never_loses_to_the_seed(name, lanes):
    """Sec. 4.3: digit strings over the kernels of the op-level plan, priced by timing the whole
    sequence.  Whatever string wins, the plan must compute the same values as the op-level plan
    (bit for bit: the same kernels, another schedule), equal the oracle, and its measured time is
    by construction at most the all-zero seed's."""
    if name == "tiny_cnn":
        desc = wl.tiny_cnn(0)
    else:
        desc = wl.resnet50(0, image=64, width=16, blocks=(2, 2), classes=10)
    reg = wl.default_registry(("igemm_s8", "igemm_r16"))
    s, g, oms = _session_and_oracle(desc, reg)
    costs = s.profile(B.ProfileOpts(warmup=3, batches=2, min_batch_us=50, max_launches=50))
    _, ids = s.search(costs, 0)
    plan = s.compile(ids).bind()
    base = plan.run()
    opts = B.make_es_opts(population=6, generations=4, tournament=3, p_init=0.3, p_mutate=0.6, p_flip=0.15, p_cross=0.6)
    best, best_ns, seed_ns, evals, hist = plan.search_graph_level(opts, _rand_u32(5), lanes=lanes, warmup=2, batches=2, reps=10)
    assert len(best) == plan.n_kernels and set(best) <= {0, 1}
    assert 0 < best_ns <= seed_ns and hist[0] <= seed_ns and hist[-1] == best_ns
    assert all(a >= b for a, b in zip(hist, hist[1:])) and 1 <= evals <= 6 * 5 * 2
    def same(a_list, b_list):
        # the lane scheduler runs the same kernels (bit for bit); a region runs its members in one common
        # tile shape, which adds in another order (to rounding)
        if lanes > 1:
            return all(np.array_equal(a, b) for a, b in zip(a_list, b_list))
        return max(norm_err(a, b) for a, b in zip(a_list, b_list)) <= 1e-5
    got = plan.run()                            # the plan is left set to the best string
    assert same(got, base)
    ref = g.run()
    assert max(norm_err(a, b) for a, b in zip(got, ref)) <= NET_TOL
    # every string gives the same values: all ones, alternating, and back to the seed
    n = plan.n_kernels
    for digits in ([1] * n, [i % 2 for i in range(n)], [0] * n):
        plan.set_handover(digits, lanes=1 if lanes == 1 else 2)
        out = plan.run()
        assert same(out, base) and max(norm_err(a, b) for a, b in zip(out, ref)) <= NET_TOL
    assert all(np.array_equal(a, b) for a, b in zip(plan.run(), base))      # all zeros: the op-level plan again, bit for bit
    assert plan.n_lanes == 1                    # all zeros is the op-level plan on the caller's stream
    assert plan.measure(warmup=2, batches=2, reps=5) > 0
    plan.destroy()
    s.close()


def test_graph_level_search_equals_the_oracle_s_on_the_same_costs():
    """The library's search drives set_handover + measure; with the measured costs recorded per
    string, the oracle's search replayed on that table must walk the same strings and end at the
    same one (the search itself is deterministic given the draws)."""
    desc = wl.tiny_cnn(0)
    reg = wl.default_registry(("igemm_s8",))
    s, g, oms = _session_and_oracle(desc, reg)
    costs = s.profile(B.ProfileOpts(warmup=3, batches=2, min_batch_us=50, max_launches=50))
    _, ids = s.search(costs, 0)
    plan = s.compile(ids).bind()
    table = {}

    def measured(d):
        plan.set_handover(d, lanes=2)
        table[tuple(d)] = float(plan.measure(warmup=1, batches=1, reps=5))
        return table[tuple(d)]
    kw = dict(population=4, generations=3, tournament=2, p_init=0.5, p_mutate=0.5, p_flip=0.2, p_cross=0.5)
    rand = _rand_u32(7, 5000)
    got = B.clg_evolve(plan.n_kernels, B.make_es_opts(**kw), rand, measured)
    from oracle import evolve as oe
    want = oe.evolve(plan.n_kernels, lambda d: table[tuple(d)], rand, **kw)
    assert got[0] == want[0] and got[1] == want[1] and got[2] == want[2] == len(table) and got[3] == want[3]
    plan.destroy()
    s.close()


# ------------------------------------------------------------------- lanes
@pytest.mark.parametrize("name", ["resnet50", "bert_base", "tiny_cnn"])
def test_lanes_give_the_same_result_as_one_stream(name):
    """Independent branches of a placement run on several HIP streams; the outputs
    must equal, bit for bit, those of the same plan on the caller's stream alone,
    on repeated executions and after switching back and forth."""
    desc = wl.MODEL_BUILDERS[name](0)
    reg = wl.default_registry(("igemm_s8", "igemm_r16"))
    s = clg.Session(desc, reg, device=0)
    s.match()
    costs = s.profile(B.ProfileOpts(warmup=5, batches=2, min_batch_us=50, max_launches=100))
    _, ids = s.search(costs, 0)
    plan = s.compile(ids).bind()
    assert plan.n_lanes == 1                    # the default
    plan.set_lanes(3)
    if name != "tiny_cnn":
        assert plan.n_lanes > 1, "the model has parallel branches"
    multi = [plan.run() for _ in range(3)]
    plan.set_lanes(1)
    assert plan.n_lanes == 1
    single = plan.run()
    plan.set_lanes(3)
    again = plan.run()
    for outs in multi + [again]:
        assert all(np.array_equal(a, b) for a, b in zip(outs, single))
    ref = Graph(desc).run()
    assert max(norm_err(a, b) for a, b in zip(single, ref)) <= NET_TOL
    plan.destroy()
    s.close()


def test_lanes_with_concats_planned_as_aliases():
    """The lane scheduler on a plan whose concats launch nothing (reduced NasNet-A: many parallel branches
    writing pieces of one buffer): same bits as on one stream."""
    desc = wl.nasnet_a(0, image=32, stem=8, filters=8, cells=1, classes=10)
    reg = wl.default_registry(("igemm_r16",), sepconv=True)
    s = clg.Session(desc, reg, device=0)
    s.match()
    costs = s.profile(B.ProfileOpts(warmup=2, batches=2, min_batch_us=30, max_launches=30))
    _, ids = s.search(costs, 0)
    plan = s.compile(ids).bind()
    assert any(k["name"].endswith("_alias") for k in plan.kernels())
    single = plan.run()
    plan.set_lanes(4)
    assert plan.n_lanes > 1
    multi = [plan.run() for _ in range(3)]
    plan.set_handover([i % 2 for i in range(plan.n_kernels)], lanes=3)
    mixed = plan.run()
    for outs in multi + [mixed]:
        assert all(np.array_equal(a, b) for a, b in zip(outs, single))
    assert max(norm_err(a, b) for a, b in zip(single, Graph(desc).run())) <= NET_TOL
    plan.destroy()
    s.close()


# ---------------------------------------------------------- concatenation planned as an alias
def _concat_graph(case):
    """Small graphs around one concat; returns (desc, expected kernel-name suffix of the concat)."""
    r = rng_for(61)
    d = wl.GraphDesc("concat_alias_" + case)
    x = d.input(f32(r, 1, 8, 6, 6))

    def branch(cout, src=None, k=1):
        w = d.const(f32(r, cout, 8, k, k) * 0.3)
        b = d.const(f32(r, cout))
        y = d.op("conv2d", [x if src is None else src, w], stride=(1, 1), pad=(k // 2, k // 2), groups=1)
        return d.op("relu", [d.op("bias_add", [y, b])])

    if case == "three_branches":                 # every operand produced by a kernel: no copy
        c = d.op("concat", [branch(4), branch(8, k=3), branch(12)], axis=1)
        d.mark_output(d.op("relu", [c]))
        return d, "_alias"
    if case == "result_is_an_output":            # the pieces go straight into the caller's buffer
        a = branch(4)
        c = d.op("concat", [a, branch(8), d.op("tanh", [a])], axis=1)
        d.mark_output(c)
        return d, "_alias"
    if case == "nested":                         # a concat inside a concat, and a piece read again later
        a, b = branch(4), branch(8)
        inner = d.op("concat", [a, b], axis=1)
        outer = d.op("concat", [branch(4), inner, d.op("relu", [inner])], axis=1)
        d.mark_output(d.op("add", [d.op("relu", [outer]), d.op("concat", [b, b, d.op("tanh", [b]), a], axis=1)]))
        return d, "nested"
    if case == "graph_input_operand":            # the caller's memory cannot move: a real copy
        c = d.op("concat", [branch(4), x], axis=1)
        d.mark_output(d.op("relu", [c]))
        return d, ""
    if case == "same_operand_twice":
        a = branch(4)
        c = d.op("concat", [a, a], axis=1)
        d.mark_output(d.op("relu", [c]))
        return d, ""
    if case == "operand_is_an_output":
        a = branch(4)
        d.mark_output(a)
        d.mark_output(d.op("relu", [d.op("concat", [a, branch(4)], axis=1)]))
        return d, ""
    if case == "operand_in_two_concats":         # the first concat gets it, the second copies
        a, b = branch(4), branch(8)
        c1 = d.op("concat", [a, b], axis=1)
        c2 = d.op("concat", [b, a], axis=1)
        d.mark_output(d.op("add", [d.op("relu", [c1]), d.op("relu", [c2])]))
        return d, "mixed"
    if case == "pieces_not_contiguous":          # batch 2: channel slices of different images interleave
        d = wl.GraphDesc("concat_alias_" + case)
        x2 = d.input(f32(r, 2, 8, 6, 6))
        ys = []
        for cout in (4, 8):
            w = d.const(f32(r, cout, 8, 1, 1) * 0.3)
            ys.append(d.op("relu", [d.op("conv2d", [x2, w], stride=(1, 1), pad=(0, 0), groups=1)]))
        d.mark_output(d.op("relu", [d.op("concat", ys, axis=1)]))
        return d, ""
    if case == "misaligned_piece":               # 3 x 3 x 3 floats: the second piece would start at byte 108
        d = wl.GraphDesc("concat_alias_" + case)
        x3 = d.input(f32(r, 1, 8, 3, 3))
        ys = []
        for cout in (3, 5):
            w = d.const(f32(r, cout, 8, 1, 1) * 0.3)
            ys.append(d.op("relu", [d.op("conv2d", [x3, w], stride=(1, 1), pad=(0, 0), groups=1)]))
        d.mark_output(d.op("relu", [d.op("concat", ys, axis=1)]))
        return d, ""
    raise KeyError(case)


CONCAT_ALIAS_CASES = ["three_branches", "result_is_an_output", "nested", "graph_input_operand", "same_operand_twice",
                      "operand_is_an_output", "operand_in_two_concats", "pieces_not_contiguous", "misaligned_piece"]


@pytest.mark.parametrize("case", CONCAT_ALIAS_CASES)
def test_concat_planned_as_an_alias(case):
    """A concat whose operands can be produced in place launches nothing; one that cannot still copies.  Either
    way the graph's outputs equal the oracle's, on two executions in a row."""
    desc, suffix = _concat_graph(case)
    reg = wl.default_registry(("igemm", "igemm_r16"))
    s = clg.Session(desc, reg, device=0)
    ms = s.match()
    costs = [1000 * m.n_nodes for m in ms]              # any cost table: operator by operator is the cheapest cover
    _, ids = s.search(costs, 0)
    plan = s.compile(ids)
    names = [k["name"] for k in plan.kernels() if k["name"].startswith("concat")]
    if suffix == "mixed":
        assert sorted(n.endswith("_alias") for n in names) == [False, True], names
    elif suffix == "nested":                            # inner and outer are aliases, the one that repeats b copies
        assert sorted(names) == ["concat2_alias", "concat3_alias", "concat4"], names
    else:
        assert names and all(n.endswith("_alias") == (suffix == "_alias") for n in names), names
    assert plan.n_launches == plan.n_kernels - sum(n.endswith("_alias") for n in names)
    ref = Graph(desc).run()
    got = plan.run()
    again = plan.run()
    plan.destroy()
    s.close()
    for a, b, c in zip(got, ref, again):
        assert norm_err(a, b) <= OP_TOL, case
        assert np.array_equal(a, c)
