"""Seeded random-weight graphs with the shapes of the evaluated workloads
(paper Sec. 5.1 "Workload": BERT, DCGAN, ResNeXt50; plus ResNet-50 and a tiny
CNN whose placements can all be enumerated).  Trained weights are irrelevant
to latency and to parity, so every tensor is drawn from a seeded generator:
one child stream per tensor, in construction order.
"""
from __future__ import annotations

import numpy as np

from .graphdesc import GraphDesc


class _Rng:
    """One independent stream per drawn tensor: default_rng([seed, index])."""

    def __init__(self, seed: int):
        self.seed = int(seed)
        self.count = 0

    def _next(self):
        g = np.random.default_rng([self.seed, self.count])
        self.count += 1
        return g

    def normal(self, shape, std=1.0):
        return (self._next().standard_normal(shape) * std).astype(np.float32)

    def uniform(self, shape, lo, hi):
        return self._next().uniform(lo, hi, shape).astype(np.float32)

    def integers(self, shape, lo, hi):
        return self._next().integers(lo, hi, shape).astype(np.int32)


def _he(rng: _Rng, shape, fan_in):
    return rng.normal(shape, std=float(np.sqrt(2.0 / fan_in)))


def _conv(g, rng, x, cin, cout, k, stride, pad, groups=1, act="relu",
          residual=None, name=""):
    """conv2d -> bias_add -> [add residual] -> [relu] as primitive ops."""
    w = g.const(_he(rng, (cout, cin // groups, k, k), (cin // groups) * k * k),
                name + ".w")
    b = g.const(rng.uniform((cout,), -0.1, 0.1), name + ".b")
    y = g.op("conv2d", [x, w], name + ".conv", stride=(stride, stride),
             pad=(pad, pad), groups=groups)
    y = g.op("bias_add", [y, b], name + ".bias", axis=1)
    if residual is not None:
        y = g.op("add", [y, residual], name + ".add")
    if act == "relu":
        y = g.op("relu", [y], name + ".relu")
    return y


# --------------------------------------------------------------------------
# config 1: tiny CNN
# --------------------------------------------------------------------------
def tiny_cnn(seed: int = 0, image: int = 32) -> GraphDesc:
    g = GraphDesc("tiny_cnn")
    rw, rx = _Rng(seed), _Rng(seed + 1000003)
    x = g.input(rx.normal((1, 3, image, image)), "x")
    l1 = _conv(g, rw, x, 3, 16, 3, 1, 1, name="l1")
    l2 = _conv(g, rw, l1, 16, 32, 3, 1, 1, name="l2")
    l3 = _conv(g, rw, l2, 32, 32, 3, 1, 1, residual=l2, name="l3")
    p = g.op("global_avg_pool2d", [l3], "gap")
    w = g.const(_he(rw, (10, 32), 32), "fc.w")
    b = g.const(rw.uniform((10,), -0.1, 0.1), "fc.b")
    y = g.op("dense", [p, w], "fc")
    logits = g.op("bias_add", [y, b], "fc.bias", axis=-1)
    prob = g.op("softmax", [logits], "softmax")
    g.mark_output(logits)
    g.mark_output(prob)
    return g


# --------------------------------------------------------------------------
# configs 2 and 3: ResNet-50 v1.5 / ResNeXt-50 32x4d (BatchNorm folded)
# --------------------------------------------------------------------------
def resnet50(seed: int = 0, image: int = 224, width: int = 64,
             blocks=(3, 4, 6, 3), groups: int = 1, group_width_mult: int = 1,
             classes: int = 1000, name: str = "resnet50", batch: int = 1) -> GraphDesc:
    """v1.5: the stride-2 convolution of a down-sampling bottleneck is its
    3x3 one; the first block of every stage has a 1x1 projection shortcut.
    `group_width_mult` widens the inner (3x3) channels: 2 with groups=32
    gives the 32x4d ResNeXt layout (128/256/512/1024 inner channels)."""
    g = GraphDesc(name)
    rw, rx = _Rng(seed), _Rng(seed + 1000003)
    x = g.input(rx.normal((batch, 3, image, image)), "x")
    y = _conv(g, rw, x, 3, width, 7, 2, 3, name="stem")
    y = g.op("max_pool2d", [y], "pool", kernel=(3, 3), stride=(2, 2),
             pad=(1, 1))
    cin = width
    for s, nblk in enumerate(blocks):
        inner = width * (2 ** s) * group_width_mult
        cout = width * (2 ** s) * 4
        for b in range(nblk):
            stride = 2 if (b == 0 and s > 0) else 1
            nm = f"s{s}b{b}"
            if b == 0:
                sc = _conv(g, rw, y, cin, cout, 1, stride, 0, act=None,
                           name=nm + ".proj")
            else:
                sc = y
            t = _conv(g, rw, y, cin, inner, 1, 1, 0, name=nm + ".c1")
            t = _conv(g, rw, t, inner, inner, 3, stride, 1, groups=groups,
                      name=nm + ".c2")
            y = _conv(g, rw, t, inner, cout, 1, 1, 0, residual=sc,
                      name=nm + ".c3")
            cin = cout
    p = g.op("global_avg_pool2d", [y], "gap")
    w = g.const(_he(rw, (classes, cin), cin), "fc.w")
    b = g.const(rw.uniform((classes,), -0.1, 0.1), "fc.b")
    d = g.op("dense", [p, w], "fc")
    logits = g.op("bias_add", [d, b], "fc.bias", axis=-1)
    prob = g.op("softmax", [logits], "softmax")
    g.mark_output(logits)
    g.mark_output(prob)
    return g


def resnext50(seed: int = 0, image: int = 224, width: int = 64,
              blocks=(3, 4, 6, 3), groups: int = 32,
              classes: int = 1000, batch: int = 1) -> GraphDesc:
    return resnet50(seed, image, width, blocks, groups=groups,
                    group_width_mult=2, classes=classes, name="resnext50", batch=batch)


# --------------------------------------------------------------------------
# config 4: BERT-base encoder (post-layer-norm, erf GELU, no mask, no pooler)
# --------------------------------------------------------------------------
def bert_base(seed: int = 0, layers: int = 12, seq: int = 128,
              hidden: int = 768, heads: int = 12, ffn: int = 3072,
              vocab: int = 30522, max_pos: int = 512,
              eps: float = 1e-12) -> GraphDesc:
    g = GraphDesc("bert_base")
    rw, rx = _Rng(seed), _Rng(seed + 1000003)
    hd = hidden // heads
    std = 0.02

    def vec(shape, mean=0.0):
        return (rw.normal(shape, std) + np.float32(mean)).astype(np.float32)

    ids = g.input(rx.integers((seq,), 0, vocab), "ids")
    pos = g.const(np.arange(seq, dtype=np.int32), "pos_ids")
    tok = g.const(np.zeros(seq, dtype=np.int32), "type_ids")
    we = g.const(rw.normal((vocab, hidden), std), "emb.word")
    pe = g.const(rw.normal((max_pos, hidden), std), "emb.pos")
    te = g.const(rw.normal((2, hidden), std), "emb.type")
    e = g.op("take", [we, ids], "emb.take_word")
    ep = g.op("take", [pe, pos], "emb.take_pos")
    et = g.op("take", [te, tok], "emb.take_type")
    e = g.op("add", [e, ep], "emb.add_pos")
    e = g.op("add", [e, et], "emb.add_type")
    x = g.op("layer_norm", [e, g.const(vec((hidden,), 1.0), "emb.ln.g"),
                            g.const(vec((hidden,)), "emb.ln.b")],
             "emb.ln", eps=eps)

    def dense(inp, nin, nout, nm, act=None, residual=None):
        w = g.const(rw.normal((nout, nin), std), nm + ".w")
        b = g.const(vec((nout,)), nm + ".b")
        y = g.op("dense", [inp, w], nm)
        y = g.op("bias_add", [y, b], nm + ".bias", axis=-1)
        if act == "gelu":
            y = g.op("gelu", [y], nm + ".gelu")
        if residual is not None:
            y = g.op("add", [y, residual], nm + ".add")
        return y

    def split_heads(t, nm):
        t = g.op("reshape", [t], nm + ".rs", dims=(seq, heads, hd))
        return g.op("transpose", [t], nm + ".tr", dims=(1, 0, 2))

    for l in range(layers):
        nm = f"L{l}"
        q = split_heads(dense(x, hidden, hidden, nm + ".q"), nm + ".q")
        k = split_heads(dense(x, hidden, hidden, nm + ".k"), nm + ".k")
        v = split_heads(dense(x, hidden, hidden, nm + ".v"), nm + ".v")
        s = g.op("batch_matmul", [q, k], nm + ".qk", transpose_b=True)
        s = g.op("mul_scalar", [s], nm + ".scale",
                 scalar=float(1.0 / np.sqrt(hd)))
        p = g.op("softmax", [s], nm + ".softmax")
        c = g.op("batch_matmul", [p, v], nm + ".pv", transpose_b=False)
        c = g.op("transpose", [c], nm + ".ctx.tr", dims=(1, 0, 2))
        c = g.op("reshape", [c], nm + ".ctx.rs", dims=(seq, hidden))
        a = dense(c, hidden, hidden, nm + ".o", residual=x)
        x1 = g.op("layer_norm",
                  [a, g.const(vec((hidden,), 1.0), nm + ".ln1.g"),
                   g.const(vec((hidden,)), nm + ".ln1.b")],
                  nm + ".ln1", eps=eps)
        f = dense(x1, hidden, ffn, nm + ".ffn1", act="gelu")
        f = dense(f, ffn, hidden, nm + ".ffn2", residual=x1)
        x = g.op("layer_norm",
                 [f, g.const(vec((hidden,), 1.0), nm + ".ln2.g"),
                  g.const(vec((hidden,)), nm + ".ln2.b")],
                 nm + ".ln2", eps=eps)
    g.mark_output(x)
    return g


# --------------------------------------------------------------------------
# config 5: DCGAN generator (BatchNorm folded into the bias)
# --------------------------------------------------------------------------
def dcgan(seed: int = 0, batch: int = 1, latent: int = 100,
          base: int = 512, out_ch: int = 3) -> GraphDesc:
    g = GraphDesc(f"dcgan_b{batch}")
    rw, rx = _Rng(seed), _Rng(seed + 1000003)
    std = 0.02
    z = g.input(rx.normal((batch, latent)), "z")
    w = g.const(rw.normal((base * 16, latent), std), "fc.w")
    b = g.const(rw.uniform((base * 16,), -0.1, 0.1), "fc.b")
    y = g.op("dense", [z, w], "fc")
    y = g.op("bias_add", [y, b], "fc.bias", axis=-1)
    y = g.op("relu", [y], "fc.relu")
    y = g.op("reshape", [y], "fc.rs", dims=(batch, base, 4, 4))
    chans = [base, base // 2, base // 4, base // 8, out_ch]
    for i in range(4):
        cin, cout = chans[i], chans[i + 1]
        nm = f"up{i}"
        w = g.const(rw.normal((cin, cout, 4, 4), std), nm + ".w")
        b = g.const(rw.uniform((cout,), -0.1, 0.1), nm + ".b")
        y = g.op("conv2d_transpose", [y, w], nm, stride=(2, 2), pad=(1, 1))
        y = g.op("bias_add", [y, b], nm + ".bias", axis=1)
        y = g.op("relu" if i < 3 else "tanh", [y],
                 nm + (".relu" if i < 3 else ".tanh"))
    g.mark_output(y)
    return g


# --------------------------------------------------------------------------
# random small DAGs for the placement-search tests (diamonds, multi-input)
# --------------------------------------------------------------------------
def random_dag(seed: int, n_ops: int = 10, ch: int = 4, image: int = 6
               ) -> GraphDesc:
    """A random DAG of conv / bias / add / relu / tanh / mul_scalar ops over
    tensors of one shape [1,ch,image,image], so that any earlier value can be
    an operand of any later op.  Ops come in short templates (conv-bias-relu,
    conv-bias-add-relu, add-relu, ...) that start from a recent or an older
    value, which gives fusable chains, parallel branches, diamonds and values
    with several consumers.  Every value without a consumer becomes a graph
    output."""
    g = GraphDesc(f"random_dag_{seed}")
    rw = _Rng(seed)
    pick = np.random.default_rng([seed, 999983])
    vals = [g.input(rw.normal((1, ch, image, image)), "x0")]
    if pick.random() < 0.4:
        vals.append(g.input(rw.normal((1, ch, image, image)), "x1"))
    used = set()
    templates = [("conv2d", "bias_add", "relu"),
                 ("conv2d", "bias_add", "add", "relu"),
                 ("conv2d", "relu"), ("conv2d", "add", "relu"),
                 ("add", "relu"), ("bias_add", "relu"), ("relu",), ("tanh",),
                 ("mul_scalar",), ("add",), ("add", "tanh"),
                 ("tanh", "mul_scalar"), ("relu", "add"), ("mul_scalar", "add")]
    n = 0
    while n < n_ops:
        tpl = templates[int(pick.integers(0, len(templates)))]
        # start from the newest value (chain) or from any value (branch)
        cur = vals[-1] if pick.random() < 0.5 else vals[int(pick.integers(0, len(vals)))]
        for kind in tpl:
            if n >= n_ops:
                break
            if kind == "conv2d":
                w = g.const(_he(rw, (ch, ch, 3, 3), ch * 9), f"w{n}")
                v = g.op("conv2d", [cur, w], f"conv{n}", stride=(1, 1),
                         pad=(1, 1), groups=1)
                used.add(cur)
            elif kind == "bias_add":
                b = g.const(rw.uniform((ch,), -0.1, 0.1), f"b{n}")
                v = g.op("bias_add", [cur, b], f"bias{n}", axis=1)
                used.add(cur)
            elif kind == "add":
                other = vals[int(pick.integers(0, len(vals)))]
                ins = [cur, other] if pick.random() < 0.7 else [other, cur]
                v = g.op("add", ins, f"add{n}")
                used.update(ins)
            elif kind == "mul_scalar":
                v = g.op("mul_scalar", [cur], f"mul{n}", scalar=0.5)
                used.add(cur)
            else:
                v = g.op(kind, [cur], f"{kind}{n}")
                used.add(cur)
            vals.append(v)
            cur = v
            n += 1
    for v in vals:
        if v not in used and g.nodes[v]["kind"] != "input":
            g.mark_output(v)
    return g


# --------------------------------------------------------------------------
# 3D-ResNet50 (one of the paper's Sec. 5.1 workloads): ResNet-50 with every
# convolution and pooling extended to three dimensions (Hara et al. 2018)
# --------------------------------------------------------------------------
def _conv3(g, rng, x, cin, cout, k, stride, pad, act="relu", residual=None, name=""):
    """conv3d -> bias_add -> [add residual] -> [relu]; k, stride, pad: (d, h, w)."""
    fan_in = cin * k[0] * k[1] * k[2]
    w = g.const(_he(rng, (cout, cin) + tuple(k), fan_in), name + ".w")
    b = g.const(rng.uniform((cout,), -0.1, 0.1), name + ".b")
    y = g.op("conv3d", [x, w], name + ".conv", stride=tuple(stride), pad=tuple(pad))
    y = g.op("bias_add", [y, b], name + ".bias", axis=1)
    if residual is not None:
        y = g.op("add", [y, residual], name + ".add")
    if act == "relu":
        y = g.op("relu", [y], name + ".relu")
    return y


def resnet3d_50(seed: int = 0, frames: int = 16, image: int = 112, width: int = 64,
                blocks=(3, 4, 6, 3), classes: int = 400, batch: int = 1) -> GraphDesc:
    """Clip of `frames` x image x image; 7x7x7 stem with stride (1, 2, 2), 3x3x3
    max pool of stride 2, bottlenecks 1x1x1 -> 3x3x3 -> 1x1x1 with the stride
    (2, 2, 2) of a down-sampling block in its 3x3x3 convolution and a 1x1x1
    projection shortcut in the first block of every stage, global average pool,
    classifier (400 action classes).  BatchNorm folded."""
    g = GraphDesc("resnet3d_50")
    rw, rx = _Rng(seed), _Rng(seed + 1000003)
    x = g.input(rx.normal((batch, 3, frames, image, image)), "x")
    y = _conv3(g, rw, x, 3, width, (7, 7, 7), (1, 2, 2), (3, 3, 3), name="stem")
    y = g.op("max_pool3d", [y], "pool", kernel=(3, 3, 3), stride=(2, 2, 2), pad=(1, 1, 1))
    cin = width
    for s, nblk in enumerate(blocks):
        inner = width * (2 ** s)
        cout = inner * 4
        for b in range(nblk):
            st = (2, 2, 2) if (b == 0 and s > 0) else (1, 1, 1)
            nm = f"s{s}b{b}"
            sc = _conv3(g, rw, y, cin, cout, (1, 1, 1), st, (0, 0, 0), act=None, name=nm + ".proj") if b == 0 else y
            t = _conv3(g, rw, y, cin, inner, (1, 1, 1), (1, 1, 1), (0, 0, 0), name=nm + ".c1")
            t = _conv3(g, rw, t, inner, inner, (3, 3, 3), st, (1, 1, 1), name=nm + ".c2")
            y = _conv3(g, rw, t, inner, cout, (1, 1, 1), (1, 1, 1), (0, 0, 0), residual=sc, name=nm + ".c3")
            cin = cout
    p = g.op("global_avg_pool3d", [y], "gap")
    w = g.const(_he(rw, (classes, cin), cin), "fc.w")
    b = g.const(rw.uniform((classes,), -0.1, 0.1), "fc.b")
    d = g.op("dense", [p, w], "fc")
    logits = g.op("bias_add", [d, b], "fc.bias", axis=-1)
    prob = g.op("softmax", [logits], "softmax")
    g.mark_output(logits)
    g.mark_output(prob)
    return g


# --------------------------------------------------------------------------
# NasNet-A (one of the paper's Sec. 5.1 workloads): cells of separable
# convolutions, poolings and identities joined by adds and a channel concat
# --------------------------------------------------------------------------
def nasnet_a(seed: int = 0, image: int = 224, stem: int = 32, filters: int = 44,
             cells: int = 4, classes: int = 1000, batch: int = 1) -> GraphDesc:
    """The mobile layout (4 normal cells per stage, 44 filters, 1056 features)
    by default.  Cell wiring after the published NASNet-A diagram (Zoph et al.
    2018): five two-branch blocks per cell, unused states concatenated.
    BatchNorm is folded into the preceding 1x1 convolution as a bias.  A
    separable convolution is relu -> depthwise k x k -> 1x1 -> bias, applied
    twice (the stride sits in the first depthwise).  Simplifications of this
    stand-in: 'same' padding everywhere (224 -> 112 -> 56 -> 28 -> 14 -> 7), and
    a previous state of twice the resolution is brought down by relu -> 1x1
    convolution of stride 2 instead of the two-path factorised reduction."""
    g = GraphDesc("nasnet_a")
    rw, rx = _Rng(seed), _Rng(seed + 1000003)
    x = g.input(rx.normal((batch, 3, image, image)), "x")

    def pw(t, cin, cout, stride, nm):                       # relu -> 1x1 -> bias
        t = g.op("relu", [t], nm + ".relu")
        return _conv(g, rw, t, cin, cout, 1, stride, 0, act=None, name=nm)

    def sep(t, c, k, stride, nm):
        for i, s in enumerate((stride, 1)):
            t = g.op("relu", [t], f"{nm}.{i}.relu")
            w = g.const(_he(rw, (c, 1, k, k), k * k), f"{nm}.{i}.dw.w")
            t = g.op("conv2d", [t, w], f"{nm}.{i}.dw", stride=(s, s), pad=(k // 2, k // 2), groups=c)
            t = _conv(g, rw, t, c, c, 1, 1, 0, act=None, name=f"{nm}.{i}.pw")
        return t

    def pool(kind, t, stride, nm):
        return g.op(kind, [t], nm, kernel=(3, 3), stride=(stride, stride), pad=(1, 1))

    def add(a, b, nm):
        return g.op("add", [a, b], nm)

    def adjust(h, hp, shape_h, shape_p, f, nm):
        """Both states to `f` channels at the current state's resolution."""
        (ch, sh), (cp, sp) = shape_h, shape_p
        hp = pw(hp, cp, f, 1 if sp == sh else 2, nm + ".prev")
        h = pw(h, ch, f, 1, nm + ".cur")
        return h, hp

    def normal(h, hp, shape_h, shape_p, f, nm):
        h, hp = adjust(h, hp, shape_h, shape_p, f, nm)
        y1 = add(sep(h, f, 3, 1, nm + ".b1l"), h, nm + ".b1")
        y2 = add(sep(hp, f, 3, 1, nm + ".b2l"), sep(h, f, 5, 1, nm + ".b2r"), nm + ".b2")
        y3 = add(pool("avg_pool2d", h, 1, nm + ".b3l"), hp, nm + ".b3")
        y4 = add(pool("avg_pool2d", hp, 1, nm + ".b4l"), pool("avg_pool2d", hp, 1, nm + ".b4r"), nm + ".b4")
        y5 = add(sep(hp, f, 5, 1, nm + ".b5l"), sep(hp, f, 3, 1, nm + ".b5r"), nm + ".b5")
        out = g.op("concat", [hp, y1, y2, y3, y4, y5], nm + ".cat", axis=1)
        return out, (6 * f, shape_h[1])

    def reduction(h, hp, shape_h, shape_p, f, nm):
        h, hp = adjust(h, hp, shape_h, shape_p, f, nm)
        y1 = add(sep(hp, f, 7, 2, nm + ".b1l"), sep(h, f, 5, 2, nm + ".b1r"), nm + ".b1")
        y2 = add(pool("max_pool2d", h, 2, nm + ".b2l"), sep(hp, f, 7, 2, nm + ".b2r"), nm + ".b2")
        y3 = add(pool("avg_pool2d", h, 2, nm + ".b3l"), sep(hp, f, 5, 2, nm + ".b3r"), nm + ".b3")
        y4 = add(pool("max_pool2d", h, 2, nm + ".b4l"), sep(y1, f, 3, 1, nm + ".b4r"), nm + ".b4")
        y5 = add(pool("avg_pool2d", y1, 1, nm + ".b5l"), y2, nm + ".b5")
        out = g.op("concat", [y2, y3, y4, y5], nm + ".cat", axis=1)
        return out, (4 * f, (shape_h[1] + 1) // 2)

    size = (image + 1) // 2
    h = _conv(g, rw, x, 3, stem, 3, 2, 1, act=None, name="stem")
    states = [(h, (stem, size)), (h, (stem, size))]          # (previous, current)

    def step(cell, f, nm):
        (hp, sp), (hc, sc) = states
        out, so = cell(hc, hp, sc, sp, f, nm)
        states[0], states[1] = (hc, sc), (out, so)

    step(reduction, filters // 4, "stem1")
    step(reduction, filters // 2, "stem2")
    for stage in range(3):
        f = filters * (2 ** stage)
        if stage:
            step(reduction, f, f"r{stage}")
        for c in range(cells):
            step(normal, f, f"s{stage}c{c}")
    y, (cin, _) = states[1]
    y = g.op("relu", [y], "head.relu")
    p = g.op("global_avg_pool2d", [y], "gap")
    w = g.const(_he(rw, (classes, cin), cin), "fc.w")
    b = g.const(rw.uniform((classes,), -0.1, 0.1), "fc.b")
    d = g.op("dense", [p, w], "fc")
    logits = g.op("bias_add", [d, b], "fc.bias", axis=-1)
    prob = g.op("softmax", [logits], "softmax")
    g.mark_output(logits)
    g.mark_output(prob)
    return g


MODEL_BUILDERS = {
    "tiny_cnn": tiny_cnn,
    "resnet50": resnet50,
    "resnext50": resnext50,
    "bert_base": bert_base,
    "dcgan_b1": lambda seed=0: dcgan(seed, batch=1),
    "dcgan_b64": lambda seed=0: dcgan(seed, batch=64),
    "nasnet_a": nasnet_a,
    "resnet3d_50": resnet3d_50,
}
