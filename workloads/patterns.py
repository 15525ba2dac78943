"""Backend-pattern registries B = [(pattern p, backend d), ...] as plain data
(paper Sec. 3 explicit pattern specification and Sec. 4.1: b = (p, d)).

A pattern is a sink-rooted tree written the way the paper's pattern language
writes it: P("relu", P("add", P("conv2d", W, W, groups=(1, 1)), W)) is
relu(add(conv2d(*, *), *)) with the constraint 1 <= groups <= 1 on the
convolution.  W is the wildcard: it matches any value and is not part of the
matched subgraph.  Registration order is significant (ties are broken by it).

A "backend" here is one of the kernel families of the GPU library; the oracle
only uses the names as identifiers.
"""
from __future__ import annotations

W = "*"

# igemm variants whose conv2d patterns carry no groups = 1 constraint
GROUPED_CONV_BACKENDS = ("igemm_r32", "igemm_r16", "igemm_r32_w4", "igemm_r32_w8", "igemm_r16_w4", "igemm_r16_w8",
                         "igemm_r16_sk", "igemm_r16_sk_w4", "igemm_r32_sk")

# igemm variants that exist for dense layers only (registering their convolution patterns would only
# repeat what the plain 16x16 variants do)
DENSE_ONLY_BACKENDS = ("igemm_r16x2_w4", "igemm_r16x2_w8")

# attribute names a constraint may refer to, in the order of the C enum
ATTR_NAMES = ("groups", "kernel_h", "kernel_w", "stride_h", "stride_w",
              "pad_h", "pad_w", "transpose_b", "axis")


def P(op: str, *args, **constraints):
    for k, v in constraints.items():
        assert k in ATTR_NAMES, k
        assert len(v) == 2
    return (op, tuple(args), tuple(sorted((k, (int(v[0]), int(v[1])))
                                          for k, v in constraints.items())))


def pattern_ops(p) -> int:
    """Number of operator (non-wildcard) nodes in a pattern."""
    if p == W:
        return 0
    return 1 + sum(pattern_ops(a) for a in p[1])


def _tails(anchor, tails):
    """anchor followed by each listed chain of unary/binary elementwise ops;
    a binary op takes the chain as its first operand and a wildcard second."""
    out = []
    for chain in tails:
        p = anchor
        for op in chain:
            if op in ("bias_add", "add"):
                p = P(op, p, W)
            else:
                p = P(op, p)
        out.append(p)
    return out


def default_registry(variants=("igemm",), sepconv=False, attention=False):
    """The registry the benchmarks and the GPU parity tests use.  `variants`
    lists the MFMA implicit-GEMM kernel variants to register as separate
    backends (same patterns each), so that the search can pick a tile
    configuration per layer.  `sepconv` adds the one-kernel separable
    convolution family (NasNet-A's building block), `attention` the one-kernel
    scaled-dot-product attention."""
    reg = []

    def add(backend, pats):
        reg.extend((backend, p) for p in pats)

    # --- glue: every primitive elementwise / layout op alone, plus short fusions
    ew_single = [P("bias_add", W, W), P("add", W, W), P("mul_scalar", W),
                 P("relu", W), P("gelu", W), P("tanh", W), P("take", W, W),
                 P("reshape", W), P("transpose", W)]
    ew_fused = [P("relu", P("add", W, W)),
                P("relu", P("bias_add", W, W)),
                P("gelu", P("bias_add", W, W)),
                P("tanh", P("bias_add", W, W)),
                P("add", P("bias_add", W, W), W),
                P("relu", P("add", P("bias_add", W, W), W)),
                P("add", P("add", P("take", W, W), W), W),
                P("transpose", P("reshape", W)),
                P("reshape", P("transpose", W))]
    add("eltwise", ew_single + ew_fused)
    add("eltwise", [P("concat", *([W] * n)) for n in range(2, 9)])

    # --- row-wise reductions
    add("rowwise", [P("softmax", W), P("layer_norm", W, W, W),
                    P("softmax", P("mul_scalar", W)),
                    P("layer_norm", P("add", W, W), W, W),
                    P("layer_norm", P("add", P("bias_add", W, W), W), W, W),
                    # an embedding: three table rows gathered, summed and normalised (the one tree-shaped kind)
                    P("layer_norm", P("add", P("add", P("take", W, W), P("take", W, W)), P("take", W, W)), W, W)])

    # --- direct (non-GEMM) spatial kernels: any conv incl. grouped, pools
    conv_any = P("conv2d", W, W)
    add("direct", _tails(conv_any, [(), ("bias_add",), ("bias_add", "relu"),
                                    ("bias_add", "add"),
                                    ("bias_add", "add", "relu")]))
    add("direct", _tails(P("conv2d_transpose", W, W), [(), ("bias_add",), ("bias_add", "relu"), ("bias_add", "tanh")]))
    add("direct", [P("max_pool2d", W), P("global_avg_pool2d", W)])
    add("direct", [P("avg_pool2d", W), P("add", P("avg_pool2d", W), W), P("add", P("max_pool2d", W), W)])
    add("direct", [P("max_pool3d", W), P("global_avg_pool3d", W)])

    # --- separable convolution in one kernel: [relu] depthwise 1x1 tail, or relu 1x1 tail
    sep_anchors = [P("conv2d", P("conv2d", P("relu", W), W), W), P("conv2d", P("conv2d", W, W), W),
                   P("conv2d", P("relu", W), W)]
    for anchor in sep_anchors if sepconv else ():
        add("sepconv", _tails(anchor, [(), ("bias_add",), ("bias_add", "relu"), ("bias_add", "add"),
                                       ("bias_add", "add", "relu")]))

    # --- attention in one kernel: q k^T, scale, softmax, p v, heads merged on store
    if attention:
        qk = P("batch_matmul", W, W)
        for scores in (P("mul_scalar", qk), qk):
            pv = P("batch_matmul", P("softmax", scores), W)
            add("attention", [P("reshape", P("transpose", pv)), pv])

    # --- MFMA implicit GEMM / GEMM variants
    for be in variants:
        dense = P("dense", W, W)
        if be in DENSE_ONLY_BACKENDS:
            add(be, _tails(dense, [(), ("bias_add",), ("bias_add", "relu"), ("bias_add", "gelu"), ("bias_add", "add")]))
            add(be, [P("transpose", P("reshape", P("bias_add", dense, W)))])
            continue
        # the register-fed kernels also run grouped convolutions
        conv = P("conv2d", W, W) if be in GROUPED_CONV_BACKENDS else P("conv2d", W, W, groups=(1, 1))
        add(be, _tails(conv, [(), ("bias_add",), ("bias_add", "relu"),
                              ("bias_add", "add"),
                              ("bias_add", "add", "relu")]))
        add(be, _tails(dense, [(), ("bias_add",), ("bias_add", "relu"),
                               ("bias_add", "gelu"), ("bias_add", "add"),
                               ("bias_add", "relu", "reshape")]))
        add(be, [P("batch_matmul", W, W),
                 P("mul_scalar", P("batch_matmul", W, W))])
        # results stored permuted: projection split into heads, heads merged
        add(be, [P("transpose", P("reshape", P("bias_add", dense, W))),
                 P("reshape", P("transpose", P("batch_matmul", W, W)))])
        if be in GROUPED_CONV_BACKENDS:      # the register-fed kernels also run 3-D convolutions
            add(be, _tails(P("conv3d", W, W), [(), ("bias_add",), ("bias_add", "relu"), ("bias_add", "add"),
                                               ("bias_add", "add", "relu")]))
        convt = P("conv2d_transpose", W, W)
        add(be, _tails(convt, [(), ("bias_add",), ("bias_add", "relu"),
                               ("bias_add", "tanh")]))
    return reg


def small_registry():
    """Two abstract backends over conv / bias / add / relu / tanh / mul_scalar
    for the CPU-only placement-search tests (random DAGs)."""
    reg = []
    singles = [P("conv2d", W, W), P("bias_add", W, W), P("add", W, W),
               P("relu", W), P("tanh", W), P("mul_scalar", W)]
    reg += [("A", p) for p in singles]
    conv = P("conv2d", W, W)
    reg += [("B", p) for p in _tails(conv, [(), ("bias_add",),
                                            ("bias_add", "relu"),
                                            ("bias_add", "add", "relu"),
                                            ("relu",), ("add", "relu")])]
    reg += [("B", P("relu", P("add", W, W))),
            ("B", P("relu", P("bias_add", W, W))),
            ("B", P("add", P("relu", W), P("relu", W))),
            ("A", P("tanh", P("add", W, W))),
            ("A", P("mul_scalar", P("tanh", W))),
            ("A", P("add", P("mul_scalar", W), W))]
    return reg


# ---- pattern rules (data only) ---------------------------------------------------
RULE_NONE, RULE_FUSABLE, RULE_ELEMWISE = 0, 1, 2
FUSABLE_OPS = ("conv2d", "conv2d_transpose", "dense", "batch_matmul", "conv3d")
ELEMWISE_OPS = ("bias_add", "add", "mul_scalar", "relu", "gelu", "tanh")


def listing_rule_classes():
    """Operator classes of the rule sketched in the paper's registration
    listing: convolutions and matrix products are fusable, the pointwise
    operators element-wise, everything else is not run."""
    cls = {k: RULE_FUSABLE for k in FUSABLE_OPS}
    cls.update({k: RULE_ELEMWISE for k in ELEMWISE_OPS})
    return cls


def rule_registry(variants=("igemm",)):
    """A registry described mostly by rules: (explicit pairs, rules).  Each MFMA
    variant gets the fusable-seeded rule (a contraction plus its element-wise
    tail, up to nine operators), the element-wise kernel family the
    element-wise-seeded one; what no rule covers (row-wise reductions, pools,
    gather, layout copies) is listed explicitly."""
    fus = {k: RULE_FUSABLE for k in FUSABLE_OPS}
    fus.update({k: RULE_ELEMWISE for k in ELEMWISE_OPS})
    elt = {k: RULE_ELEMWISE for k in ELEMWISE_OPS}
    # an MFMA backend runs groups seeded by a contraction only (the generator drops what its kernels do not
    # run); the element-wise family gets the element-wise operators as seeds of growing groups
    rules = [(be, dict(fus), 9, False) for be in variants]
    rules.append(("eltwise", elt, 8, True))
    explicit = [("eltwise", p) for p in (P("take", W, W), P("reshape", W), P("transpose", W),
                                         P("add", P("add", P("take", W, W), W), W),
                                         P("transpose", P("reshape", W)), P("reshape", P("transpose", W)))]
    explicit += [("rowwise", p) for p in (P("softmax", W), P("layer_norm", W, W, W),
                                          P("softmax", P("mul_scalar", W)),
                                          P("layer_norm", P("add", W, W), W, W))]
    explicit += [("direct", p) for p in (P("max_pool2d", W), P("global_avg_pool2d", W))]
    return explicit, rules
