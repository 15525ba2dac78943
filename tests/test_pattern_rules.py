"""Pattern rules and the pattern generator (paper Sec. 3): the oracle's generator
against a hand-derived list and against brute force, then the library's
generator against the oracle's (CPU only)."""
from itertools import combinations, permutations
import os

import pytest

import workloads as wl
from workloads import patterns as wp
from workloads.patterns import P, W
from oracle.graph import Graph
from oracle.match import enumerate_matches
from oracle import rules as orules
import paper_2111_00655_amd as clg

HERE = os.path.dirname(os.path.abspath(__file__))
CLS = wp.listing_rule_classes()


def parse(text):
    """'relu(add(*,*))' -> nested pattern tuple."""
    text = text.strip()
    if text == "*":
        return W
    op, rest = text.split("(", 1)
    assert rest.endswith(")")
    rest, args, depth, cur = rest[:-1], [], 0, ""
    for ch in rest:
        if ch == "," and depth == 0:
            args.append(cur)
            cur = ""
        else:
            depth += ch == "("
            depth -= ch == ")"
            cur += ch
    args.append(cur)
    return P(op, *[parse(a) for a in args])


def golden():
    with open(os.path.join(HERE, "golden", "tiny_cnn_generated_patterns.txt")) as f:
        return [parse(l) for l in f if l.strip() and not l.startswith("#")]


def test_oracle_generator_reproduces_the_hand_derived_list():
    g = Graph(wl.tiny_cnn(0))
    assert orules.generate(g, CLS, 9, True) == golden()


def test_limits_and_switches():
    g = Graph(wl.tiny_cnn(0))
    singles = orules.generate(g, CLS, 1, True)
    assert all(wp.pattern_ops(p) == 1 for p in singles)
    assert [p[0] for p in singles] == ["conv2d", "bias_add", "relu", "add", "dense"]
    two = orules.generate(g, CLS, 2, True)
    assert max(wp.pattern_ops(p) for p in two) == 2 and set(singles) <= set(two)
    no_grow = orules.generate(g, CLS, 9, False)
    # element-wise seeds stay alone, fusable seeds still grow
    assert P("relu", P("bias_add", W, W)) not in no_grow and P("relu", P("bias_add", P("conv2d", W, W), W)) in no_grow
    assert orules.generate(g, {}, 9, True) == []
    only_conv = orules.generate(g, {"conv2d": wp.RULE_FUSABLE}, 9, True)
    assert only_conv == [P("conv2d", W, W)]          # nothing element-wise to absorb


def chain_pattern(graph, chain):
    pat = None
    for k, v in enumerate(chain):
        nd = graph.nodes[v]
        pos = nd["inputs"].index(chain[k - 1]) if k else -1
        pat = (nd["kind"], tuple(pat if j == pos else W for j in range(len(nd["inputs"]))), ())
    return pat


def brute_force(graph, cls, max_ops, grow):
    """Every operator subset of at most max_ops nodes that, in some order, is a chain
    seed -> ... -> sink in which each node is the only consumer of the one before,
    uses it once, is element-wise, and the one before is no graph output."""
    found = set()
    ops = graph.op_ids
    for r in range(1, max_ops + 1):
        for sub in combinations(ops, r):
            for chain in permutations(sub):
                if cls.get(graph.nodes[chain[0]]["kind"], 0) == 0:
                    continue
                if r > 1 and cls[graph.nodes[chain[0]]["kind"]] == wp.RULE_ELEMWISE and not grow:
                    continue
                ok = True
                for a, b in zip(chain, chain[1:]):
                    nd = graph.nodes[b]
                    ok = ok and graph.consumers[a] == [b] and a not in graph.outputs and \
                        nd["inputs"].count(a) == 1 and cls.get(nd["kind"], 0) == wp.RULE_ELEMWISE
                if ok:
                    found.add(chain_pattern(graph, chain))
    return found


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("grow", [True, False])
def test_oracle_generator_equals_brute_force_on_random_dags(seed, grow):
    g = Graph(wl.random_dag(seed, 7))
    cls = {"conv2d": wp.RULE_FUSABLE, "bias_add": wp.RULE_ELEMWISE, "add": wp.RULE_ELEMWISE,
           "relu": wp.RULE_ELEMWISE, "tanh": wp.RULE_ELEMWISE, "mul_scalar": wp.RULE_ELEMWISE}
    got = orules.generate(g, cls, 4, grow)
    assert len(got) == len(set(got))
    assert set(got) == brute_force(g, cls, 4, grow)


@pytest.mark.parametrize("name", ["tiny_cnn", "dcgan_b1"])
def test_every_generated_pattern_matches_somewhere(name):
    g = Graph(wl.MODEL_BUILDERS[name](0))
    pats = orules.generate(g, CLS, 9, True)
    assert pats
    for p in pats:
        assert enumerate_matches(g, [("B", p)]), p


# ---- the library's generator ---------------------------------------------------------
def library_patterns(desc, variants=("igemm",)):
    explicit, rules = wp.rule_registry(variants)
    s = clg.Session(desc, explicit, device=None, rules=rules)
    full = s.full_registry()
    s.close()
    assert full[:len(explicit)] == explicit
    return full[len(explicit):], rules


@pytest.mark.parametrize("name", ["tiny_cnn", "resnet50", "resnext50", "bert_base", "dcgan_b1"])
def test_library_generator_equals_the_oracle(name):
    desc = wl.MODEL_BUILDERS[name](0)
    got, rules = library_patterns(desc)
    g = Graph(desc)
    want = []
    for backend, cls, max_ops, grow in rules:
        seeds = wp.FUSABLE_OPS if backend != "eltwise" else wp.ELEMWISE_OPS

        def seed_kind(p):
            while True:
                inner = [a for a in p[1] if a != W]
                if not inner:
                    return p[0]
                p = inner[0]

        # an MFMA backend runs contraction-seeded groups, the element-wise family the others
        want += [(backend, p) for p in orules.generate(g, cls, max_ops, grow) if seed_kind(p) in seeds]
    assert got == want


@pytest.mark.parametrize("seed", range(4))
def test_library_generator_equals_the_oracle_on_random_dags(seed):
    desc = wl.random_dag(seed, 12)
    cls = {"conv2d": wp.RULE_FUSABLE, "bias_add": wp.RULE_ELEMWISE, "add": wp.RULE_ELEMWISE,
           "relu": wp.RULE_ELEMWISE, "tanh": wp.RULE_ELEMWISE, "mul_scalar": wp.RULE_ELEMWISE}
    s = clg.Session(desc, [], device=None, rules=[("eltwise", {k: wp.RULE_ELEMWISE for k in cls if k != "conv2d"}, 5, True)])
    got = [p for _, p in s.full_registry()]
    s.close()
    want = orules.generate(Graph(desc), {k: wp.RULE_ELEMWISE for k in cls if k != "conv2d"}, 5, True)
    assert got == want


def test_generated_registry_matches_and_search_agree_with_the_oracle():
    """Matches and the placement found over a rule-generated registry are those of the oracle."""
    from oracle import search
    from workloads.costs import synthetic_costs
    desc = wl.tiny_cnn(0)
    explicit, rules = wp.rule_registry(("igemm", "igemm_s"))
    s = clg.Session(desc, explicit, device=None, rules=rules)
    reg = s.full_registry()
    g = Graph(desc)
    oms = enumerate_matches(g, reg)
    lms = s.match()
    assert [(m.pattern, m.first, m.sink) for m in lms] == [(m.pattern, m.first, m.sink) for m in oms]
    costs = synthetic_costs(len(oms), 3, [len(m.nodes) for m in oms], ties=True)
    assert s.search(costs, 0) == search.dp(g, reg, oms, costs, 0)
    s.close()


def test_rule_errors():
    from paper_2111_00655_amd import binding as B
    s = clg.Session(wl.tiny_cnn(0), [], device=None)
    be = B.clg_register_backend(s.ctx, "igemm")
    with pytest.raises(clg.ClgError) as e:
        B.clg_generate_patterns(s.ctx, s.graph, be, B.make_rule(CLS, 0, True))
    assert e.value.status == "INVALID_ARG"
    with pytest.raises(clg.ClgError) as e:
        B.clg_generate_patterns(s.ctx, s.graph, 99, B.make_rule(CLS, 4, True))
    assert e.value.status == "UNKNOWN_ID"
    bad = B.make_rule(CLS, 4, True)
    bad.op_class[0] = 7
    with pytest.raises(clg.ClgError) as e:
        B.clg_generate_patterns(s.ctx, s.graph, be, bad)
    assert e.value.status == "INVALID_ARG"
    n1 = B.clg_generate_patterns(s.ctx, s.graph, be, B.make_rule(CLS, 9, False))
    assert n1 > 0 and B.clg_generate_patterns(s.ctx, s.graph, be, B.make_rule(CLS, 9, False)) == 0   # nothing twice
    s.close()
